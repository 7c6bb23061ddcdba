#!/usr/bin/env python3
"""Benchmark of the SR-AdamW update path on one MI355X.

A step is one pass of the whole hot path over a resident synthetic parameter set: (global
gradient norm when the config clips) + the fused SR-AdamW update of every tensor.  Default
workload: the 6.7B flat-buffer configuration (BF16 p/g/m/v, SR on all three write-backs,
moments warm-started by 100 seeded steps).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1..5] [--warm-steps N]
                  [--cpu-seconds S] [--no-cpu-baseline] [--mode M] [--graph]
  python bench.py --op cast|cast_e4m3|cast_e5m2|accumulate|accumulate_norm [--config N]   (the other two entry points,
                  on an array of the config's size; their own metric, not the headline one)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published peak


# step variants: name -> (flags by name, FP32 moments, aux dtype, algorithmic bytes per element)
#   sr            BF16 p,g,m,v read + p,m,v written                        8 + 6  = 14
#   rne_moments   same traffic, moments rounded to nearest (the paper's own setting)
#   nearest       same traffic, every write-back to nearest (the "BF16" strategy of Section 5.1)
#   fp32_moments  2+2+4+4 read, 2+4+4 written                              12 + 10 = 22
#   kahan         BF16 p,g,m,v,c read + p,m,v,c written                    10 + 8  = 18
#   master        x32,g,m32,v32 read + x32,p16,m32,v32 written (O2 style)  14 + 14 = 28
#   fp8_moments   2+2+1+1 read, 2+1+1 written (extension: E4M3 m, E5M2 v)   6 + 4  = 10
#   fp8_params    1+2+2+2 read, 1+2+2 written (extension: E4M3 p)           7 + 5  = 12
#   fp8_all       1+2+1+1 read, 1+1+1 written (extension: both)             5 + 3  = 8
MODES = {
    "sr": ((), False, None, 14),
    "rne_moments": (("SR_FLAG_RNE_MOMENTS",), False, None, 14),
    "nearest": (("SR_FLAG_RNE_PARAMS", "SR_FLAG_RNE_MOMENTS"), False, None, 14),
    "fp32_moments": (("SR_FLAG_FP32_MOMENTS",), True, None, 22),
    "kahan": (("SR_FLAG_KAHAN",), False, "bf16", 18),
    "master": (("SR_FLAG_MASTER_FP32", "SR_FLAG_FP32_MOMENTS"), True, "f32", 28),
    "fp8_moments": (("SR_FLAG_FP8_MOMENTS",), False, None, 10),
    # extension: the parameter as E4M3 codes too (1+2+2+2 read, 1+2+2 written; with 8-bit moments 1+2+1+1 and 1+1+1)
    "fp8_params": (("SR_FLAG_FP8_PARAMS",), False, None, 12),
    "fp8_all": (("SR_FLAG_FP8_PARAMS", "SR_FLAG_FP8_MOMENTS"), False, None, 8),
}


def fp8_scale_exponents(cfg):
    """Power-of-two scales of the 8-bit moments for a workload: eight gradient standard deviations
    (outliers included) map to the top of E4M3 for m, their square to the top of E5M2 for v."""
    import math
    g = 8.0 * max(cfg.grad_std, cfg.outlier_std if cfg.outlier_frac > 0 else 0.0)
    return int(math.floor(math.log2(448.0 / g))), int(math.floor(math.log2(57344.0 / (g * g))))


def calibrate_copy(torch, dev):
    """One device copy of exactly 2^30 bytes (2^30 read, 2^30 written), the last dispatch of the run:
    a dispatch of known traffic that fixes the unit of the FETCH_SIZE / WRITE_SIZE counters."""
    src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)
    torch.cuda.synchronize()


def kernel_source_sha16() -> str:
    """Hash of the kernel and launcher sources: ties a counter summary under profiles/ to the code
    it was measured on."""
    import hashlib
    h = hashlib.sha256()
    for name in ("sr_device.h", "sr_host.h", "sr_kernels.h", "sradamw.hip"):
        h.update(open(os.path.join(ROOT, "paper_2502_20566_amd", "csrc", name), "rb").read())
    return h.hexdigest()[:16]


def profile_traffic(tag: str):
    """(HBM bytes per step, where from) out of profiles/hbm_traffic_<tag>.txt -- a rocprofv3 counter
    summary -- while it was made from the kernel sources this library is built from (the summary
    records their hash); (None, why) otherwise."""
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{tag}.txt")
    if not os.path.exists(tpath):
        return None, None
    fields = {}
    for line in open(tpath):
        if "=" in line and not line.startswith((" ", "#")):
            k, v = line.split("=", 1)
            fields[k.strip()] = v.strip()
    rel = os.path.relpath(tpath, ROOT)
    if fields.get("kernel_source_sha16") != kernel_source_sha16() or "hbm_bytes_per_step" not in fields:
        return None, f"{rel} is stale (made from other kernel sources)"
    return int(fields["hbm_bytes_per_step"]), rel


def algorithmic_bytes_per_element(mode, clip) -> int:
    # the norm pass of a clipping config reads the gradients once more
    return MODES[mode][3] + (2 if clip is not None else 0)


def cpu_baseline(W, B, torch, cfg, state, step_no, seed, seconds, flags, fp8_exps=None, norm=None, p_exp=None):
    """Time the CPU oracle (as it stands) on a bounded window of the same workload and check the
    GPU against it on that window.  `state` holds flat device tensors p, g, m, v, aux (first
    tensor; aux may be None).  `flags`: the step's flag bits (same values on both sides).
    `norm`: the gradient norm the device computed for this step when the config clips (the oracle
    takes the same binary32 value, so the clip scale is the same on both sides), else None."""
    import numpy as np
    from oracle import ref
    p, g, m, v, aux = state
    threads = min(ref.max_threads(), os.cpu_count() or 1)
    max_norm = cfg.clip if norm is not None else 0.0

    def window(lo, n):
        def cp(t):
            s = t[lo:lo + n]
            return W.bf16_to_u16_numpy(s) if s.dtype == torch.bfloat16 else s.cpu().numpy().copy()
        d = dict(p=cp(p), g=cp(g), m=cp(m), v=cp(v), tensor_id=0, elem_offset=lo)
        if fp8_exps is not None:
            d["m_exp"], d["v_exp"] = fp8_exps
        if p_exp is not None:
            d["p_exp"] = p_exp
        if aux is not None:
            d["aux"] = cp(aux)
        return d

    # calibrate on 2^21 elements, then size the sample for about `seconds` of CPU work
    n0 = min(1 << 21, p.numel())
    w0 = window(0, n0)
    # the workload's share of updates below one BF16 spacing of the parameter (what nearest rounding
    # would mostly lose; Section 2.2), from the oracle's unrounded result on this window
    sub_ulp = None
    if aux is None and p_exp is None:
        sc = ref.adamw_scalars(step=step_no, norm=norm, max_norm=max_norm, **cfg.hyper)
        if fp8_exps is not None:
            y, _, _ = ref.adamw_unrounded_fp8m(w0["p"], w0["g"], w0["m"], w0["v"], sc, *fp8_exps)
        else:
            y, _, _ = ref.adamw_unrounded(w0["p"], w0["g"], w0["m"], w0["v"], sc, flags)
        p32 = ref.bf16_bits_to_f32(w0["p"])
        sub_ulp = float(np.mean(np.abs(y.astype(np.float64) - p32) < np.spacing(np.abs(p32)).astype(np.float64) * 65536.0))
    t0 = time.perf_counter()
    ref.sr_adamw_step([w0], cfg.hyper, step_no, seed, flags, norm=norm, max_norm=max_norm, nthreads=1)
    rate1 = n0 / (time.perf_counter() - t0)
    w0 = window(0, n0)
    t0 = time.perf_counter()
    ref.sr_adamw_step([w0], cfg.hyper, step_no, seed, flags, norm=norm, max_norm=max_norm, nthreads=threads)
    rate0 = n0 / (time.perf_counter() - t0)
    n = int(min(p.numel(), max(n0, rate0 * seconds), 3 << 30))
    n -= n % 8
    lo = ((p.numel() - n) // 2) & ~7                      # a window from the middle of the buffer
    w = window(lo, n)
    t0 = time.perf_counter()
    ref.sr_adamw_step([w], cfg.hyper, step_no, seed, flags, norm=norm, max_norm=max_norm, nthreads=threads)
    dt = time.perf_counter() - t0
    return dict(value=n / dt, unit="params/s", cores=threads, kind="oracle", one_thread_value=rate1,
                sub_ulp_update_fraction=sub_ulp,
                sample=f"{n} contiguous elements from the middle of the buffer, one step "
                       f"(step {step_no}), {dt:.1f} s"), (lo, n, w)


def time_launches(torch, np, fn, warmup, steps):
    """HIP events on the launch stream around each of `steps` calls of fn, after `warmup` calls."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0 = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    e1 = [torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    t0 = time.perf_counter()
    for i in range(steps):
        e0[i].record()
        fn()
        e1[i].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return wall, [a.elapsed_time(b) for a, b in zip(e0, e1)]


def run_aux_op(args, torch, np, B, W, cfg):
    """The standalone SR cast (Eq. 2 on a binary32 array) or the BF16 gradient accumulation with SR,
    on one flat array of the config's element count.  Same JSON shape as the step, own metric."""
    from oracle import ref
    dev = "cuda:0"
    n = sum(W.numel_of(shape) for _, shape, _ in cfg.shapes)
    flat = [("flat", (n,), "weight")]
    seed, tid = cfg.seed, 3
    threads = min(ref.max_threads(), os.cpu_count() or 1)
    n_cpu = min(n, 1 << 26) & ~7 or n
    lo = ((n - n_cpu) // 2) & ~7
    def placed_arrays(roles, run):
        """The op's arrays chosen among spare allocations (as for the step), or None."""
        if args.placement == "plain" or n < (1 << 28):
            return None, {"policy": "as the allocator returns them"}
        from paper_2502_20566_amd.placement import place_state_buffers

        def time_layout(a, reps=3):
            run(a)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                run(a)
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps
        return place_state_buffers(roles, dev, time_layout, n_layouts=12, slowest=args.placement == "slowest")

    if args.op.startswith("cast"):
        out_dtype = torch.bfloat16 if args.op == "cast" else torch.uint8
        fmt = B.SR_FP8_E5M2 if args.op == "cast_e5m2" else B.SR_FP8_E4M3
        run = ((lambda a: B.sr_cast_f32_bf16(a["src"], a["dst"], seed, 7, tid)) if args.op == "cast" else
               (lambda a: B.sr_cast_f32_fp8(a["src"], a["dst"], fmt, seed, 7, tid)))
        placed, placement = placed_arrays({"src": (torch.float32, n), "dst": (out_dtype, n)}, run)
        src = placed["src"] if placed else torch.empty(n, dtype=torch.float32, device=dev)
        for k, at in enumerate(range(0, n, 1 << 28)):            # generated in pieces of 2^28 elements
            piece = src[at:at + (1 << 28)]
            piece.copy_(W.make_cast_input(piece.numel(), dev, W.data_seed(cfg.index, 900 + k)))
        host = src[lo:lo + n_cpu].cpu().numpy()
        if args.op == "cast":
            dst = placed["dst"] if placed else torch.empty(n, dtype=torch.bfloat16, device=dev)
            fn = lambda: B.sr_cast_f32_bf16(src, dst, seed, 7, tid)
            bpe, kernel, metric = 6, "cast_kernel", "sr_cast_elements_per_sec"
            wall, dev_ms = time_launches(torch, np, fn, args.warmup, args.steps)
            t0 = time.perf_counter()
            want = ref.sr_cast_f32_bf16(host, seed, 7, tid, elem_offset=lo, nthreads=threads)
            dt = time.perf_counter() - t0
            bad = int((W.bf16_to_u16_numpy(dst[lo:lo + n_cpu]) != want).sum())
        else:                                                    # 8-bit formats: 4 B read + 1 B written
            ofmt = ref.E4M3 if args.op == "cast_e4m3" else ref.E5M2
            dst = placed["dst"] if placed else torch.empty(n, dtype=torch.uint8, device=dev)
            fn = lambda: B.sr_cast_f32_fp8(src, dst, fmt, seed, 7, tid)
            bpe, kernel, metric = 5, "cast_fp8_kernel", "sr_cast_fp8_elements_per_sec"
            wall, dev_ms = time_launches(torch, np, fn, args.warmup, args.steps)
            n_cpu = min(n_cpu, 1 << 24)                          # the value-based 8-bit oracle is slow
            host = host[:n_cpu]
            t0 = time.perf_counter()
            want = ref.sr_cast_f32_fp8(host, ofmt, seed, 7, tid, elem_offset=lo, nthreads=threads)
            dt = time.perf_counter() - t0
            bad = int((dst[lo:lo + n_cpu].cpu().numpy() != want).sum())
    else:
        with_norm = args.op == "accumulate_norm"
        norm = torch.zeros(1, dtype=torch.float32, device=dev) if with_norm else None
        ws = (torch.empty(max(B.lib().sr_accumulate_workspace_bytes(1, n), 256), dtype=torch.uint8, device=dev)
              if with_norm else None)
        placed, placement = placed_arrays({"acc": (torch.bfloat16, n), "g": (torch.bfloat16, n)},
                                          lambda a: B.sr_grad_accumulate(B.AccumList([a["acc"]], [a["g"]], tensor_ids=[tid]),
                                                                         0.25, 1, seed, 0, norm, ws))
        if placed:
            acc, g = placed["acc"], placed["g"]
            W.fill_grads([acc], W.data_seed(cfg.index, 901), cfg.grad_std)
            W.fill_grads([g], W.data_seed(cfg.index, 902), cfg.grad_std)
        else:
            acc = W.make_grads(flat, dev, W.data_seed(cfg.index, 901), cfg.grad_std)[0]
            g = W.make_grads(flat, dev, W.data_seed(cfg.index, 902), cfg.grad_std)[0]
        al = B.AccumList([acc], [g], tensor_ids=[tid])
        k = [0]

        def fn():
            k[0] += 1
            B.sr_grad_accumulate(al, 0.25, k[0], seed, 0, norm, ws)
        bpe, kernel, metric = 6, "accumulate_kernel", "sr_grad_accumulate_elements_per_sec"
        wall, dev_ms = time_launches(torch, np, fn, args.warmup, args.steps)
        a0 = W.bf16_to_u16_numpy(acc[lo:lo + n_cpu])
        g0 = W.bf16_to_u16_numpy(g[lo:lo + n_cpu])
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ref.grad_accumulate(a0, g0, 0.25, k[0], seed, tensor_id=tid, elem_offset=lo, nthreads=threads)
        want = a0                                                # updated in place
        dt = time.perf_counter() - t0
        bad = int((W.bf16_to_u16_numpy(acc[lo:lo + n_cpu]) != want).sum())
    if args.calibrate_copy:
        calibrate_copy(torch, dev)
    avg = float(np.mean(dev_ms))
    achieved = bpe * n / (avg * 1e-3) / 1e9
    traffic, traffic_source = profile_traffic(f"config{cfg.index}_op_{args.op}")
    print(json.dumps({
        "metric": metric, "value": n * args.steps / wall, "unit": "elements/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.op} on one flat array of config {cfg.index}'s size", "numel": n,
                   "bytes_per_element": bpe, "placement": placement},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": kernel,
                     "avg_launch_ms": avg, "median_launch_ms": float(np.median(dev_ms)),
                     "min_launch_ms": float(np.min(dev_ms))},
        "cpu_baseline": {"value": n_cpu / dt, "unit": "elements/s", "cores": threads, "kind": "oracle",
                         "sample": f"{n_cpu} contiguous elements from the middle of the array, {dt:.1f} s"},
        "parity_sample": "bit-exact" if bad == 0 else f"{bad} mismatches"}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed steps (default 20; 200 for configurations whose step moves under 10 GB, where "
                         "the first steps after the synchronisation run below full clocks and would dominate)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps before them (default 3; 20 for those)")
    ap.add_argument("--config", type=int, default=5)
    ap.add_argument("--mode", choices=sorted(MODES), default=None,
                    help="step variant (default: the config's own: sr, or fp32_moments for config 4)")
    ap.add_argument("--op", choices=("step", "cast", "cast_e4m3", "cast_e5m2", "accumulate", "accumulate_norm"),
                    default="step")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time its replays (same step number "
                         "on every replay; removes launch gaps of many-tensor lists)")
    ap.add_argument("--step-events", choices=("auto", "on", "off"), default="auto",
                    help="an event pair around every step (on), one pair around the timed region (off), "
                         "or by step size (auto: per step from 10 GB per step upwards)")
    ap.add_argument("--resident-waves", type=int, default=0,
                    help="measurement only: override the number of waves the library lets reside per "
                         "compute unit in its streaming kernels (0 = the library's own setting, 32 = no cap)")
    ap.add_argument("--placement", choices=("probe", "plain", "slowest"), default="probe",
                    help="flat configurations: choose the state's arrays among spare allocations by timing "
                         "a sample of layouts (probe: the no-arithmetic probe for an all-BF16 state, the step "
                         "itself on zero-filled candidates otherwise), or take them as the allocator returns "
                         "them (plain); slowest keeps the worst probed layout, to measure what placement costs")
    ap.add_argument("--placement-candidates", type=int, default=8)
    ap.add_argument("--placement-layouts", type=int, default=40)
    ap.add_argument("--warm-steps", type=int, default=None, help="seeded steps that warm the moments")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region, do one device copy of 2^30 bytes (a dispatch of "
                         "known traffic that scales the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                 "run it with --gpus 1")

    import numpy as np
    import torch
    from paper_2502_20566_amd import binding as B
    from paper_2502_20566_amd import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the update path has no CPU fallback")
    B.lib()                                               # fail loudly if the library is missing
    if args.resident_waves:
        B.lib().sr_debug_set(B.SR_DEBUG_RESIDENT_WAVES, args.resident_waves)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    cfg = W.config(args.config)
    short_steps = args.op == "step" and 22 * cfg.numel < 1e10
    if args.steps is None:
        args.steps = 200 if short_steps else 20
    if args.warmup is None:
        args.warmup = 20 if short_steps else 3
    if args.op != "step":
        run_aux_op(args, torch, np, B, W, cfg)
        return
    warm = cfg.warm_steps if args.warm_steps is None else args.warm_steps
    mode = args.mode or ("fp32_moments" if cfg.fp32_moments else "sr")
    flag_names, fp32_moments, aux_kind, _ = MODES[mode]
    flags = 0
    for name in flag_names:
        flags |= getattr(B, name)

    placement = {"policy": "as the allocator returns them"}
    import math
    fp8m, fp8p = mode in ("fp8_moments", "fp8_all"), mode in ("fp8_params", "fp8_all")
    fp8_exps = fp8_scale_exponents(cfg) if fp8m else None
    # the weights go onto the E4M3 grid with the library's own stochastic cast: eight standard
    # deviations (gains of 1 included) map to the top of the format
    p_exp = int(math.floor(math.log2(448.0 / max(8.0 * cfg.param_std, 1.0)))) if fp8p else None

    def quantise(src, dst, tensor_id):
        for at in range(0, src.numel(), 1 << 28):
            piece = src[at:at + (1 << 28)].float() * float(2.0 ** p_exp)
            B.sr_cast_f32_fp8(piece, dst[at:at + (1 << 28)], B.SR_FP8_E4M3, cfg.seed, 0, tensor_id)
        torch.cuda.synchronize()

    sizes = [W.numel_of(shape) for _, shape, _ in cfg.shapes]
    starts = [sum(sizes[:i]) for i in range(len(sizes))]

    def views(buf):
        """The list's tensors as consecutive slices of one backing array."""
        return [buf[o:o + n] for o, n in zip(starts, sizes)]

    def tensor_list(a):
        k = len(sizes)
        return B.TensorList(views(a["p"]), views(a["g"]), views(a["m"]), views(a["v"]), fp32_moments,
                            aux=views(a["aux"]) if "aux" in a else None,
                            fp8_exponents=None if fp8_exps is None else [fp8_exps] * k,
                            fp8_param_exponents=None if p_exp is None else [p_exp] * k)

    placed = None
    # lists keep one allocation per tensor: held as slices of placed backing arrays they gained
    # 0-1% (measured on configs 2-4), not worth a storage layout of the benchmark's own
    if args.placement in ("probe", "slowest") and len(sizes) == 1 and cfg.numel >= (1 << 28):
        from paper_2502_20566_amd import placement as P
        slowest = args.placement == "slowest"
        if MODES[mode][3] == 14 and len(sizes) == 1:
            four, placement = P.place_flat_buffers(cfg.numel, dev, args.placement_candidates, args.placement_layouts, slowest=slowest)
            placed = None if four is None else dict(zip("pgmv", four))
        else:
            # arrays of several sizes: the step itself, on zero-filled candidates, is the probe
            moment = torch.float32 if fp32_moments else torch.uint8 if fp8m else torch.bfloat16
            roles = {"p": (torch.uint8 if fp8p else torch.bfloat16, cfg.numel), "g": (torch.bfloat16, cfg.numel),
                     "m": (moment, cfg.numel), "v": (moment, cfg.numel)}
            if aux_kind is not None:
                roles["aux"] = (torch.float32 if aux_kind == "f32" else torch.bfloat16, cfg.numel)
            reps = max(2, int(30.0 / (MODES[mode][3] * cfg.numel / 6.0e9)))      # about 30 ms of timed work
            probe_norm = torch.ones(1, dtype=torch.float32, device=dev)
            probe_ws = [None]

            def time_layout(a):
                tl_ = tensor_list(a)
                if probe_ws[0] is None:
                    probe_ws[0] = torch.empty(max(tl_.workspace_bytes(), 256), dtype=torch.uint8, device=dev)

                def step_():
                    if cfg.clip is not None:
                        B.grad_global_norm(tl_, probe_norm, probe_ws[0])
                        B.sr_adamw_step(tl_, cfg.hyper, 1, cfg.seed, flags, probe_norm, cfg.clip)
                    else:
                        B.sr_adamw_step(tl_, cfg.hyper, 1, cfg.seed, flags)
                step_()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    step_()
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / reps

            placed, placement = P.place_state_buffers(roles, dev, time_layout, n_layouts=min(args.placement_layouts, 24), slowest=slowest)
    if placed is not None:
        tmp = W.make_params(cfg.shapes, dev, W.data_seed(cfg.index, 0), cfg.param_std)
        for i, (src, dst) in enumerate(zip(tmp, views(placed["p"]))):
            if fp8p:
                quantise(src, dst, i)
            else:
                dst.copy_(src)
        if aux_kind == "f32":
            for src, dst in zip(tmp, views(placed["aux"])):
                dst.copy_(src)                            # binary32 master parameters
        elif aux_kind == "bf16":
            placed["aux"].zero_()                         # Kahan compensation starts at zero
        del tmp
        torch.cuda.empty_cache()
        placed["m"].zero_()
        placed["v"].zero_()
        params, grads, ms, vs = views(placed["p"]), views(placed["g"]), views(placed["m"]), views(placed["v"])
        aux = views(placed["aux"]) if "aux" in placed else None
    else:
        params = W.make_params(cfg.shapes, dev, W.data_seed(cfg.index, 0), cfg.param_std)
        ms, vs = W.make_moments(cfg.shapes, dev, fp32_moments)
        if fp8m:
            ms = [torch.zeros(m.numel(), dtype=torch.uint8, device=dev) for m in ms]
            vs = [torch.zeros(v.numel(), dtype=torch.uint8, device=dev) for v in vs]
        grads = [torch.empty_like(p) for p in params]
        aux = None
        if aux_kind == "f32":
            aux = [p.float() for p in params]             # binary32 master parameters
        elif aux_kind == "bf16":
            aux = [torch.zeros_like(p) for p in params]   # Kahan compensation starts at zero
        if fp8p:
            p8s = []
            for i, p_ in enumerate(params):
                q = torch.empty(p_.numel(), dtype=torch.uint8, device=dev)
                quantise(p_, q, i)
                p8s.append(q)
            params = p8s
            del p8s
            torch.cuda.empty_cache()
    tl = B.TensorList(params, grads, ms, vs, fp32_moments, aux=aux,
                      fp8_exponents=None if fp8_exps is None else [fp8_exps] * len(params),
                      fp8_param_exponents=None if p_exp is None else [p_exp] * len(params))
    norm = torch.zeros(1, dtype=torch.float32, device=dev)
    ws = torch.empty(max(tl.workspace_bytes(), 256), dtype=torch.uint8, device=dev)
    numel = tl.total_numel

    def one_step(t):
        if cfg.clip is not None:
            B.grad_global_norm(tl, norm, ws)
            B.sr_adamw_step(tl, cfg.hyper, t, cfg.seed, flags, norm, cfg.clip)
        else:
            B.sr_adamw_step(tl, cfg.hyper, t, cfg.seed, flags)

    # warm-start of the moments: seeded steps with fresh gradients (a seed per step)
    t = 0
    for _ in range(warm):
        t += 1
        W.fill_grads(grads, W.data_seed(cfg.index, t), cfg.grad_std, cfg.outlier_frac, cfg.outlier_std)
        one_step(t)
    t += 1
    W.fill_grads(grads, W.data_seed(cfg.index, t), cfg.grad_std, cfg.outlier_frac, cfg.outlier_std)
    torch.cuda.synchronize()

    # CPU oracle on a bounded window (needs the state BEFORE the step it reproduces)
    cpu = None
    check = None
    if not args.no_cpu_baseline:
        nv = None
        if cfg.clip is not None:
            # the norm of this step's gradients as the device computes it: the oracle clips with
            # the same binary32 value
            B.grad_global_norm(tl, norm, ws)
            torch.cuda.synchronize()
            nv = float(norm.item())
        cpu, check = cpu_baseline(W, B, torch, cfg, (params[0], grads[0], ms[0], vs[0],
                                                     None if aux is None else aux[0]), t, cfg.seed,
                                  args.cpu_seconds, flags, fp8_exps, nv, p_exp)

    # the step the oracle reproduced, then the parity check of that window
    parity = "not checked"
    if check is not None:
        one_step(t)
        torch.cuda.synchronize()
        lo, n, w = check
        got_p = params[0][lo:lo + n].cpu().numpy() if p_exp is not None else W.bf16_to_u16_numpy(params[0][lo:lo + n])
        bad = int((got_p != w["p"]).sum())
        if fp32_moments or fp8_exps is not None:
            bad += int((ms[0][lo:lo + n].cpu().numpy().view(np.uint32 if fp32_moments else np.uint8)
                        != w["m"].view(np.uint32 if fp32_moments else np.uint8)).sum())
            bad += int((vs[0][lo:lo + n].cpu().numpy().view(np.uint32 if fp32_moments else np.uint8)
                        != w["v"].view(np.uint32 if fp32_moments else np.uint8)).sum())
        else:
            bad += int((W.bf16_to_u16_numpy(ms[0][lo:lo + n]) != w["m"]).sum())
            bad += int((W.bf16_to_u16_numpy(vs[0][lo:lo + n]) != w["v"]).sum())
        if aux_kind == "f32":
            bad += int((aux[0][lo:lo + n].cpu().numpy() != w["aux"]).sum())
        elif aux_kind == "bf16":
            bad += int((W.bf16_to_u16_numpy(aux[0][lo:lo + n]) != w["aux"]).sum())
        parity = "bit-exact" if bad == 0 else f"{bad} mismatches"
        del got_p
        t += 1

    step_fn = one_step
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                one_step(t)
        torch.cuda.current_stream().wait_stream(side)
        step_fn = lambda _t: graph.replay()
    for _ in range(args.warmup):
        step_fn(t)
    torch.cuda.synchronize()

    # timed region: exactly K steps, inputs resident, HIP events on the launch stream.  Long steps
    # (one big launch) get an event pair each, so that median and minimum are known; steps of a
    # few hundred microseconds get ONE pair around the region, because an event record drains the
    # queue and the refill would be charged to every step (measured: 0.345 against 0.28 ms per
    # step on the 124M-element list).
    per_step = args.step_events == "on" or (args.step_events == "auto" and MODES[mode][3] * numel >= 1e10)
    n_ev = args.steps if per_step else 1
    ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(n_ev)]
    ev1 = [torch.cuda.Event(enable_timing=True) for _ in range(n_ev)]
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    if per_step:
        for i in range(args.steps):
            ev0[i].record()
            step_fn(t + i)
            ev1[i].record()
    else:
        ev0[0].record()
        for i in range(args.steps):
            step_fn(t + i)
        ev1[0].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_start
    ms_per_step = wall * 1e3 / args.steps
    dev_ms = [a.elapsed_time(b) for a, b in zip(ev0, ev1)]
    dev_avg_ms = float(np.sum(dev_ms)) / args.steps

    # ceiling of the access pattern on these very buffers: the step's 4-read/3-write traffic with
    # no arithmetic (BF16 strategies without an auxiliary tensor, flat or list alike)
    ceiling = None
    if MODES[mode][3] == 14 or mode == "fp8_moments":
        def probe():
            for p_, g_, m_, v_ in zip(params, grads, ms, vs):
                (B.sr_stream_probe_fp8m if fp8_exps is not None else B.sr_stream_probe)(p_, g_, m_, v_)
        probe()
        torch.cuda.synchronize()
        reps = max(3, min(args.steps, 10))
        pe0 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
        pe1 = [torch.cuda.Event(enable_timing=True) for _ in range(reps)]
        for i in range(reps):
            pe0[i].record()
            probe()
            pe1[i].record()
        torch.cuda.synchronize()
        probe_ms = float(np.mean([a.elapsed_time(b) for a, b in zip(pe0, pe1)]))
        ceiling = {"kind": "the step's reads and writes of the same buffers, no arithmetic (sr_stream_probe" +
                           ("_fp8m: 6 B read, 4 B written per element)" if fp8_exps is not None else ": 8 B read, 6 B written per element)"),
                   "ms": probe_ms, "GBps": MODES[mode][3] * numel / (probe_ms * 1e-3) / 1e9}

    # a plain device copy of the same footprint per buffer (1 read : 1 write), torch's copy kernel
    device_copy = None
    if ceiling is not None:
        big = max(range(len(params)), key=lambda i: params[i].numel())
        src_t, dst_t = params[big], grads[big]                 # the gradients are not needed any more
        dst_t.copy_(src_t)
        torch.cuda.synchronize()
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for _ in range(3):
            dst_t.copy_(src_t)
        c1.record()
        torch.cuda.synchronize()
        copy_ms = c0.elapsed_time(c1) / 3
        device_copy = {"kind": "torch copy_ of the largest parameter tensor into its gradient buffer",
                       "bytes": 4 * src_t.numel(), "ms": copy_ms, "GBps": 4 * src_t.numel() / (copy_ms * 1e-3) / 1e9}

    if args.calibrate_copy:
        calibrate_copy(torch, dev)

    bpe = algorithmic_bytes_per_element(mode, cfg.clip)
    value = numel * args.steps / wall
    achieved = bpe * numel / (dev_avg_ms * 1e-3) / 1e9
    # HBM bytes per step measured with rocprofv3 PMC counters: taken from the summary under
    # profiles/ for this config and mode, and only while that summary was made from the kernel
    # sources this library is built from (it records their hash); otherwise null
    traffic, traffic_source = profile_traffic(f"config{cfg.index}_{mode}")

    out = {
        # the headline metric as the baseline names it; `value` is its first quantity (params/s),
        # the other two are hbm_GBps and pct_of_hbm_peak below
        "metric": "SR-AdamW params updated/sec and achieved HBM GB/s (% of MI355X peak)",
        "value": value,
        "unit": "params/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"config {cfg.index}: {cfg.name}", "numel": numel, "tensors": len(params),
                   "mode": mode, "storage": "bf16 gradients; parameters " + ("e4m3 codes, scale exponent %d" % p_exp if p_exp is not None else "bf16"),
                   "moments": "fp32" if fp32_moments else "e4m3/e5m2" if fp8_exps else "bf16",
                   "fp8_scale_exponents": fp8_exps, "clip": cfg.clip,
                   "warm_steps": warm, "bytes_per_element": bpe, "hip_graph": bool(args.graph),
                   "placement": placement, "resident_waves_override": args.resident_waves or None},
        "hbm_GBps": bpe * numel / (ms_per_step * 1e-3) / 1e9,
        "pct_of_hbm_peak": 100.0 * bpe * numel / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "adamw_kernel" if cfg.clip is None and len(params) <= 320 else
                     "all launches of a step (norm passes + adamw_kernel per 320 tensors)", "avg_launch_ms": dev_avg_ms,
                     "median_launch_ms": float(np.median(dev_ms)) if per_step else None,
                     "min_launch_ms": float(np.min(dev_ms)) if per_step else None,
                     "events": "a pair per step" if per_step else "one pair around the timed region",
                     "copy_ceiling": ceiling, "device_copy": device_copy,
                     "frac_of_copy_ceiling": None if ceiling is None else
                     (MODES[mode][3] * numel / (dev_avg_ms * 1e-3) / 1e9) / ceiling["GBps"]},
        "cpu_baseline": cpu,
        "parity_sample": parity,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
