"""Placement of the flat arrays of an optimizer state in device memory.

Allocation logic only (which allocations hold p, g, m, v and the auxiliary array); the timing runs
the library through the C ABI: its no-arithmetic probe of the step's traffic for the all-BF16
state, the step itself on a zero state for the other storage formats.  Used by bench.py; a
training job can call either once at start-up.
"""
import itertools
import random
import statistics

import torch

from . import binding as B


def place_flat_buffers(n, dev, n_candidates=8, n_layouts=40, slowest=False):
    """Where p, g, m, v lie in physical memory moves the 4-read/3-write stream by several percent on
    MI355X (14.1 to 15.4 ms for the same kernel on the 6.7B buffers; the ranking of layouts is stable
    within a process and follows no rule in the virtual addresses).  So the four flat arrays are
    chosen among a few more allocations of the same size: the no-arithmetic probe of the step's
    traffic (sr_stream_probe) is timed on a sample of assignments and the fastest is kept; the
    spare allocations are freed.  Returns ((p, g, m, v), report), or (None, report) when the
    device has no room for the candidates."""
    free, _ = torch.cuda.mem_get_info()
    n_candidates = max(4, min(n_candidates, int((free - (24 << 30)) // (2 * n))))
    if n_candidates < 5:
        return None, {"policy": "as the allocator returns them", "why": "no room for spare candidates"}
    bufs = [torch.zeros(n, dtype=torch.bfloat16, device=dev) for _ in range(n_candidates)]

    def probe_ms(perm, reps=2):
        a = [bufs[i] for i in perm]
        B.sr_stream_probe(*a)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            B.sr_stream_probe(*a)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    rng = random.Random(0)
    layouts = [tuple(range(4))]
    every = list(itertools.permutations(range(n_candidates), 4))
    layouts += rng.sample(every, min(n_layouts - 1, len(every)))
    times = [probe_ms(l) for l in layouts]
    # the best few once more, with more repetitions, so that one lucky timing does not decide
    order = sorted(range(len(layouts)), key=lambda i: times[i], reverse=slowest)
    finals = {i: probe_ms(layouts[i], 4) for i in order[:4]}
    best = (max if slowest else min)(finals, key=finals.get)
    chosen = tuple(bufs[i] for i in layouts[best])
    report = {"policy": ("SLOWEST (a measurement of what placement costs)" if slowest else "fastest") +
                        " of the probed layouts (sr_stream_probe on spare allocations of the same size)",
              "candidates": n_candidates, "layouts_tried": len(layouts),
              "probe_ms": {"chosen": finals[best], "as_allocated": times[0], "median": float(statistics.median(times)),
                           "worst": max(times), "best_first_pass": min(times)}}
    del bufs
    torch.cuda.empty_cache()
    return chosen, report


def place_state_buffers(roles, dev, time_layout, spare=2, n_layouts=24, slowest=False):
    """The same choice for a state whose arrays differ in size (binary32 or 8-bit moments, master
    parameters, 8-bit parameters).  roles: {name: (dtype, numel)}.  Arrays of equal byte size form a
    class; every class gets `spare` allocations more than it has arrays, a layout assigns distinct
    allocations of its class to each array, and time_layout({name: tensor}) -> milliseconds times
    whatever the caller runs on it (bench.py: the update itself on the zero-filled candidates;
    only the ranking of the layouts is used, the 8-bit conversions take a shorter path on
    zeros).  Returns ({name: tensor}, report), or
    (None, report) when the device has no room."""
    classes = {}
    for name, (dtype, numel) in roles.items():
        classes.setdefault(numel * torch.empty(0, dtype=dtype).element_size(), []).append(name)
    free, _ = torch.cuda.mem_get_info()
    while spare >= 1 and sum(nbytes * (len(names) + spare) for nbytes, names in classes.items()) > free - (24 << 30):
        spare -= 1
    if spare < 1:
        return None, {"policy": "as the allocator returns them", "why": "no room for spare candidates"}
    cands = {nbytes: [torch.zeros(nbytes, dtype=torch.uint8, device=dev) for _ in range(len(names) + spare)]
             for nbytes, names in classes.items()}

    def tensors(layout):
        out = {}
        for nbytes, names in classes.items():
            for name, idx in zip(names, layout[nbytes]):
                out[name] = cands[nbytes][idx].view(roles[name][0])
        return out

    rng = random.Random(0)
    layouts = [{nbytes: tuple(range(len(names))) for nbytes, names in classes.items()}]
    for _ in range(n_layouts - 1):
        layouts.append({nbytes: tuple(rng.sample(range(len(cands[nbytes])), len(names))) for nbytes, names in classes.items()})
    times = [time_layout(tensors(l)) for l in layouts]
    order = sorted(range(len(layouts)), key=lambda i: times[i], reverse=slowest)
    finals = {i: time_layout(tensors(layouts[i])) for i in order[:4]}
    best = (max if slowest else min)(finals, key=finals.get)
    chosen = tensors(layouts[best])
    report = {"policy": ("SLOWEST (a measurement of what placement costs)" if slowest else "fastest") +
                        " of the probed layouts (the step itself on a zero state, spare allocations per array size)",
              "spare_per_size": spare, "layouts_tried": len(layouts),
              "probe_ms": {"chosen": finals[best], "as_allocated": times[0], "median": float(statistics.median(times)),
                           "worst": max(times), "best_first_pass": min(times)}}
    del cands
    torch.cuda.empty_cache()
    return chosen, report
