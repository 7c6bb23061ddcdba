"""The linear-loss toy of Section 2.2 run through the library: f(x) = -(x - 2) + 1 for x < 3, else 0,
minimised by Adam from x0 = 2 with a decaying learning rate that has a floor.  The paper does not
give its schedule, so the step counts here are not the paper's (4600 for FP32, about 7700 for
BF16+SR); what is checked is the behaviour it reports: full-precision updates reach x = 3, BF16
with nearest rounding never leaves x0 (every update is far below half a BF16 spacing), BF16 with
SR gets there but later on average: a walk that is behind when the learning rate has decayed
waits on ever smaller updates, which gives the arrival times a heavy right tail.
"""
import pytest
import torch

from paper_2502_20566_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda"


def run(flags, fp32_moments, master, n=256, max_steps=30000):
    p = torch.full((n,), 2.0, dtype=torch.bfloat16, device=DEV)
    mdt = torch.float32 if fp32_moments else torch.bfloat16
    m = torch.zeros(n, dtype=mdt, device=DEV)
    v = torch.zeros(n, dtype=mdt, device=DEV)
    g = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    aux = [p.float()] if master else None
    tl = B.TensorList([p], [g], [m], [v], fp32_moments, aux=aux)
    hit = torch.full((n,), -1, dtype=torch.int64, device=DEV)
    x = aux[0] if master else p
    for t in range(1, max_steps + 1):
        lr = max(1e-5, 1.2e-3 * 0.999 ** t)                 # our schedule: geometric decay with a floor
        g.copy_(torch.where(x.float() < 3.0, -1.0, 0.0))    # the loss has slope -1 below 3, 0 above
        B.sr_adamw_step(tl, dict(lr=lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0), t, 1234, flags)
        if t % 50 == 0:
            reached = (x.float() >= 3.0) & (hit < 0)
            hit[reached] = t
            if bool((hit >= 0).all()):
                break
    torch.cuda.synchronize()
    return hit.cpu().numpy(), x.float().cpu().numpy()


def test_linear_loss_toy_behaviour():
    hit32, _ = run(B.SR_FLAG_MASTER_FP32 | B.SR_FLAG_FP32_MOMENTS, True, True, n=8)
    assert (hit32 > 0).all() and len(set(hit32.tolist())) == 1      # deterministic, converges
    t32 = int(hit32[0])

    hit_nr, x_nr = run(B.SR_FLAG_RNE_PARAMS | B.SR_FLAG_RNE_MOMENTS, False, False, n=8, max_steps=3000)
    assert (hit_nr < 0).all() and (x_nr == 2.0).all()               # stagnation: Q(x + u) = x

    hit_sr, x_sr = run(B.SR_FLAG_FP32_MOMENTS, True, False, n=256)   # SR on the parameter, exact moments
    done = hit_sr > 0
    assert done.mean() >= 0.95                                       # the walks arrive (positive updates only
    assert ((x_sr[~done] > 2.5) & (x_sr[~done] < 3.0)).all()         #  move x up), a few are still crawling
    assert hit_sr[done].mean() > 1.05 * t32                          # later on average: a heavy right tail of
    assert hit_sr[done].max() > 2 * t32                              #  walks that wait on floor-sized updates
    assert hit_sr[done].min() > 0.4 * t32
