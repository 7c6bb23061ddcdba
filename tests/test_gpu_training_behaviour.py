"""The paper's central empirical claim at toy scale (Sections 2.2 and 5): with updates below the BF16
spacing of the weights, BF16 training with nearest rounding stagnates, BF16 with stochastic rounding
follows FP32-master mixed precision, and Kahan compensation does too.  A 64-128-16 tanh student is
fitted to a fixed FP32 teacher on fresh Gaussian batches with SRAdamW at lr = 1e-4 (Adam moves every
weight by about lr per step; weights near 0.1 have a BF16 spacing of 4.9e-4, so nearest rounding
drops most updates).  Not the paper's experiment (no data or model of its own is used): a
behavioural check of the library in a training loop, with thresholds far from the observed values
(final losses: master 0.00301, sr 0.00302, kahan 0.00301, nearest 0.0677).  The same fit with the
moments held in 8 bits (an extension beyond the paper) must learn as well; here |m| stays below
1.1e-2 and v below 1.3e-4 (measured), so m 2^14 and v 2^28 stay inside E4M3 and E5M2, and scales
64 times larger, which saturate both moments early in the run, must still learn (final losses
0.00301 and 0.00288)."""
import pytest
import torch

from paper_2502_20566_amd.optimizer import SRAdamW

pytestmark = pytest.mark.gpu
DEV = "cuda"


def final_loss(strategy: str, steps: int = 600, lr: float = 1e-4, **kw) -> float:
    torch.manual_seed(0)
    teacher = torch.nn.Sequential(torch.nn.Linear(64, 128), torch.nn.Tanh(), torch.nn.Linear(128, 16)).to(DEV)
    torch.manual_seed(1)
    student = torch.nn.Sequential(torch.nn.Linear(64, 128), torch.nn.Tanh(), torch.nn.Linear(128, 16))
    student = student.to(DEV).to(torch.bfloat16)
    opt = SRAdamW(student.parameters(), lr=lr, betas=(0.9, 0.95), weight_decay=0.0, seed=0, strategy=strategy, **kw)
    gen = torch.Generator(device=DEV).manual_seed(2)
    tail = []
    for t in range(steps):
        x = torch.randn(256, 64, device=DEV, generator=gen)
        with torch.no_grad():
            y = teacher(x)
        loss = (student(x.to(torch.bfloat16)).float() - y).pow(2).mean()
        loss.backward()
        opt.step()
        opt.zero_grad()
        if t >= steps - 50:
            tail.append(float(loss.detach()))
    return sum(tail) / len(tail)


def test_sr_tracks_master_weights_and_nearest_rounding_stagnates():
    master = final_loss("master")
    sr = final_loss("sr")
    sr_param = final_loss("sr_param")
    kahan = final_loss("kahan")
    nearest = final_loss("nearest")
    assert master < 0.01                                     # the reference run learns (start: 0.14)
    assert abs(sr - master) < 0.05 * master                  # SR on p, m, v follows it
    assert abs(sr_param - master) < 0.05 * master            # SR on p only (the paper's setting) too
    assert abs(kahan - master) < 0.05 * master
    assert nearest > 5 * master                              # plain BF16 is stuck far above


def test_eight_bit_moments_learn_like_bf16_moments():
    sr = final_loss("sr")
    fp8 = final_loss("fp8_moments", fp8_exponents=(14, 28))
    assert sr < 0.01 and abs(fp8 - sr) < 0.25 * sr          # noisier second moments, same fit
    saturating = final_loss("fp8_moments", fp8_exponents=(20, 40))
    assert abs(saturating - sr) < 0.25 * sr                  # no infinity is stored, nothing freezes
