"""What the reduced-precision pseudo-gradient costs numerically (Section "All-Reduce in FP16":
the paper reports no noticeable effect on training): the averaged pseudo-gradient of one round
on the 150M set, 8 workers, in every reduced-precision mode against the FP32 mode, element by
element against the bound the rounding itself implies, with the measured statistics printed.

After the first outer step the momentum buffer IS the averaged pseudo-gradient (b starts at
zero: b <- mu*0 + mean), so it can be read back directly."""
import pytest

import oracle
import synth
from harness import GpuSide

pytestmark = pytest.mark.gpu

H = 20


@pytest.mark.timeout(600)
def test_reduced_precision_average_stays_within_its_rounding_bound():
    import torch
    wl = synth.llama_150m()
    k = 8
    ref = GpuSide(wl, k, oracle.PG_F32)
    for step in range(H):
        ref.dl.inner_step(ref.gen_grads(step))
    theta_after = ref.dl.theta.clone()                      # [k, n_pad] after H inner steps
    theta0_before = ref.dl.theta0.clone()
    ref.dl.outer_step()
    torch.cuda.synchronize()
    mean32 = ref.dl.mom.clone()
    n_pad = ref.n_pad
    ref.dl.close()
    del ref

    # per element: mean over workers of |delta_r| (FP32 subtraction, as the kernel forms it)
    mean_abs = torch.zeros(n_pad, device="cuda")
    for r in range(k):
        mean_abs += (theta0_before - theta_after[r]).abs()
    mean_abs /= k
    scale = mean32.abs().mean().item()
    assert 1e-4 < scale < 1e-1, scale                       # a realistic pseudo-gradient magnitude
    print("\nmean |averaged pseudo-gradient| after %d inner steps: %.3e" % (H, scale))

    for name, pg, rm, u, floor in (("f16", oracle.PG_F16, False, 2.0 ** -11, 2.0 ** -25),
                                   ("f16 + rounded mean", oracle.PG_F16, True, 2.0 ** -11, 2.0 ** -25),
                                   ("bf16", oracle.PG_BF16, False, 2.0 ** -8, 0.0),
                                   ("bf16 + rounded mean", oracle.PG_BF16, True, 2.0 ** -8, 0.0)):
        side = GpuSide(wl, k, pg, round_mean=rm)
        side.dl.theta.copy_(theta_after)
        side.dl.outer_step()
        torch.cuda.synchronize()
        diff = (side.dl.mom - mean32).abs()
        # each worker's pseudo-gradient moves by at most u*|delta_r| (normal range) or half a
        # binary16 subnormal step; the FP32 sums of k terms differ by a few of their own roundings
        bound = u * mean_abs + floor + (2 * k) * 2.0 ** -24 * mean_abs
        if rm:
            bound = bound + u * (mean32.abs() + bound) + floor
        worst = (diff - bound).max().item()
        assert worst <= 0.0, "%s: an element exceeds its rounding bound by %.3e" % (name, worst)
        rel = diff.mean().item() / scale
        print("%-20s max |diff| %.3e  mean |diff| %.3e  = %.2e of the mean magnitude; "
              "largest ratio to the bound %.3f"
              % (name, diff.max().item(), diff.mean().item(), rel,
                 (diff / bound.clamp_min(1e-45)).max().item()))
        # and the mode does change the result (it is not silently the FP32 path)
        assert diff.max().item() > 0.0
        assert rel < u                                        # far below one unit of the format
        side.dl.close()
        del side, diff, bound
