"""Edge classes of inputs driven through the hot-path kernels themselves (diloco_outer_step,
diloco_unscale_check, diloco_inner_step), not through side kernels:

* every one of the 2^32 binary32 patterns as a pseudo-gradient of the fused outer step, for
  binary16 and bfloat16 pseudo-gradients (Section "All-Reduce in FP16"; overflow to inf,
  subnormals, NaN/inf propagation since the scaler plays no part in the outer step);
* every one of the 65 536 binary16 codes as a gradient of the inner step, with a power-of-two
  and a non power-of-two unscale factor;
* a flagged worker skipping its step with FP32 gradients under a loss scale ("General
  Implementation Details": the gradient scaler acts in the inner step);
* the average in the binary32 subnormal range (k a power of two and not).

NaNs compare by class only where they went through arithmetic: IEEE 754 leaves the sign and
payload of a NaN result unspecified.  Everything else is compared bit for bit.
"""
import numpy as np
import pytest

import oracle
import synth
from harness import (PAPER_HP, GpuSide, SampledCpuSide, gather_gpu, oracle_layout,
                     sample_indices)

pytestmark = pytest.mark.gpu

LOG2_CHUNK = 27
CHUNK = 1 << LOG2_CHUNK
N_CHUNKS = 1 << (32 - LOG2_CHUNK)
# chunks (top 5 pattern bits) that hold the binary16 / bfloat16 decision points: zero and the
# binary32 subnormals (0), 2^-25 and 2^-24 (6), 2^-14 (7), 65504..65520 (8), the bfloat16 overflow
# edge, inf and NaN (15); and their negative twins
EDGE_CHUNKS = [0, 6, 7, 8, 15, 16, 22, 23, 24, 31]


def same_bits(name, got, want):
    got, want = got.reshape(-1), want.reshape(-1)
    nan_w, nan_g = np.isnan(want), np.isnan(got)
    assert np.array_equal(nan_w, nan_g), name + ": NaN positions differ"
    ok = (got.view(np.uint32) == want.view(np.uint32)) | nan_w
    if not ok.all():
        i = int(np.argmin(ok))
        raise AssertionError("%s: %d mismatches; first at %d: got %08x want %08x"
                             % (name, int((~ok).sum()), i, got.view(np.uint32)[i],
                                want.view(np.uint32)[i]))


def run_outer_chunks(pg, k, round_mean, chunks):
    """theta0 = 0, mom = 0, theta_0 = -x for every pattern x of the chunk, the other workers at
    theta0: worker 0's pseudo-gradient is exactly x.  One outer step, everything compared."""
    import torch
    import paper_2407_07852_amd as D
    hp = dict(PAPER_HP)
    dl = D.DiLoCo([CHUNK], k, fill_theta0=lambda t, lay, off: t.zero_(), pg_dtype=pg,
                  pg_round_mean=int(round_mean), **hp)
    assert dl.layout.n_pad == CHUNK
    base = torch.arange(CHUNK, dtype=torch.int64, device="cuda")
    th0_c = np.zeros(CHUNK, dtype=np.float32)
    b_c = np.zeros(CHUNK, dtype=np.float32)
    theta_c = np.zeros((k, CHUNK), dtype=np.float32)
    scratch = (np.empty((k, CHUNK), dtype=np.float32), np.empty(CHUNK, dtype=np.float32))
    for c in chunks:
        first = c * CHUNK
        neg = ((base + first) & 0xFFFFFFFF) ^ 0x80000000            # bit pattern of -x
        dl.theta0.zero_()
        dl.mom.zero_()
        dl.theta.zero_()
        dl.theta[0].view(torch.int32).copy_((neg + (1 << 31)) % (1 << 32) - (1 << 31))
        dl.outer_step()
        th0_c[:] = 0
        b_c[:] = 0
        theta_c[:] = 0
        theta_c[0].view(np.uint32)[:] = np.arange(first, first + CHUNK, dtype=np.uint32) ^ 0x80000000
        oracle.outer_step(th0_c, b_c, theta_c, hp["outer_lr"], hp["outer_momentum"], pg, scratch,
                          round_mean=round_mean)
        tag = "pg%d k%d rm%d chunk %d" % (pg, k, int(round_mean), c)
        same_bits(tag + " theta0", dl.theta0.cpu().numpy(), th0_c)
        same_bits(tag + " mom", dl.mom.cpu().numpy(), b_c)
        for r in sorted({0, k - 1}):
            same_bits(tag + " theta[%d]" % r, dl.theta[r].cpu().numpy(), theta_c[r])
        print(tag, "ok", flush=True)
    dl.close()


@pytest.mark.timeout(1500)
@pytest.mark.parametrize("pg", [oracle.PG_F16, oracle.PG_BF16])
def test_outer_step_rounds_every_float_pattern(pg):
    run_outer_chunks(pg, 1, False, range(N_CHUNKS))


@pytest.mark.timeout(900)
@pytest.mark.parametrize("pg", [oracle.PG_F16, oracle.PG_BF16])
@pytest.mark.parametrize("k,round_mean", [(9, False), (2, True), (8, True)])
def test_outer_step_edge_chunks_other_kernels(pg, k, round_mean):
    """The run-time-k kernel (k = 9) and the rounded average (k = 2, 8: the halved / eighthed value
    is re-rounded, which is live in the subnormal range) on the chunks that hold every decision
    point of the two formats."""
    run_outer_chunks(pg, k, round_mean, EDGE_CHUNKS)


def test_outer_step_in_the_fp32_subnormal_range():
    """Sums and averages that land among the binary32 subnormals; k = 8 and 16 take the
    multiply-by-1/k form of the average, k = 3 and 11 the division."""
    import torch
    import paper_2407_07852_amd as D
    n = 3 * 8192
    rng = np.random.default_rng(77)
    for k in (3, 8, 11, 16):
        # magnitudes up to 2^-125 (exponent field 0 or 1), random signs and mantissas
        def tiny(size):
            bits = rng.integers(0, 2 << 23, size=size, dtype=np.uint32)
            bits |= rng.integers(0, 2, size=size, dtype=np.uint32) << 31
            return bits.view(np.float32)
        th0, b, th = tiny(n), tiny(n), tiny((k, n))
        dl = D.DiLoCo([n], k, fill_theta0=lambda t, lay, off: t.copy_(torch.from_numpy(th0)),
                      **PAPER_HP)
        dl.mom.copy_(torch.from_numpy(b))
        dl.theta.copy_(torch.from_numpy(th))
        dl.outer_step()
        th0_c, b_c, th_c = th0.copy(), b.copy(), th.copy()
        mean = oracle.outer_step(th0_c, b_c, th_c, PAPER_HP["outer_lr"], PAPER_HP["outer_momentum"],
                                 False)
        assert (np.abs(mean) < 2.0 ** -126).mean() > 0.4      # many averages really are subnormal
        same_bits("k%d theta0" % k, dl.theta0.cpu().numpy(), th0_c)
        same_bits("k%d mom" % k, dl.mom.cpu().numpy(), b_c)
        same_bits("k%d theta" % k, dl.theta.cpu().numpy(), th_c)
        dl.close()


@pytest.mark.parametrize("inv_scale", [2.0 ** -16, 1.0 / 1000.0])
def test_inner_step_on_every_binary16_gradient_code(inv_scale):
    """All 65 536 binary16 codes as gradients (subnormals, 65504, both zeros, inf, NaN).  Worker 1
    holds every code; workers 0 and 2 hold every FINITE code.  Flags must be exactly [0, 1, 0],
    worker 1 untouched bit for bit, workers 0 and 2 equal to the oracle bit for bit."""
    import torch
    import paper_2407_07852_amd as D
    numel = [65536 + 777, 65536, 40000, 25536 + 13]      # several tiles, ragged tails
    k, bad = 3, 1
    hp = dict(PAPER_HP)
    rng = np.random.default_rng(5)
    offsets, n_pad = oracle.plan_layout(numel, 64, 8192)
    real = np.zeros(n_pad, dtype=bool)
    for off, n in zip(offsets, numel):
        real[int(off):int(off) + n] = True
    th_init = np.where(real, rng.normal(scale=0.02, size=n_pad), 0).astype(np.float32)
    dl = D.DiLoCo(numel, k, fill_theta0=lambda t, lay, off: t.copy_(torch.from_numpy(th_init)), **hp)
    assert dl.layout.n_pad == n_pad and list(dl.offsets) == [int(o) for o in offsets]
    cpu = oracle.DiLoCoOracle(th_init, k, hp["inner_lr"], hp["beta1"], hp["beta2"], hp["eps"],
                              hp["weight_decay"], hp["outer_lr"], hp["outer_momentum"])
    flags = dl.new_flags()
    g = dl.new_grads(torch.float16)
    codes = np.arange(65536, dtype=np.uint16)
    finite = np.where((codes & 0x7C00) == 0x7C00, codes & 0x83FF | 0x3800, codes).astype(np.uint16)
    n_real = int(real.sum())
    for step in range(2):
        gc = []
        for r in range(k):
            src = codes if r == bad else finite
            # every code appears (n_real > 2 * 65536), at positions that differ per worker and step
            seq = np.roll(np.resize(src, n_real), 1237 * r + 4099 * step)
            if r != bad:
                assert np.unique(seq).size == np.unique(finite).size
            else:
                assert np.unique(seq).size == 65536
            flat = np.zeros(n_pad, dtype=np.uint16)
            flat[real] = seq
            gc.append(flat)
            g[r].view(torch.int16).copy_(torch.from_numpy(flat.view(np.int16)))
        want_flags = [oracle.found_inf(x) for x in gc]
        assert want_flags == [0, 1, 0]
        dl.unscale_check(g, inv_scale, flags)
        assert flags.cpu().tolist() == want_flags
        before = [t[bad].clone() for t in (dl.theta, dl.m, dl.v)]
        dl.inner_step(g, flags=flags)
        cpu.inner_step(gc, found_inf_flags=want_flags, inv_scale=float(np.float32(inv_scale)))
        for t, b in zip((dl.theta, dl.m, dl.v), before):
            assert torch.equal(t[bad].view(torch.int32), b.view(torch.int32))
        for r in range(k):
            w = cpu.workers[r]
            for name, dev in (("theta", dl.theta), ("m", dl.m), ("v", dl.v)):
                same_bits("step %d %s[%d]" % (step, name, r), dev[r].cpu().numpy(), getattr(w, name))
        assert dl.steps() == [step + 1, 0, step + 1]
    dl.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("loss_scale", [65536.0, 1000.0])
def test_fp32_gradients_under_a_loss_scale_with_one_skipped_worker(loss_scale):
    """150M set, k = 4, FP32 gradients multiplied by a loss scale; one worker's gradient holds a
    single inf.  The check flags exactly that worker; its weights, moments and step count stay
    bit for bit; the others take the step with the unscale fused in and match the oracle on the
    sampled indices (the path is elementwise)."""
    import torch
    wl = synth.llama_150m()
    k, bad = 4, 2
    inv_scale = float(np.float32(1.0 / loss_scale))
    gpu = GpuSide(wl, k)
    offsets, n_pad = oracle_layout(wl)
    idx = sample_indices(wl, offsets, n_pad, every=4099 * 4)
    cpu = SampledCpuSide(wl, k, idx)
    idx_dev = torch.from_numpy(idx.astype(np.int64)).cuda()
    flags = gpu.dl.new_flags()
    sigma = 1e-3 * loss_scale
    for step in range(2):
        g = gpu.gen_grads(step, sigma=sigma)
        gc = cpu.gen_grads(step, sigma=sigma)
        hit = int(offsets[5]) + 12345                    # a real element of a matrix
        if step == 0:
            g[bad, hit] = float("inf")
        gpu.dl.unscale_check(g, inv_scale, flags)
        want = [1 if (r == bad and step == 0) else 0 for r in range(k)]
        assert flags.cpu().tolist() == want
        before = [t[bad].clone() for t in (gpu.dl.theta, gpu.dl.m, gpu.dl.v)] if step == 0 else None
        gpu.dl.inner_step(g, flags=flags)
        cpu.o.inner_step(gc, found_inf_flags=want, inv_scale=inv_scale)
        if step == 0:
            for t, b in zip((gpu.dl.theta, gpu.dl.m, gpu.dl.v), before):
                assert torch.equal(t[bad].view(torch.int32), b.view(torch.int32))
            del before
        for name, dev in (("theta", gpu.dl.theta), ("m", gpu.dl.m), ("v", gpu.dl.v)):
            got = gather_gpu(gpu, dev, idx_dev)
            for r in range(k):
                same_bits("step %d %s[%d]" % (step, name, r), got[r], getattr(cpu.o.workers[r], name))
    assert gpu.dl.steps() == [2, 2, 1, 2] and [w.t for w in cpu.o.workers] == [2, 2, 1, 2]
    gpu.dl.close()
