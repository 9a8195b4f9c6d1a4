"""GPU parity on the Llama-shaped workloads: 150M set (k=8) full arrays for a shortened round,
then whole H=500 rounds at 150Mx8 (FP32 and FP16 pseudo-gradients) and 1.1Bx8 (FP16) on sampled
elements, in the launch configuration the benchmark times (library defaults)."""
import numpy as np
import pytest

import synth
from harness import (CpuSide, GpuSide, SampledCpuSide, compare, compare_state, gather_gpu,
                     sample_indices, STEP_RTOL, STEP_ATOL, ROUND_RTOL)

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(900)
def test_150m_k8_short_round_full_arrays():
    """Step 1 and a shortened H=2 round with the outer step, every element of every buffer."""
    wl = synth.llama_150m()
    k = 8
    gpu, cpu = GpuSide(wl, k, False, h=2), CpuSide(wl, k, False)
    assert gpu.n_pad == cpu.n_pad == 234119168
    for step in range(2):
        g = gpu.gen_grads(step)
        gc = cpu.gen_grads(step)
        if step == 0:
            assert compare("grads[7]", gpu.host(g[7]), gc[7], 0, 0) == 0
        assert gpu.dl.inner_step(g) == (1 if step == 1 else 0)
        cpu.o.inner_step(gc)
        del gc
        mism = compare_state(gpu, cpu)
        assert mism == 0, "inner step %d: %d last-bit mismatches" % (step, mism)
        print("150M k=8 inner step %d: bitwise equal" % step, flush=True)
    gpu.dl.outer_step()
    cpu.o.outer_step()
    assert compare("theta0", gpu.host(gpu.dl.theta0), cpu.o.theta0, ROUND_RTOL, STEP_ATOL) == 0
    assert compare("mom", gpu.host(gpu.dl.mom), cpu.o.b, ROUND_RTOL, STEP_ATOL) == 0
    assert compare_state(gpu, cpu, ROUND_RTOL, STEP_ATOL, what=("theta",)) == 0
    gpu.dl.close()


def _sampled_round(wl, k, pg_f16, H, rounds=1):
    gpu = GpuSide(wl, k, pg_f16, h=H)
    idx = sample_indices(wl, np.asarray(gpu.dl.offsets, dtype=np.uint64), gpu.n_pad)
    cpu = SampledCpuSide(wl, k, idx, pg_f16)
    assert gpu.n_pad == cpu.n_pad and list(gpu.dl.offsets) == [int(o) for o in cpu.offsets]
    torch = gpu.torch
    idx_dev = torch.from_numpy(idx.astype(np.int64)).to("cuda")
    assert compare("theta0 init", gather_gpu(gpu, gpu.dl.theta0, idx_dev), cpu.o.theta0, 0, 0) == 0
    for rnd in range(rounds - 1):
        # earlier rounds: compared after their outer step only
        for step in range(rnd * H, (rnd + 1) * H):
            gpu.dl.inner_step(gpu.gen_grads(step))
            cpu.o.inner_step(cpu.gen_grads(step))
        gpu.dl.outer_step()
        cpu.o.outer_step()
        assert compare("theta0 r%d" % rnd, gather_gpu(gpu, gpu.dl.theta0, idx_dev), cpu.o.theta0,
                       0, 0) == 0
        assert compare("mom r%d" % rnd, gather_gpu(gpu, gpu.dl.mom, idx_dev), cpu.o.b, 0, 0) == 0
    first = (rounds - 1) * H
    for step in range(first, first + H):
        g = gpu.gen_grads(step)
        rc = gpu.dl.inner_step(g)
        assert rc == (1 if step == first + H - 1 else 0)
        cpu.o.inner_step(cpu.gen_grads(step))
        step -= first
        if step in (0, H // 2, H - 1):
            th, m, v = (gather_gpu(gpu, t, idx_dev) for t in (gpu.dl.theta, gpu.dl.m, gpu.dl.v))
            mism = 0
            for r in range(k):
                w = cpu.o.workers[r]
                mism += compare("theta[%d]" % r, th[r], w.theta, ROUND_RTOL, STEP_ATOL)
                mism += compare("m[%d]" % r, m[r], w.m, ROUND_RTOL, 1e-12)
                mism += compare("v[%d]" % r, v[r], w.v, ROUND_RTOL, 1e-15)
            assert mism == 0, "after inner step %d: %d sampled last-bit mismatches" % (step, mism)
            print("%s k=%d inner step %d: %d samples bitwise equal" % (wl.name, k, step, idx.size),
                  flush=True)
    assert gpu.dl.steps() == [H * rounds] * k
    gpu.dl.outer_step()
    cpu.o.outer_step()
    assert compare("theta0", gather_gpu(gpu, gpu.dl.theta0, idx_dev), cpu.o.theta0, ROUND_RTOL,
                   STEP_ATOL) == 0
    assert compare("mom", gather_gpu(gpu, gpu.dl.mom, idx_dev), cpu.o.b, ROUND_RTOL, STEP_ATOL) == 0
    th = gather_gpu(gpu, gpu.dl.theta, idx_dev)
    for r in range(k):
        assert compare("theta[%d]" % r, th[r], cpu.o.workers[r].theta, ROUND_RTOL, STEP_ATOL) == 0
    # properties that hold at any size: all workers equal theta0, pads still zero
    for r in range(k):
        assert torch.equal(gpu.dl.theta[r], gpu.dl.theta0)
    assert not bool((gpu.dl.theta0[gpu.kind == 0] != 0).any())
    gpu.dl.close()


@pytest.mark.timeout(900)
@pytest.mark.parametrize("pg_f16", [False, True])
def test_150m_k8_h500_round_sampled(pg_f16):
    _sampled_round(synth.llama_150m(), 8, pg_f16, 500)


@pytest.mark.timeout(1500)
def test_1_1b_k8_h500_round_sampled_fp16():
    _sampled_round(synth.llama_1_1b(), 8, True, 500)


@pytest.mark.timeout(900)
def test_1_1b_k4_h125_round_sampled_fp16():
    """The 1.1B configuration as the paper ran it: 4 workers, 125 local steps."""
    _sampled_round(synth.llama_1_1b(), 4, True, 125)


@pytest.mark.timeout(900)
def test_150m_k4_h50_three_rounds_sampled():
    """The paper's worker-count ablation setting (H = 50), three consecutive rounds so that the
    outer momentum and the persistent AdamW moments both matter."""
    _sampled_round(synth.llama_150m(), 4, True, 50, rounds=3)


@pytest.mark.timeout(900)
def test_150m_fp16_pseudo_gradient_with_subnormals():
    """Outer step alone with an injected delta ~ N(0, 4.87e-3): about 1 % of the pseudo-gradient
    elements fall below 2^-14, the binary16 subnormal range.  Full arrays, bitwise."""
    wl = synth.llama_150m()
    k = 8
    gpu, cpu = GpuSide(wl, k, True), CpuSide(wl, k, True)
    torch = gpu.torch
    sub = 0
    for r in range(k):
        key = synth.key(synth.STREAM_DELTA, r, 0)
        x = gpu.dl.theta[r]
        synth.device_fill_f32(x.data_ptr(), gpu.n_pad, key, 4.87e-3, gpu.kind.data_ptr(),
                              stream=torch.cuda.current_stream().cuda_stream)
        torch.sub(gpu.dl.theta0, x, out=x)                      # theta_r = theta0 - x
        xc = synth.host_fill_f32(cpu.n_pad, key, 4.87e-3, cpu.kind)
        cpu.o.workers[r].theta[:] = cpu.o.theta0 - xc
        d = cpu.o.theta0 - cpu.o.workers[r].theta
        real = cpu.kind != 0
        sub += int(((np.abs(d) < 2.0 ** -14) & real).sum())
        assert compare("theta[%d] in" % r, gpu.host(x), cpu.o.workers[r].theta, 0, 0) == 0
    frac = sub / (k * wl.n_params)
    assert 0.005 < frac < 0.02, frac
    gpu.dl.outer_step()
    cpu.o.outer_step()
    assert compare("theta0", gpu.host(gpu.dl.theta0), cpu.o.theta0, 0, 0) == 0
    assert compare("mom", gpu.host(gpu.dl.mom), cpu.o.b, 0, 0) == 0
    assert compare_state(gpu, cpu, 0, 0, what=("theta",)) == 0
    print("fp16 pseudo-gradient: %.3f %% of elements in the binary16 subnormal range" % (100 * frac))
    gpu.dl.close()
