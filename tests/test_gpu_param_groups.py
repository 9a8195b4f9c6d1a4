"""Per-tensor parameter groups (weight-decay exclusion, per-group learning-rate scale) and the
learning-rate schedule in the inner step: HIP library against the oracle."""
import numpy as np
import pytest

import oracle
import synth
from harness import (CpuSide, GpuSide, SampledCpuSide, compare, compare_state, gather_gpu,
                     order_by_group, sample_indices, ROUND_RTOL, STEP_ATOL)

pytestmark = pytest.mark.gpu


def _no_decay_groups(wl, embed_last=1):
    """group 0: matrices (decay 0.1); group 1: norm vectors (no decay); group 2: embeddings
    (no decay, half learning rate)."""
    grp = [1 if v else 0 for v in wl.is_vector]
    for t in range(len(grp) - embed_last, len(grp)):
        grp[t] = 2
    return grp, [1.0, 1.0, 0.5], [0.1, 0.0, 0.0]


def test_tiny_with_groups_and_schedule():
    import paper_2407_07852_amd as D
    wl = synth.tiny()
    grp, lr_scale, wd = [0, 2, 1], [1.0, 3.0, 0.25], [0.1, 0.0, 0.7]
    gpu, cpu = GpuSide(wl, 2), CpuSide(wl, 2)
    gpu.set_groups(grp, lr_scale, wd)
    cpu.set_groups(grp, lr_scale, wd)
    for step in range(4):
        lr = D.diloco_lr_at(step + 1, 3, 10, 4e-4, 0.1)
        assert lr == oracle.lr_at(step + 1, 3, 10, 4e-4, 0.1)
        gpu.dl.inner_step(gpu.gen_grads(step), lr=lr)
        cpu.o.inner_step(cpu.gen_grads(step), lr=lr)
        assert compare_state(gpu, cpu, 0, 0) == 0
    # back to the single group of the config
    gpu.set_groups([], [], [])
    cpu.o.groups = None
    gpu.dl.inner_step(gpu.gen_grads(4))
    cpu.o.inner_step(cpu.gen_grads(4))
    assert compare_state(gpu, cpu, 0, 0) == 0
    gpu.dl.close()


@pytest.mark.parametrize("f16_grads,layout_mode", [(False, 1), (True, 1), (True, 2)])
def test_ragged_tensors_many_groups(f16_grads, layout_mode):
    """40 tiny tensors (1..4096 elements, several inside one 256-element tile), 8 groups."""
    wl = synth.Workload("ragged40", [(s,) if j % 3 else (1, s)
                                     for j, s in enumerate(synth.ragged_sizes(40))])
    grp = [(7 * j + 3) % 8 for j in range(40)]
    lr_scale = [1.0, 0.5, 2.0, 0.0, 1.5, 0.25, 3.0, 1.0]
    wd = [0.1, 0.0, 0.3, 0.5, 0.0, 1.0, 0.01, 0.2]
    gpu, cpu = GpuSide(wl, 3, layout_mode=layout_mode), CpuSide(wl, 3)
    gpu.set_groups(grp, lr_scale, wd)
    cpu.set_groups(grp, lr_scale, wd)
    flags = gpu.dl.new_flags()
    for step in range(3):
        g = gpu.gen_grads(step, f16=f16_grads)
        gc = cpu.gen_grads(step, f16=f16_grads)
        if f16_grads:
            gpu.dl.unscale_check(g, 1.0 / 65536, flags)
            gpu.dl.inner_step(g, flags=flags)
            cpu.o.inner_step(gc, found_inf_flags=[0, 0, 0], inv_scale=1.0 / 65536)
        else:
            gpu.dl.inner_step(g)
            cpu.o.inner_step(gc)
    assert compare_state(gpu, cpu, 0, 0) == 0
    gpu.dl.outer_step()
    cpu.o.outer_step()
    assert compare("theta0", gpu.host(gpu.dl.theta0), cpu.o.theta0, 0, 0) == 0
    gpu.dl.close()


@pytest.mark.timeout(600)
def test_150m_k8_groups_sampled():
    """150M set, k=8: norm vectors and the embedding exempt from decay, 20 inner steps on a
    warm-up schedule, then the outer step; sampled elements."""
    import paper_2407_07852_amd as D
    wl = synth.llama_150m()
    k, H = 8, 20
    grp, lr_scale, wd = _no_decay_groups(wl)
    gpu = GpuSide(wl, k, False, h=H)
    gpu.set_groups(grp, lr_scale, wd)
    idx = order_by_group(sample_indices(wl, np.asarray(gpu.dl.offsets, dtype=np.uint64), gpu.n_pad),
                         gpu.dl.offsets, grp)
    cpu = SampledCpuSide(wl, k, idx)
    cpu.set_groups(grp, lr_scale, wd)
    idx_dev = gpu.torch.from_numpy(idx.astype(np.int64)).to("cuda")
    for step in range(H):
        lr = D.diloco_lr_at(step, 10, 0, 4e-4, 1.0)
        gpu.dl.inner_step(gpu.gen_grads(step), lr=lr)
        cpu.o.inner_step(cpu.gen_grads(step), lr=lr)
    th, m, v = (gather_gpu(gpu, t, idx_dev) for t in (gpu.dl.theta, gpu.dl.m, gpu.dl.v))
    mism = 0
    for r in range(k):
        w = cpu.o.workers[r]
        mism += compare("theta[%d]" % r, th[r], w.theta, ROUND_RTOL, STEP_ATOL)
        mism += compare("m[%d]" % r, m[r], w.m, ROUND_RTOL, 1e-12)
        mism += compare("v[%d]" % r, v[r], w.v, ROUND_RTOL, 1e-15)
    assert mism == 0
    # decay really differs between groups: a norm vector element stayed closer to 1
    gpu.dl.outer_step()
    cpu.o.outer_step()
    assert compare("theta0", gather_gpu(gpu, gpu.dl.theta0, idx_dev), cpu.o.theta0, ROUND_RTOL,
                   STEP_ATOL) == 0
    gpu.dl.close()


def test_group_errors():
    import paper_2407_07852_amd as D
    dl = D.DiLoCo([10, 20], 2, fill_theta0=lambda t, lay, off: t.zero_())
    for bad in (([0, 2], [1.0, 1.0], [0.0, 0.0]),                 # group id out of range
                ([0, 1], [1.0, -1.0], [0.0, 0.0]),                # negative scale
                ([0, 1], [1.0, 1.0], [0.0, float("nan")]),
                ([0] * 2, [1.0] * 9, [0.0] * 9)):                 # too many groups
        with pytest.raises(D.DilocoError) as e:
            dl.set_param_groups(*bad)
        assert e.value.code == D.ERR_INVALID_ARG
    dl.close()
