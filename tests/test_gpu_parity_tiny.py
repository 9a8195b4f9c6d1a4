"""GPU parity on the Tiny workload (3 tensors, 787 456 parameters, k=2, H=4): the HIP library
against the CPU oracle, full arrays after every inner step and after the outer step."""
import numpy as np
import pytest

import synth
from harness import CpuSide, GpuSide, compare, compare_state, STEP_RTOL, STEP_ATOL, ROUND_RTOL

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("layout_mode", [1, 2])   # buffer-major, worker-major
@pytest.mark.parametrize("pg_f16", [False, True])
def test_tiny_round(pg_f16, layout_mode):
    wl = synth.tiny()
    gpu, cpu = GpuSide(wl, 2, pg_f16, h=4, layout_mode=layout_mode), CpuSide(wl, 2, pg_f16)
    assert gpu.n_pad == cpu.n_pad and list(gpu.dl.offsets) == [int(o) for o in cpu.offsets]
    assert compare("theta0 init", gpu.host(gpu.dl.theta0), cpu.o.theta0, 0, 0) == 0
    assert compare_state(gpu, cpu, 0, 0) == 0
    for step in range(4):
        g = gpu.gen_grads(step)
        gc = cpu.gen_grads(step)
        for r in range(2):
            assert compare("grads", gpu.host(g[r]), gc[r], 0, 0) == 0
        rc = gpu.dl.inner_step(g)
        assert rc == (1 if step == 3 else 0)
        cpu.o.inner_step(gc)
        mism = compare_state(gpu, cpu)
        assert mism == 0, "inner step %d: %d elements differ in the last bit" % (step, mism)
    assert gpu.dl.steps() == [4, 4]
    gpu.dl.outer_step()
    cpu.o.outer_step()
    for name, got, want in (("theta0", gpu.dl.theta0, cpu.o.theta0), ("mom", gpu.dl.mom, cpu.o.b)):
        assert compare(name, gpu.host(got), want, ROUND_RTOL, STEP_ATOL) == 0
    assert compare_state(gpu, cpu, ROUND_RTOL, STEP_ATOL) == 0
    # every worker restarts from the new outer weights; pads are still zero
    th0 = gpu.host(gpu.dl.theta0)
    for r in range(2):
        assert np.array_equal(gpu.host(gpu.dl.theta[r]), th0)
    assert not th0[gpu.kind_np == 0].any()
    gpu.dl.close()
