"""The inner step enqueues one kernel and no memset, so an even number of inner steps can be
captured into a HIP graph and replayed; every replay is checked against the oracle, with eager
work and synchronisations between the replays."""
import numpy as np
import pytest

import synth
from harness import CpuSide, GpuSide, compare, compare_state

pytestmark = pytest.mark.gpu


def test_captured_pair_of_inner_steps_replays_correctly():
    import torch
    wl = synth.tiny()
    k = 2
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        gpu = GpuSide(wl, k, True)          # the context borrows the capturing stream
        g = gpu.gen_grads(0)
        flags = gpu.dl.new_flags()
    side.synchronize()
    cpu = CpuSide(wl, k, True)
    gc = cpu.gen_grads(0)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        gpu.dl.unscale_check(g, 1.0, flags)
        gpu.dl.inner_step(g, flags=flags)
        gpu.dl.inner_step(g)
    torch.cuda.synchronize()
    # capture itself executes nothing
    assert gpu.dl.steps() == [0, 0]

    for replay in range(4):
        graph.replay()
        torch.cuda.synchronize()
        cpu.o.inner_step(gc, found_inf_flags=[0, 0])
        cpu.o.inner_step(gc)
        assert compare_state(gpu, cpu, 0, 0) == 0, "replay %d" % replay
        assert flags.cpu().tolist() == [0, 0]
        # eager work of the same context between replays
        with torch.cuda.stream(side):
            gpu.dl.outer_step()
        side.synchronize()
        cpu.o.outer_step()
        assert compare("theta0", gpu.host(gpu.dl.theta0), cpu.o.theta0, 0, 0) == 0
    assert gpu.dl.steps() == [8, 8]
    gpu.dl.close()
