"""C-ABI behaviour on the GPU: edge cases (k = 1, odd k, k above the unrolled kernels, tensors
of one element, no inner steps), packing from separate tensors, determinism, error paths."""
import numpy as np
import pytest

import oracle
import synth
from harness import CpuSide, GpuSide, compare, compare_state, PAPER_HP

pytestmark = pytest.mark.gpu


def _ragged(n):
    return synth.Workload("ragged%d" % n, [(s,) if j % 3 else (1, s)
                                           for j, s in enumerate(synth.ragged_sizes(n))])


@pytest.mark.parametrize("k,layout_mode", [(1, 0), (3, 0), (5, 0), (8, 0), (9, 0), (16, 0), (33, 0),
                                           (64, 0), (1, 2), (8, 2), (9, 2), (64, 2)])
@pytest.mark.parametrize("pg_f16", [False, True])
def test_round_for_various_k(k, layout_mode, pg_f16):
    wl = _ragged(40)
    gpu, cpu = GpuSide(wl, k, pg_f16, h=3, layout_mode=layout_mode), CpuSide(wl, k, pg_f16)
    for step in range(3):
        gpu.dl.inner_step(gpu.gen_grads(step))
        cpu.o.inner_step(cpu.gen_grads(step))
    assert compare_state(gpu, cpu) == 0
    gpu.dl.outer_step()
    cpu.o.outer_step()
    assert compare("theta0", gpu.host(gpu.dl.theta0), cpu.o.theta0, 0, 0) == 0
    assert compare("mom", gpu.host(gpu.dl.mom), cpu.o.b, 0, 0) == 0
    assert compare_state(gpu, cpu, 0, 0, what=("theta",)) == 0
    # a second round: the outer momentum now matters
    for step in range(3, 5):
        gpu.dl.inner_step(gpu.gen_grads(step))
        cpu.o.inner_step(cpu.gen_grads(step))
    gpu.dl.outer_step()
    cpu.o.outer_step()
    assert compare("theta0", gpu.host(gpu.dl.theta0), cpu.o.theta0, 0, 0) == 0
    assert compare("mom", gpu.host(gpu.dl.mom), cpu.o.b, 0, 0) == 0
    gpu.dl.close()


@pytest.mark.parametrize("k", [2, 8, 11])
@pytest.mark.parametrize("pg,round_mean", [(oracle.PG_BF16, False), (oracle.PG_BF16, True),
                                           (oracle.PG_F16, True), (oracle.PG_F32, True)])
def test_reduced_precision_pseudo_gradient_modes(k, pg, round_mean):
    """bfloat16 pseudo-gradients and the re-rounded average, two rounds, bitwise."""
    wl = _ragged(30)
    gpu = GpuSide(wl, k, pg, round_mean=round_mean)
    cpu = CpuSide(wl, k, pg, round_mean=round_mean)
    for rnd in range(2):
        for step in range(2 * rnd, 2 * rnd + 2):
            gpu.dl.inner_step(gpu.gen_grads(step))
            cpu.o.inner_step(cpu.gen_grads(step))
        gpu.dl.outer_step()
        cpu.o.outer_step()
        assert compare("theta0", gpu.host(gpu.dl.theta0), cpu.o.theta0, 0, 0) == 0
        assert compare("mom", gpu.host(gpu.dl.mom), cpu.o.b, 0, 0) == 0
    assert compare_state(gpu, cpu, 0, 0, what=("theta",)) == 0
    if pg != oracle.PG_F32 and round_mean:
        # the momentum buffer after the FIRST outer step was the rounded mean itself; after two
        # rounds theta0 moved by multiples of representable steps only in combination, so just
        # check the mode is not a no-op against the unrounded run
        ref = CpuSide(wl, k, pg, round_mean=False)
        for step in range(4):
            ref.o.inner_step(ref.gen_grads(step))
            if step % 2 == 1:
                ref.o.outer_step()
        assert not np.array_equal(ref.o.theta0, cpu.o.theta0)
    gpu.dl.close()


@pytest.mark.parametrize("tune", [dict(inner_block=256, outer_block=256),
                                  dict(inner_block=128, outer_block=64),
                                  dict(inner_block=64, outer_block=128, outer_anyk=1),
                                  dict(inner_waves=0, outer_waves=0, check_waves=0),
                                  dict(inner_waves=3, outer_waves=16, check_block=64, check_vec=8,
                                       check_persist=2)])
def test_launch_shapes_do_not_change_results(tune):
    wl = synth.tiny()
    gpu, cpu = GpuSide(wl, 4, True), CpuSide(wl, 4, True)
    gpu.dl.set_tuning(**tune)
    flags = gpu.dl.new_flags()
    for step in range(2):
        g = gpu.gen_grads(step)
        gpu.dl.unscale_check(g, 1.0, flags)
        assert flags.cpu().tolist() == [0] * 4
        gpu.dl.inner_step(g, flags=flags)
        cpu.o.inner_step(cpu.gen_grads(step))
    gpu.dl.outer_step()
    cpu.o.outer_step()
    assert compare_state(gpu, cpu, 0, 0) == 0
    assert compare("theta0", gpu.host(gpu.dl.theta0), cpu.o.theta0, 0, 0) == 0
    gpu.dl.close()


def test_outer_step_without_inner_steps():
    """H = 0: every pseudo-gradient is +0; with b = 0 the outer step is the identity, afterwards
    only the momentum acts."""
    wl = _ragged(10)
    gpu, cpu = GpuSide(wl, 4), CpuSide(wl, 4)
    before = gpu.host(gpu.dl.theta0).copy()
    gpu.dl.outer_step()
    assert np.array_equal(gpu.host(gpu.dl.theta0).view(np.uint32), before.view(np.uint32))
    assert not gpu.host(gpu.dl.mom).any()
    gpu.dl.inner_step(gpu.gen_grads(0)); cpu.o.inner_step(cpu.gen_grads(0))
    gpu.dl.outer_step(); cpu.o.outer_step()
    gpu.dl.outer_step(); cpu.o.outer_step()          # second one: momentum decay only
    assert compare("theta0", gpu.host(gpu.dl.theta0), cpu.o.theta0, 0, 0) == 0
    assert compare("mom", gpu.host(gpu.dl.mom), cpu.o.b, 0, 0) == 0
    gpu.dl.close()


def test_init_from_separate_tensors_packs_and_zeroes_pads():
    import torch
    import paper_2407_07852_amd as D
    numel = [1, 63, 64, 65, 1000, 7]
    params = [torch.full((n,), float(i + 1), device="cuda") for i, n in enumerate(numel)]
    lay, offs = D.diloco_query_layout(D.make_config(numel, 2))
    dl = D.DiLoCo(numel, 2, init_params=params)
    flat = dl.theta0.cpu().numpy()
    want = np.zeros(lay.n_pad, dtype=np.float32)
    for i, (o, n) in enumerate(zip(offs, numel)):
        want[o:o + n] = i + 1
    assert np.array_equal(flat, want)
    for t in (dl.theta[0], dl.theta[1]):
        assert np.array_equal(t.cpu().numpy(), want)
    assert not dl.m.cpu().numpy().any() and not dl.v.cpu().numpy().any() and not dl.mom.cpu().numpy().any()
    assert dl.steps() == [0, 0]
    dl.close()


def test_deterministic():
    wl = synth.tiny()
    outs = []
    for _ in range(2):
        gpu = GpuSide(wl, 3, True)
        for step in range(3):
            gpu.dl.inner_step(gpu.gen_grads(step))
        gpu.dl.outer_step()
        outs.append((gpu.host(gpu.dl.theta0).copy(), gpu.host(gpu.dl.mom).copy(),
                     gpu.host(gpu.dl.m).copy()))
        gpu.dl.close()
    for a, b in zip(*outs):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_lr_argument_and_zero_lr():
    wl = _ragged(5)
    gpu, cpu = GpuSide(wl, 2), CpuSide(wl, 2)
    g, gc = gpu.gen_grads(0), cpu.gen_grads(0)
    gpu.dl.inner_step(g, lr=1e-3); cpu.o.inner_step(gc, lr=1e-3)
    gpu.dl.inner_step(g, lr=0.0); cpu.o.inner_step(gc, lr=0.0)     # moments move, weights do not
    assert compare_state(gpu, cpu, 0, 0) == 0
    gpu.dl.close()


def test_layout_modes_give_identical_results_and_accessors_agree():
    """The same rounds (FP16 gradients with a skipped worker, FP16 pseudo-gradient, one plain and
    one delayed outer step) in the buffer-major and the worker-major arena: every buffer bitwise
    equal; the accessors return the addresses the layout describes."""
    import torch
    import paper_2407_07852_amd as D
    wl = _ragged(40)
    k = 5
    sides = [GpuSide(wl, k, True, layout_mode=mode) for mode in (D.LAYOUT_BUFFER_MAJOR,
                                                                 D.LAYOUT_WORKER_MAJOR)]
    for side, mode in zip(sides, (D.LAYOUT_BUFFER_MAJOR, D.LAYOUT_WORKER_MAJOR)):
        L = side.dl.layout
        assert L.layout_mode == mode
        base = side.dl.arena.data_ptr()
        for which, off in ((D.BUF_THETA, L.off_theta), (D.BUF_M, L.off_m), (D.BUF_V, L.off_v),
                           (D.BUF_GRADS, L.off_grads)):
            for r in (0, k - 1):
                assert D.diloco_get_buffer(side.dl.ctx, which, r) == base + off + r * L.stride * 4
        assert side.dl.arena_grads().data_ptr() == base + L.off_grads
        flags = side.dl.new_flags()
        for step in range(3):
            g = side.gen_grads(step, f16=True, inject_replica=2 if step == 1 else None,
                               inject_period=97)
            side.dl.unscale_check(g, 1.0 / 65536, flags)
            side.dl.inner_step(g, flags=flags)
        side.dl.outer_step()
        side.dl.inner_step(side.gen_grads(3))
        side.dl.outer_begin()
        side.dl.inner_step(side.gen_grads(4))
        side.dl.outer_finish()
        torch.cuda.synchronize()
    a, b = sides
    assert a.dl.steps() == b.dl.steps() == [5, 5, 4, 5, 5]
    for name in ("theta0", "mom", "theta", "m", "v"):
        x, y = getattr(a.dl, name), getattr(b.dl, name)
        assert torch.equal(x.contiguous().view(torch.int32), y.contiguous().view(torch.int32)), name
    for side in sides:
        side.dl.close()


def test_per_tensor_views_alias_the_flat_buffers():
    """A model's parameters and gradients as views of the arena: writing through the views is
    what the steps see, and what the steps write is what the views show."""
    import torch
    import paper_2407_07852_amd as D
    shapes = [(3, 50), (7,), (64, 2), (1,)]
    numel = [150, 7, 128, 1]
    k = 2
    init = [torch.full(sh, float(j + 1), device="cuda") for j, sh in enumerate(shapes)]
    dl = D.DiLoCo(numel, k, init_params=init, inner_lr=0.5, weight_decay=0.0)
    grads = dl.new_grads()
    for r in range(k):
        params = dl.tensors(dl.theta[r], shapes)
        gviews = dl.tensors(grads[r], shapes)
        for j, (p, g) in enumerate(zip(params, gviews)):
            assert p.shape == torch.Size(shapes[j]) and torch.all(p == j + 1)
            g.fill_(1.0 if r == 0 else -1.0)
    dl.inner_step(grads)
    torch.cuda.synchronize()
    # first AdamW step with |g| = 1: every element moves by lr against the gradient's sign
    for r, sign in ((0, -1.0), (1, 1.0)):
        for j, p in enumerate(dl.tensors(dl.theta[r], shapes)):
            assert torch.allclose(p, torch.full_like(p, j + 1 + sign * 0.5), atol=1e-6)
    # the pads between the tensors stayed zero
    flat = dl.theta[0]
    used = torch.zeros(dl.layout.n_pad, dtype=torch.bool, device="cuda")
    for off, n in zip(dl.offsets, numel):
        used[off:off + n] = True
    assert not flat[~used].any()
    dl.close()


def test_error_paths():
    import torch
    import paper_2407_07852_amd as D
    numel = [100, 5]
    dl = D.DiLoCo(numel, 2, fill_theta0=lambda t, lay, off: t.zero_())
    g = dl.new_grads()
    flags = dl.new_flags()
    n_pad = dl.layout.n_pad

    def code(fn):
        with pytest.raises(D.DilocoError) as e:
            fn()
        return e.value.code

    assert code(lambda: D.diloco_inner_step(dl.ctx, None, n_pad, D.F32)) == D.ERR_INVALID_ARG
    assert code(lambda: D.diloco_inner_step(dl.ctx, g.data_ptr(), n_pad, 7)) == D.ERR_INVALID_ARG
    assert code(lambda: D.diloco_inner_step(dl.ctx, g.data_ptr(), n_pad - 8, D.F32)) == D.ERR_INVALID_ARG
    assert code(lambda: D.diloco_inner_step(dl.ctx, g.data_ptr() + 4, n_pad, D.F32)) == D.ERR_ALIGN
    assert code(lambda: D.diloco_inner_step(dl.ctx, g.data_ptr(), n_pad + 4, D.F32)) == D.ERR_ALIGN
    # a gradient buffer whose k replicas cannot fit the allocation it lives in (a PyTorch
    # segment of the small-block pool is 2 MiB; two replicas at the arena's stride need more)
    small = torch.zeros(n_pad, device="cuda")
    assert code(lambda: D.diloco_inner_step(dl.ctx, small.data_ptr(), 1 << 24, D.F32)) == D.ERR_INVALID_ARG
    host = np.zeros(2 * n_pad, dtype=np.float32)
    assert code(lambda: D.diloco_inner_step(dl.ctx, host.ctypes.data, n_pad, D.F32)) == D.ERR_INVALID_ARG
    # flags without a preceding check of these gradients
    assert code(lambda: D.diloco_inner_step(dl.ctx, g.data_ptr(), g.stride(0), D.F32, -1.0,
                                            flags.data_ptr())) == D.ERR_STATE
    assert code(lambda: D.diloco_unscale_check(dl.ctx, g.data_ptr(), g.stride(0), D.F32, 0.0,
                                               flags.data_ptr())) == D.ERR_INVALID_ARG
    assert code(lambda: D.diloco_get_buffer(dl.ctx, D.BUF_THETA, 2)) == D.ERR_INVALID_ARG
    # binary16 gradients without the flags of a preceding check: refused, not stepped unscaled
    g16 = dl.new_grads(torch.float16)
    assert code(lambda: D.diloco_inner_step(dl.ctx, g16.data_ptr(), g16.stride(0), D.F16)) == D.ERR_STATE
    assert "unscale_check" in D.diloco_last_error(dl.ctx)
    assert code(lambda: D.diloco_set_tuning(dl.ctx, "inner_block", 96)) == D.ERR_INVALID_ARG
    assert code(lambda: D.diloco_set_tuning(dl.ctx, "no_such_knob", 1)) == D.ERR_INVALID_ARG
    assert "no_such_knob" in D.diloco_last_error(dl.ctx)
    # nothing was launched by any failed call
    assert dl.steps() == [0, 0]
    # arena too small / misaligned
    lay, _ = D.diloco_query_layout(D.make_config(numel, 2))
    arena = torch.zeros(lay.arena_bytes // 4, device="cuda")
    cfg = D.make_config(numel, 2, arena=arena.data_ptr(), arena_bytes=lay.arena_bytes - 4)
    assert code(lambda: D.diloco_init(cfg)) == D.ERR_ARENA_TOO_SMALL
    cfg = D.make_config(numel, 2, arena=arena.data_ptr() + 16, arena_bytes=lay.arena_bytes)
    assert code(lambda: D.diloco_init(cfg)) == D.ERR_ALIGN
    tiny_arena = torch.zeros(1024, device="cuda")
    cfg = D.make_config(numel, 2, arena=tiny_arena.data_ptr(), arena_bytes=lay.arena_bytes)
    assert code(lambda: D.diloco_init(cfg)) == D.ERR_INVALID_ARG   # does not fit its allocation
    dl.close()


def test_generator_twins_agree():
    """Host and device twins of the input generator produce the same bits."""
    import torch
    n = 1 << 20
    kind = (np.arange(n) % 7 != 0).astype(np.uint8) + (np.arange(n) % 11 == 0)
    kd = torch.from_numpy(kind).cuda()
    for sigma, ones in ((1e-3, False), (0.02, True)):
        key = synth.key(1, 3, 17)
        out = torch.empty(n, device="cuda")
        synth.device_fill_f32(out.data_ptr(), n, key, sigma, kd.data_ptr(), first=123, ones_as_one=ones,
                              stream=torch.cuda.current_stream().cuda_stream)
        want = synth.host_fill_f32(n, key, sigma, kind, first=123, ones_as_one=ones)
        assert np.array_equal(out.cpu().numpy().view(np.uint32), want.view(np.uint32))
    out = torch.empty(n, dtype=torch.int16, device="cuda")
    synth.device_fill_f16(out.data_ptr(), n, synth.key(1, 0, 0), kd.data_ptr(),
                          inject_key=synth.key(3), inject_period=1000,
                          stream=torch.cuda.current_stream().cuda_stream)
    want = synth.host_fill_f16(n, synth.key(1, 0, 0), kind, inject_key=synth.key(3), inject_period=1000)
    assert np.array_equal(out.cpu().numpy().view(np.uint16), want)
    assert ((want & 0x7C00) == 0x7C00).sum() > 500
