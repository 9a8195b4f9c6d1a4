"""The entry point that allocates nothing (diloco_inner_step_noalloc, for callers that cannot
call hipMalloc) against diloco_inner_step on the same inputs: bit for bit, on two calls in a row,
the second with a smaller problem (fewer workers, fewer elements, one worker flagged)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

HP = dict(inner_lr=4e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1)


def fresh_state(torch, k):
    st = np.zeros(k, dtype=[("p1", "<f8"), ("p2", "<f8"), ("step", "<i4"), ("pad", "<i4")])
    st["p1"] = 1.0
    st["p2"] = 1.0
    return torch.from_numpy(st.view(np.uint8).copy()).cuda()


def one_case(torch, D, numel, k, steps, flagged, seed):
    """Reference: a context stepped with diloco_inner_step.  Candidate: the same buffers stepped
    with diloco_inner_step_noalloc.  Returns nothing; asserts bitwise equality after every step."""
    gen = torch.Generator(device="cuda").manual_seed(seed)
    ref = D.DiLoCo(numel, k, fill_theta0=lambda t, lay, off: t.normal_(0, 0.02, generator=gen), **HP)
    L = ref.layout
    # the candidate's own buffers, laid out like the arena's worker sections
    span = (k - 1) * L.slot + L.n_pad
    cand = [torch.zeros(span, dtype=torch.float32, device="cuda") for _ in range(3)]
    views = [torch.as_strided(c, (k, L.n_pad), (L.slot, 1)) for c in cand]
    views[0].copy_(ref.theta)
    state = fresh_state(torch, k)
    grads = ref.new_grads()
    flags = ref.new_flags()
    stream = torch.cuda.current_stream().cuda_stream
    for step in range(steps):
        grads.normal_(0, 1e-3, generator=gen)
        lr = 4e-4 * (step + 1) / steps
        use_flags = flagged is not None and step == 0
        if use_flags:
            grads[flagged, 7] = float("inf")
            ref.unscale_check(grads, 0.5, flags)
            assert flags.cpu().tolist() == [int(r == flagged) for r in range(k)]
        ref.inner_step(grads, lr=lr, flags=flags if use_flags else None)
        D.diloco_inner_step_noalloc(
            theta=cand[0].data_ptr(), m=cand[1].data_ptr(), v=cand[2].data_ptr(), stride=L.slot,
            n_pad=L.n_pad, k_workers=k, grad_dtype=D.F32, grads=grads.data_ptr(),
            grad_stride=grads.stride(0), inv_scale=0.5 if use_flags else 1.0,
            found_inf=flags.data_ptr() if use_flags else None, step_state=state.data_ptr(),
            lr=lr, beta1=HP["beta1"], beta2=HP["beta2"], eps=HP["eps"],
            weight_decay=HP["weight_decay"], stream=stream)
        for name, got, want in zip("theta m v".split(), views, (ref.theta, ref.m, ref.v)):
            assert torch.equal(got.view(torch.int32), want.view(torch.int32)), (name, step)
    st = state.cpu().numpy().view([("p1", "<f8"), ("p2", "<f8"), ("step", "<i4"), ("pad", "<i4")])
    assert st["step"].tolist() == ref.steps()
    ref.close()


def test_noalloc_inner_step_matches_the_context_path_twice_in_a_row():
    import torch
    import paper_2407_07852_amd as D
    # first call sequence: 5 workers, several tiles and a ragged tail
    one_case(torch, D, [300000, 70001, 64, 5], 5, steps=3, flagged=None, seed=1)
    # second, smaller: 2 workers (the static table still holds 5 entries of the first), one
    # worker flagged on its first step
    one_case(torch, D, [9000, 100], 2, steps=2, flagged=1, seed=2)


def test_noalloc_with_binary16_gradients_and_flags():
    """binary16 gradients under a loss scale through the entry point that allocates nothing: the
    flags come from a context's check of the same buffer; results equal the context path's."""
    import torch
    import paper_2407_07852_amd as D
    k, numel = 3, [20000, 513]
    gen = torch.Generator(device="cuda").manual_seed(9)
    ref = D.DiLoCo(numel, k, fill_theta0=lambda t, lay, off: t.normal_(0, 0.02, generator=gen), **HP)
    L = ref.layout
    span = (k - 1) * L.slot + L.n_pad
    cand = [torch.zeros(span, dtype=torch.float32, device="cuda") for _ in range(3)]
    views = [torch.as_strided(c, (k, L.n_pad), (L.slot, 1)) for c in cand]
    views[0].copy_(ref.theta)
    state = fresh_state(torch, k)
    g = ref.new_grads(torch.float16)
    flags = ref.new_flags()
    inv = 1.0 / 1024
    for step in range(2):
        g.copy_((torch.randn(g.shape, generator=gen, device="cuda") * 1.0).to(torch.float16))
        if step == 0:
            g[2, 100] = float("nan")
        ref.unscale_check(g, inv, flags)
        assert flags.cpu().tolist() == [0, 0, int(step == 0)]
        ref.inner_step(g, flags=flags)
        D.diloco_inner_step_noalloc(
            theta=cand[0].data_ptr(), m=cand[1].data_ptr(), v=cand[2].data_ptr(), stride=L.slot,
            n_pad=L.n_pad, k_workers=k, grad_dtype=D.F16, grads=g.data_ptr(), grad_stride=g.stride(0),
            inv_scale=inv, found_inf=flags.data_ptr(), step_state=state.data_ptr(),
            lr=HP["inner_lr"], beta1=HP["beta1"], beta2=HP["beta2"], eps=HP["eps"],
            weight_decay=HP["weight_decay"], stream=torch.cuda.current_stream().cuda_stream)
        for name, got, want in zip("theta m v".split(), views, (ref.theta, ref.m, ref.v)):
            assert torch.equal(got.view(torch.int32), want.view(torch.int32)), (name, step)
    ref.close()


def test_noalloc_rejects_what_it_cannot_hold():
    import torch
    import paper_2407_07852_amd as D
    buf = torch.zeros(8192 * 3, device="cuda")
    st = fresh_state(torch, 65)
    base = dict(theta=buf.data_ptr(), m=buf.data_ptr(), v=buf.data_ptr(), stride=8192, n_pad=8192,
                k_workers=65, grad_dtype=D.F32, grads=buf.data_ptr(), grad_stride=8192,
                inv_scale=1.0, found_inf=None, step_state=st.data_ptr(), lr=1e-3, beta1=0.9,
                beta2=0.999, eps=1e-8, weight_decay=0.0, stream=None)
    with pytest.raises(D.DilocoError) as e:
        D.diloco_inner_step_noalloc(**base)
    assert e.value.code == D.ERR_INVALID_ARG and "static step table" in str(e.value)
    with pytest.raises(D.DilocoError) as e:
        D.diloco_inner_step_noalloc(**dict(base, k_workers=1, n_pad=8000))
    assert e.value.code == D.ERR_INVALID_ARG
    with pytest.raises(D.DilocoError) as e:
        D.diloco_inner_step_noalloc(**dict(base, k_workers=1, theta=buf.data_ptr() + 4))
    assert e.value.code == D.ERR_ALIGN
    assert torch.count_nonzero(buf).item() == 0        # nothing was launched
