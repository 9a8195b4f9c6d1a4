"""Shared test plumbing: builds the same seeded workload on both sides -- numpy arrays for the
CPU oracle, device buffers for the HIP library -- and compares them.  No optimizer arithmetic
lives here."""
import numpy as np

import oracle
import synth

PAPER_HP = dict(inner_lr=4e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1,
                outer_lr=0.7, outer_momentum=0.9)
W_SIGMA, G_SIGMA = 0.02, 1e-3

# tolerances of the contract: per step 1e-6 relative / 1e-7 absolute, 1e-5 relative after a round
STEP_RTOL, STEP_ATOL = 1e-6, 1e-7
ROUND_RTOL = 1e-5


def oracle_layout(wl):
    return oracle.plan_layout(wl.numel, 64, 8192)


class GpuSide:
    """The HIP library on the workload, inputs generated on the device."""

    def __init__(self, wl, k, pg_f16=False, hp=None, h=0, round_mean=False, layout_mode=0):
        """pg_f16: False (FP32), True (FP16) or an oracle.PG_* code (the library uses the same
        numbering).  layout_mode: the library's DILOCO_LAYOUT_* (0 = automatic)."""
        import torch
        import paper_2407_07852_amd as D
        self.torch, self.D, self.wl, self.k = torch, D, wl, k
        hp = dict(PAPER_HP if hp is None else hp)
        self.kind = None

        def fill(theta0, layout, offsets):
            self.kind_np = wl.kind_map(offsets, layout.n_pad)
            self.kind = torch.from_numpy(self.kind_np).to(theta0.device)
            synth.device_fill_f32(theta0.data_ptr(), layout.n_pad, synth.key(synth.STREAM_WEIGHTS),
                                  W_SIGMA, self.kind.data_ptr(), ones_as_one=True,
                                  stream=torch.cuda.current_stream().cuda_stream)

        self.dl = D.DiLoCo(wl.numel, k, fill_theta0=fill, h_inner_steps=h,
                           pg_dtype=oracle._pg_code(pg_f16), pg_round_mean=int(round_mean),
                           layout_mode=layout_mode, **hp)
        self.n_pad = self.dl.layout.n_pad
        self.grads = None

    def gen_grads(self, step, f16=False, inject_replica=None, inject_period=0, sigma=G_SIGMA):
        torch = self.torch
        dt = torch.float16 if f16 else torch.float32
        if self.grads is None or self.grads.dtype != dt:
            self.grads = self.dl.new_grads(dt)
        s = torch.cuda.current_stream().cuda_stream
        for r in range(self.k):
            key = synth.key(synth.STREAM_GRADS, r, step)
            if f16:
                inj = inject_replica is not None and r == inject_replica
                synth.device_fill_f16(self.grads[r].data_ptr(), self.n_pad, key,
                                      self.kind.data_ptr(),
                                      inject_key=synth.key(synth.STREAM_NONFINITE) if inj else 0,
                                      inject_period=inject_period if inj else 0, stream=s)
            else:
                synth.device_fill_f32(self.grads[r].data_ptr(), self.n_pad, key, sigma,
                                      self.kind.data_ptr(), stream=s)
        return self.grads

    def host(self, t):
        return t.detach().cpu().numpy()

    def set_groups(self, group_of_tensor, lr_scale, weight_decay):
        self.dl.set_param_groups(list(group_of_tensor), list(lr_scale), list(weight_decay))


class CpuSide:
    """The oracle on the same workload, inputs generated on the host."""

    def __init__(self, wl, k, pg_f16=False, hp=None, round_mean=False):
        hp = dict(PAPER_HP if hp is None else hp)
        self.wl, self.k = wl, k
        self.offsets, self.n_pad = oracle_layout(wl)
        self.kind = wl.kind_map(self.offsets, self.n_pad)
        theta0 = synth.host_fill_f32(self.n_pad, synth.key(synth.STREAM_WEIGHTS), W_SIGMA,
                                     self.kind, ones_as_one=True)
        self.o = oracle.DiLoCoOracle(theta0, k, hp["inner_lr"], hp["beta1"], hp["beta2"],
                                     hp["eps"], hp["weight_decay"], hp["outer_lr"],
                                     hp["outer_momentum"], pg_f16, round_mean)

    def set_groups(self, group_of_tensor, lr_scale, weight_decay):
        self.o.groups = oracle.ParamGroups(self.offsets, self.wl.numel, group_of_tensor, lr_scale,
                                           weight_decay)

    def gen_grads(self, step, f16=False, inject_replica=None, inject_period=0):
        out = []
        for r in range(self.k):
            key = synth.key(synth.STREAM_GRADS, r, step)
            if f16:
                inj = inject_replica is not None and r == inject_replica
                out.append(synth.host_fill_f16(
                    self.n_pad, key, self.kind,
                    inject_key=synth.key(synth.STREAM_NONFINITE) if inj else 0,
                    inject_period=inject_period if inj else 0))
            else:
                out.append(synth.host_fill_f32(self.n_pad, key, G_SIGMA, self.kind))
        return out


def compare(name, got, want, rtol, atol):
    """Element-by-element comparison; returns the number of bitwise mismatches."""
    got = np.asarray(got).reshape(-1)
    want = np.asarray(want).reshape(-1)
    assert got.shape == want.shape, (name, got.shape, want.shape)
    nan_w, nan_g = np.isnan(want), np.isnan(got)
    assert np.array_equal(nan_w, nan_g), name + ": NaN positions differ"
    ok = np.isclose(got, want, rtol=rtol, atol=atol, equal_nan=True)
    if not ok.all():
        i = int(np.argmin(ok))
        raise AssertionError("%s: %d of %d outside tolerance; first at %d: got %r want %r"
                             % (name, int((~ok).sum()), got.size, i, got[i], want[i]))
    return int((got.view(np.uint32) != want.view(np.uint32))[~nan_w].sum())


def compare_state(gpu, cpu, rtol=STEP_RTOL, atol=STEP_ATOL, what=("theta", "m", "v")):
    """Full-array comparison of every worker's state; returns total bitwise mismatches."""
    mism = 0
    for r in range(gpu.k):
        w = cpu.o.workers[r]
        for name in what:
            mism += compare("%s[%d]" % (name, r), gpu.host(getattr(gpu.dl, name)[r]),
                            getattr(w, name), rtol, atol)
    return mism


# ---------------------------------------------------------------- sampled parity (large sets)
def sample_indices(wl, offsets, n_pad, every=4099, edge=64):
    """First/last `edge` elements of every tensor, every pad element next to a tensor, every
    `every`-th flat index.  The path is elementwise, so the oracle run on these indices alone
    equals the oracle run on everything (pinned by test_elementwise_independence)."""
    parts = [np.arange(0, n_pad, every, dtype=np.int64)]
    for off, n in zip(offsets, wl.numel):
        off, n = int(off), int(n)
        parts.append(np.arange(off, off + min(edge, n)))
        parts.append(np.arange(off + max(0, n - edge), off + n))
        parts.append(np.arange(off + n, min(n_pad, (off + n + 63) // 64 * 64)))   # gap after it
    parts.append(np.arange(max(0, n_pad - edge), n_pad))
    return np.unique(np.concatenate(parts))


class SampledCpuSide:
    """The oracle restricted to a set of flat indices."""

    def __init__(self, wl, k, idx, pg_f16=False, hp=None):
        hp = dict(PAPER_HP if hp is None else hp)
        self.k, self.idx = k, np.ascontiguousarray(idx, dtype=np.uint64)
        offsets, n_pad = oracle_layout(wl)
        self.offsets, self.n_pad = offsets, n_pad
        # kind of each sampled index, without building the whole map
        ends = offsets + wl.numel
        t = np.searchsorted(offsets, self.idx, side="right") - 1
        inside = self.idx < ends[t]
        self.kind_at = np.where(inside, np.where(wl.is_vector[t], synth.KIND_ONE,
                                                 synth.KIND_NORMAL), synth.KIND_PAD).astype(np.uint8)
        theta0 = synth.host_gather_f32(self.idx, synth.key(synth.STREAM_WEIGHTS), W_SIGMA,
                                       self.kind_at, ones_as_one=True)
        self.o = oracle.DiLoCoOracle(theta0, k, hp["inner_lr"], hp["beta1"], hp["beta2"],
                                     hp["eps"], hp["weight_decay"], hp["outer_lr"],
                                     hp["outer_momentum"], pg_f16)

        self.tensor_at = t

    def set_groups(self, group_of_tensor, lr_scale, weight_decay):
        """Groups for a sampled index set: self.idx must have been ordered with
        order_by_group() so that each group's samples are one contiguous run."""
        g = np.asarray(group_of_tensor, dtype=np.uint8)[self.tensor_at]
        cuts = np.flatnonzero(np.diff(g.astype(np.int64))) + 1
        starts = np.concatenate([[0], cuts]).astype(np.uint64)
        lens = np.diff(np.concatenate([starts, [g.size]]).astype(np.int64)).astype(np.uint64)
        assert len(starts) <= len(lr_scale), "samples are not ordered by group"
        self.o.groups = oracle.ParamGroups(starts, lens, g[starts.astype(np.int64)], lr_scale,
                                           weight_decay)

    def gen_grads(self, step, sigma=G_SIGMA):
        return [synth.host_gather_f32(self.idx, synth.key(synth.STREAM_GRADS, r, step), sigma,
                                      self.kind_at) for r in range(self.k)]


def order_by_group(idx, offsets, group_of_tensor):
    """Reorders flat indices so that those of the same parameter group are contiguous (pads
    count with the tensor before them, as the library's 64-element chunks do)."""
    idx = np.asarray(idx, dtype=np.uint64)
    t = np.searchsorted(np.asarray(offsets, dtype=np.uint64), idx, side="right") - 1
    g = np.asarray(group_of_tensor)[t]
    return idx[np.argsort(g, kind="stable")]


def gather_gpu(gpu, t, idx_dev):
    """Rows of a [reps][n_pad] device view at the sampled flat indices, on the host."""
    return gpu.torch.index_select(t, t.dim() - 1, idx_dev).cpu().numpy()
