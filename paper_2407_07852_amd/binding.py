"""ctypes binding of libdiloco_hip.so: the same entry points as include/diloco.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels; PyTorch is used
for device memory and the stream handle, nothing else.  There is no CPU fallback: a missing
library or a failing call raises.
"""
import ctypes as C
import os

import torch  # first: the HIP runtime it loads is the one the library binds to

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libdiloco_hip.so")

OK, ROUND_COMPLETE = 0, 1
ERR_INVALID_ARG, ERR_ALIGN, ERR_ARENA_TOO_SMALL, ERR_HIP, ERR_STATE = -1, -2, -3, -4, -5
F32, F16, BF16 = 0, 1, 2
BUF_THETA0, BUF_MOM, BUF_THETA, BUF_M, BUF_V, BUF_GRADS = 0, 1, 2, 3, 4, 5
LAYOUT_AUTO, LAYOUT_BUFFER_MAJOR, LAYOUT_WORKER_MAJOR = 0, 1, 2
MAX_WORKERS, TENSOR_ALIGN, TILE, MAX_GROUPS = 64, 64, 8192, 8

EXPORTS = ["diloco_query_layout", "diloco_init", "diloco_unscale_check", "diloco_inner_step",
           "diloco_outer_step", "diloco_get_buffer", "diloco_get_layout", "diloco_get_steps",
           "diloco_cast_f32_to_f16", "diloco_set_tuning", "diloco_last_error", "diloco_destroy",
           "diloco_set_param_groups", "diloco_lr_at", "diloco_cast_f32_to_bf16",
           "diloco_inner_step_noalloc", "diloco_outer_begin", "diloco_outer_finish"]


class Config(C.Structure):
    _fields_ = [("n_tensors", C.c_uint32), ("numel", C.POINTER(C.c_uint64)),
                ("k_workers", C.c_uint32), ("h_inner_steps", C.c_uint32),
                ("inner_lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("weight_decay", C.c_double),
                ("outer_lr", C.c_double), ("outer_momentum", C.c_double),
                ("pg_dtype", C.c_int32), ("pg_round_mean", C.c_int32), ("arena", C.c_void_p), ("arena_bytes", C.c_uint64),
                ("stream", C.c_void_p), ("layout_mode", C.c_int32), ("reserved", C.c_int32)]


class Layout(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("n_pad", "stride", "arena_bytes", "off_theta0",
                                          "off_mom", "off_theta", "off_m", "off_v", "off_grads",
                                          "slot")] + \
               [("layout_mode", C.c_int32), ("reserved", C.c_int32)]


class InnerCall(C.Structure):
    """diloco_inner_call: every pointer a device address."""
    _fields_ = [("theta", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p),
                ("stride", C.c_uint64), ("n_pad", C.c_uint64), ("k_workers", C.c_uint32),
                ("grad_dtype", C.c_int32), ("grads", C.c_void_p), ("grad_stride", C.c_uint64),
                ("inv_scale", C.c_float), ("found_inf", C.c_void_p), ("step_state", C.c_void_p),
                ("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double),
                ("eps", C.c_double), ("weight_decay", C.c_double), ("stream", C.c_void_p)]


STEP_STATE_BYTES = 24  # diloco_step_state: two doubles, two int32


class DilocoError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("diloco error %d: %s" % (code, msg))
        self.code = code


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s is missing: run `python __graft_entry__.py` (build()) first; "
                              "there is no fallback path" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        vp, u64, u32, i32 = C.c_void_p, C.c_uint64, C.c_uint32, C.c_int32
        L.diloco_query_layout.argtypes = [C.POINTER(Config), C.POINTER(Layout), C.POINTER(u64)]
        L.diloco_init.argtypes = [C.POINTER(Config), C.POINTER(vp), C.POINTER(vp)]
        L.diloco_unscale_check.argtypes = [vp, vp, u64, i32, C.c_float, vp]
        L.diloco_inner_step.argtypes = [vp, vp, u64, i32, C.c_double, vp]
        L.diloco_outer_step.argtypes = [vp]
        L.diloco_outer_begin.argtypes = [vp, vp, u64, vp]
        L.diloco_outer_finish.argtypes = [vp]
        L.diloco_get_buffer.argtypes = [vp, C.c_int, u32, C.POINTER(vp)]
        L.diloco_get_layout.argtypes = [vp, C.POINTER(Layout)]
        L.diloco_get_steps.argtypes = [vp, C.POINTER(u32)]
        L.diloco_cast_f32_to_f16.argtypes = [vp, vp, u64, vp]
        L.diloco_cast_f32_to_bf16.argtypes = [vp, vp, u64, vp]
        L.diloco_set_tuning.argtypes = [vp, C.c_char_p, C.c_int]
        L.diloco_last_error.argtypes = [vp]
        L.diloco_last_error.restype = C.c_char_p
        L.diloco_destroy.argtypes = [vp]
        L.diloco_set_param_groups.argtypes = [vp, C.POINTER(C.c_uint8), u32,
                                              C.POINTER(C.c_double), C.POINTER(C.c_double)]
        L.diloco_lr_at.argtypes = [u64, u64, u64, C.c_double, C.c_double]
        L.diloco_inner_step_noalloc.argtypes = [C.POINTER(InnerCall)]
        for n in EXPORTS:
            if n not in ("diloco_last_error", "diloco_lr_at"):
                getattr(L, n).restype = C.c_int
        L.diloco_lr_at.restype = C.c_double
        _lib = L
    return _lib


def _check(rc, ctx=None):
    if rc < 0:
        raise DilocoError(rc, lib().diloco_last_error(ctx).decode())
    return rc


def make_config(numel, k_workers, h_inner_steps=0, inner_lr=4e-4, beta1=0.9, beta2=0.999,
                eps=1e-8, weight_decay=0.1, outer_lr=0.7, outer_momentum=0.9, pg_dtype=F32,
                pg_round_mean=0, arena=None, arena_bytes=0, stream=None, layout_mode=0):
    arr = (C.c_uint64 * len(numel))(*[int(n) for n in numel])
    cfg = Config(len(numel), C.cast(arr, C.POINTER(C.c_uint64)), k_workers, h_inner_steps,
                 inner_lr, beta1, beta2, eps, weight_decay, outer_lr, outer_momentum, pg_dtype,
                 int(pg_round_mean), arena, arena_bytes, stream, int(layout_mode), 0)
    cfg._keep = arr
    return cfg


def diloco_query_layout(cfg):
    """-> (Layout, list of tensor offsets in elements)."""
    lay = Layout()
    offs = (C.c_uint64 * max(1, cfg.n_tensors))()
    _check(lib().diloco_query_layout(C.byref(cfg), C.byref(lay), offs))
    return lay, list(offs)[:cfg.n_tensors]


def diloco_init(cfg, init_params=None):
    """init_params: list of device addresses (ints) of FP32 tensors, or None.  -> ctx handle."""
    ctx = C.c_void_p()
    ptrs = None
    if init_params is not None:
        ptrs = (C.c_void_p * len(init_params))(*init_params)
    _check(lib().diloco_init(C.byref(cfg), ptrs, C.byref(ctx)))
    return ctx


def diloco_unscale_check(ctx, grads_ptr, grad_stride, grad_dtype, inv_scale, found_inf_ptr):
    return _check(lib().diloco_unscale_check(ctx, grads_ptr, grad_stride, grad_dtype, inv_scale,
                                             found_inf_ptr), ctx)


def diloco_inner_step(ctx, grads_ptr, grad_stride, grad_dtype, lr=-1.0, found_inf_ptr=None):
    return _check(lib().diloco_inner_step(ctx, grads_ptr, grad_stride, grad_dtype, lr,
                                          found_inf_ptr), ctx)


def diloco_outer_step(ctx):
    return _check(lib().diloco_outer_step(ctx), ctx)


def diloco_outer_begin(ctx, snapshot_ptr, snapshot_bytes, side_stream=None):
    return _check(lib().diloco_outer_begin(ctx, snapshot_ptr, snapshot_bytes, side_stream), ctx)


def diloco_outer_finish(ctx):
    return _check(lib().diloco_outer_finish(ctx), ctx)


def diloco_get_buffer(ctx, which, replica=0):
    p = C.c_void_p()
    _check(lib().diloco_get_buffer(ctx, which, replica, C.byref(p)), ctx)
    return p.value


def diloco_get_layout(ctx):
    lay = Layout()
    _check(lib().diloco_get_layout(ctx, C.byref(lay)), ctx)
    return lay


def diloco_get_steps(ctx, k):
    out = (C.c_uint32 * k)()
    _check(lib().diloco_get_steps(ctx, out), ctx)
    return list(out)


def diloco_cast_f32_to_f16(in_ptr, out_ptr, n, stream=None):
    return _check(lib().diloco_cast_f32_to_f16(in_ptr, out_ptr, n, stream))


def diloco_cast_f32_to_bf16(in_ptr, out_ptr, n, stream=None):
    return _check(lib().diloco_cast_f32_to_bf16(in_ptr, out_ptr, n, stream))


def diloco_set_tuning(ctx, name, value):
    return _check(lib().diloco_set_tuning(ctx, name.encode(), value), ctx)


def diloco_set_param_groups(ctx, group_of_tensor, lr_scale, weight_decay):
    """group_of_tensor: one group id per tensor; lr_scale / weight_decay: one value per group.
    Empty lists restore the single group of the config."""
    n = len(lr_scale)
    assert len(weight_decay) == n
    got = (C.c_uint8 * max(1, len(group_of_tensor)))(*group_of_tensor)
    ls = (C.c_double * max(1, n))(*lr_scale)
    wd = (C.c_double * max(1, n))(*weight_decay)
    return _check(lib().diloco_set_param_groups(ctx, got, n, ls, wd), ctx)


def diloco_lr_at(step, warmup_steps, total_steps, base_lr, final_ratio=1.0):
    return lib().diloco_lr_at(step, warmup_steps, total_steps, base_lr, final_ratio)


def diloco_inner_step_noalloc(**fields):
    """Fields of diloco_inner_call by name (device addresses as ints); allocates nothing on the
    device."""
    call = InnerCall(**fields)
    return _check(lib().diloco_inner_step_noalloc(C.byref(call)))


def diloco_last_error(ctx=None):
    return lib().diloco_last_error(ctx).decode()


def diloco_destroy(ctx):
    return _check(lib().diloco_destroy(ctx))


class DiLoCo:
    """Memory and stream plumbing around one context: allocates the arena with PyTorch,
    exposes the flat buffers as tensor views of it, forwards the steps to the library."""

    def __init__(self, numel, k_workers, device="cuda:0", init_params=None, fill_theta0=None,
                 arena=None, **hyper):
        """init_params: list of FP32 device tensors packed into theta0; or fill_theta0: a
        callable(theta0_view, layout, offsets) that writes the flat padded theta0 itself.
        arena: optional 1-D float32 device tensor to use as the arena (at least
        layout.arena_bytes / 4 elements, 256-byte aligned) instead of a new allocation."""
        self.device = torch.device(device)
        self.k = k_workers
        cfg = make_config(numel, k_workers, **hyper)
        self.layout, self.offsets = diloco_query_layout(cfg)
        self.numel = [int(n) for n in numel]
        with torch.cuda.device(self.device):
            if arena is None:
                arena = torch.empty(self.layout.arena_bytes // 4, dtype=torch.float32,
                                    device=self.device)
            assert arena.dtype == torch.float32 and arena.is_contiguous() and arena.dim() == 1
            assert arena.numel() * 4 >= self.layout.arena_bytes, "arena tensor too small"
            self.arena = arena
            self.stream = torch.cuda.current_stream(self.device)
            cfg.arena = self.arena.data_ptr()
            cfg.arena_bytes = self.layout.arena_bytes
            cfg.stream = self.stream.cuda_stream
            self.cfg = cfg
            L = self.layout
            self.theta0 = self._view(L.off_theta0, 1)[0]
            self.mom = self._view(L.off_mom, 1)[0]
            self.theta = self._view(L.off_theta, k_workers)
            self.m = self._view(L.off_m, k_workers)
            self.v = self._view(L.off_v, k_workers)
            ptrs = None
            if init_params is not None:
                ptrs = [t.data_ptr() for t in init_params]
            elif fill_theta0 is not None:
                fill_theta0(self.theta0, self.layout, self.offsets)
            self.ctx = diloco_init(cfg, ptrs)

    def _view(self, off_bytes, reps):
        L = self.layout
        flat = self.arena[off_bytes // 4: off_bytes // 4 + (reps - 1) * L.stride + L.n_pad]
        return torch.as_strided(flat, (reps, L.n_pad), (L.stride, 1))

    def grads_numel(self):
        """Elements of a dense [k][slot] buffer (a gradient buffer outside the arena, or the
        delayed outer step's snapshot)."""
        return (self.k - 1) * self.layout.slot + self.layout.n_pad

    def arena_grads(self, dtype=torch.float32):
        """The arena's own gradient slots as a [k][n_pad] view of the given dtype (float32 or
        float16): next to each worker's state in the worker-major layout, after the moments in
        the buffer-major one.  Not cleared."""
        L = self.layout
        if dtype == torch.float32:
            return torch.as_strided(self.arena, (self.k, L.n_pad), (L.stride, 1), L.off_grads // 4)
        assert dtype == torch.float16
        return torch.as_strided(self.arena.view(torch.float16), (self.k, L.n_pad),
                                (2 * L.stride, 1), L.off_grads // 2)

    def new_grads(self, dtype=torch.float32, out=None):
        """A zeroed gradient buffer [k][n_pad] of the given dtype.  By default the arena's own
        gradient slots (every call returns the same memory); with out, a 1-D device tensor of
        that dtype with at least grads_numel() elements, dense rows `slot` elements apart in
        it."""
        L = self.layout
        if out is None:
            return self.arena_grads(dtype).zero_()
        assert out.dtype == dtype and out.numel() >= self.grads_numel()
        flat = out[:self.grads_numel()].zero_()
        return torch.as_strided(flat, (self.k, L.n_pad), (L.slot, 1))

    def tensors(self, row, shapes):
        """Per-tensor views of one flat row (a worker's weights `theta[r]`, its gradients
        `new_grads()[r]`, `theta0`, a moment row): the parameter tensor list of the model, in
        place.  shapes: one shape per tensor of the list given at construction."""
        assert len(shapes) == len(self.numel)
        out = []
        for off, n, shape in zip(self.offsets, self.numel, shapes):
            view = row[off:off + n].view(*shape)
            assert view.numel() == n, "shape %r does not hold %d elements" % (tuple(shape), n)
            out.append(view)
        return out

    def new_flags(self):
        return torch.zeros(self.k, dtype=torch.int32, device=self.device)

    @staticmethod
    def _gdtype(g):
        return F16 if g.dtype == torch.float16 else F32

    def unscale_check(self, grads, inv_scale, flags):
        return diloco_unscale_check(self.ctx, grads.data_ptr(), grads.stride(0),
                                    self._gdtype(grads), inv_scale, flags.data_ptr())

    def inner_step(self, grads, lr=-1.0, flags=None):
        return diloco_inner_step(self.ctx, grads.data_ptr(), grads.stride(0), self._gdtype(grads),
                                 lr, None if flags is None else flags.data_ptr())

    def outer_step(self):
        return diloco_outer_step(self.ctx)

    def outer_begin(self, snapshot=None, side_stream=None):
        """Delayed outer step, first half.  snapshot: optional 1-D float32 device tensor of at
        least grads_numel() elements (allocated and kept on first use otherwise); side_stream:
        a torch stream for the update (a new default-priority stream otherwise)."""
        if snapshot is None:
            if getattr(self, "_snapshot", None) is None:
                self._snapshot = torch.empty(self.grads_numel(), dtype=torch.float32,
                                             device=self.device)
            snapshot = self._snapshot
        if side_stream is None:
            if getattr(self, "_side", None) is None:
                self._side = torch.cuda.Stream(device=self.device)
            side_stream = self._side
        self._snap_in_use, self._side_in_use = snapshot, side_stream
        return diloco_outer_begin(self.ctx, snapshot.data_ptr(), snapshot.numel() * 4,
                                  side_stream.cuda_stream)

    def outer_finish(self):
        return diloco_outer_finish(self.ctx)

    def steps(self):
        return diloco_get_steps(self.ctx, self.k)

    def set_param_groups(self, group_of_tensor, lr_scale, weight_decay):
        return diloco_set_param_groups(self.ctx, group_of_tensor, lr_scale, weight_decay)

    def set_tuning(self, **kw):
        for name, value in kw.items():
            diloco_set_tuning(self.ctx, name, int(value))

    def close(self):
        if getattr(self, "ctx", None) is not None:
            diloco_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
