"""ctypes front end of the CPU oracle (oracle/diloco_oracle.cpp).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg import this
package.  It imports nothing from the GPU package, and the GPU package never imports it.
All arrays are C-contiguous numpy arrays that the C++ side updates in place.
"""
import ctypes as C

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(_build.build())
        sz, f32, f64, u16, i32, u32, u64, vp = (C.c_size_t, C.c_float, C.c_double, C.c_uint16,
                                                C.c_int32, C.c_uint32, C.c_uint64, C.c_void_p)
        sig = {
            "oracle_f32_to_f16_rne": (u16, [f32]),
            "oracle_f16_to_f32": (f32, [u16]),
            "oracle_cast_f32_to_f16": (None, [vp, vp, sz]),
            "oracle_cast_pattern_range": (None, [u32, sz, vp]),
            "oracle_cast_f16_to_f32": (None, [vp, vp, sz]),
            "oracle_adamw_step_f32": (None, [vp, vp, vp, vp, sz, f64, f64, f64, f64, f64, vp, vp]),
            "oracle_adamw_step_f64": (None, [vp, vp, vp, vp, sz, f64, f64, f64, f64, f64, vp, vp]),
            "oracle_adamw_step_groups_f32": (None, [vp, vp, vp, vp, u32, vp, vp, vp, vp, vp, f64, f64,
                                                    f64, f64, vp, vp]),
            "oracle_adamw_step_groups_f64": (None, [vp, vp, vp, vp, u32, vp, vp, vp, vp, vp, f64, f64,
                                                    f64, f64, vp, vp]),
            "oracle_lr_at": (f64, [u64, u64, u64, f64, f64]),
            "oracle_unscale_f16": (None, [vp, f32, vp, sz]),
            "oracle_unscale_f32": (None, [vp, f32, vp, sz]),
            "oracle_found_inf_f16": (i32, [vp, sz]),
            "oracle_found_inf_f32": (i32, [vp, sz]),
            "oracle_pseudo_grad_f32": (None, [vp, vp, vp, sz]),
            "oracle_pseudo_grad_f64": (None, [vp, vp, vp, sz]),
            "oracle_round_through_f16": (None, [vp, sz]),
            "oracle_replica_mean_f32": (None, [vp, sz, sz, vp]),
            "oracle_replica_mean_f64": (None, [vp, sz, sz, vp]),
            "oracle_nesterov_step_f32": (None, [vp, vp, vp, sz, f64, f64]),
            "oracle_nesterov_step_f64": (None, [vp, vp, vp, sz, f64, f64]),
            "oracle_outer_step_f32": (None, [vp, vp, vp, sz, sz, f64, f64, i32, i32, vp, vp]),
            "oracle_outer_update_from_snapshot_f32": (None, [vp, vp, vp, sz, sz, f64, f64, i32, i32,
                                                             vp, vp]),
            "oracle_merge_delayed_f32": (None, [vp, vp, vp, sz, sz]),
            "oracle_merge_delayed_f64": (None, [vp, vp, vp, sz, sz]),
            "oracle_f32_to_bf16_rne": (u16, [f32]),
            "oracle_bf16_to_f32": (f32, [u16]),
            "oracle_cast_f32_to_bf16": (None, [vp, vp, sz]),
            "oracle_cast_pattern_range_bf16": (None, [u32, sz, vp]),
            "oracle_round_through_bf16": (None, [vp, sz]),
            "oracle_plan_layout": (u64, [vp, u32, u64, u64, vp]),
            "oracle_num_threads": (C.c_int, []),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        _lib = L
    return _lib


def _p(a, dtype):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], \
        (type(a), getattr(a, "dtype", None), dtype)
    return a.ctypes.data


# ---- binary16 casts ---------------------------------------------------------
def f32_to_f16_bits(x):
    """RNE cast of a float32 array to binary16 bit patterns (uint16)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().oracle_cast_f32_to_f16(_p(x, np.float32), _p(out, np.uint16), x.size)
    return out


def cast_pattern_range(first, n):
    """binary16 codes of the n consecutive float32 bit patterns starting at `first`."""
    out = np.empty(n, dtype=np.uint16)
    lib().oracle_cast_pattern_range(int(first) & 0xFFFFFFFF, n, _p(out, np.uint16))
    return out


def f32_to_bf16_bits(x):
    """RNE cast of a float32 array to bfloat16 bit patterns (uint16)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.uint16)
    lib().oracle_cast_f32_to_bf16(_p(x, np.float32), _p(out, np.uint16), x.size)
    return out


def cast_pattern_range_bf16(first, n):
    out = np.empty(n, dtype=np.uint16)
    lib().oracle_cast_pattern_range_bf16(int(first) & 0xFFFFFFFF, n, _p(out, np.uint16))
    return out


def bf16_bits_to_f32(h):
    h = np.ascontiguousarray(h, dtype=np.uint16)
    return np.array([lib().oracle_bf16_to_f32(int(x)) for x in h.reshape(-1)],
                    dtype=np.float32).reshape(h.shape)


PG_F32, PG_F16, PG_BF16 = 0, 1, 2


def _pg_code(pg):
    """Accepts the historical bool (False = FP32, True = FP16) or a PG_* code."""
    return {False: PG_F32, True: PG_F16}.get(pg, pg) if isinstance(pg, bool) else int(pg)


def f16_bits_to_f32(h):
    h = np.ascontiguousarray(h, dtype=np.uint16)
    out = np.empty(h.shape, dtype=np.float32)
    lib().oracle_cast_f16_to_f32(_p(h, np.uint16), _p(out, np.float32), h.size)
    return out


# ---- inner step -------------------------------------------------------------
class AdamWState:
    """One worker's AdamW state: weights, moments, running products beta^t, step count."""

    def __init__(self, theta, dtype=np.float32):
        self.dtype = np.dtype(dtype)
        self.theta = np.array(theta, dtype=self.dtype, order="C").reshape(-1)
        self.m = np.zeros_like(self.theta)
        self.v = np.zeros_like(self.theta)
        self.p1 = C.c_double(1.0)
        self.p2 = C.c_double(1.0)
        self.t = 0


def adamw_step(st, g, lr, beta1, beta2, eps, weight_decay):
    """One AdamW step of one worker, in place on st (float32 or float64 state)."""
    g = np.ascontiguousarray(g, dtype=st.dtype).reshape(-1)
    assert g.size == st.theta.size
    fn = lib().oracle_adamw_step_f32 if st.dtype == np.float32 else lib().oracle_adamw_step_f64
    fn(_p(st.theta, st.dtype), _p(st.m, st.dtype), _p(st.v, st.dtype), _p(g, st.dtype),
       st.theta.size, lr, beta1, beta2, eps, weight_decay, C.addressof(st.p1), C.addressof(st.p2))
    st.t += 1


class ParamGroups:
    """Per-tensor parameter groups over a flat layout: tensor t occupies
    [offsets[t], offsets[t]+numel[t]) and belongs to group group_of_tensor[t]."""

    def __init__(self, offsets, numel, group_of_tensor, lr_scale, weight_decay):
        self.offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
        self.numel = np.ascontiguousarray(numel, dtype=np.uint64)
        self.group_of_tensor = np.ascontiguousarray(group_of_tensor, dtype=np.uint8)
        self.lr_scale = np.ascontiguousarray(lr_scale, dtype=np.float64)
        self.weight_decay = np.ascontiguousarray(weight_decay, dtype=np.float64)
        assert self.offsets.size == self.numel.size == self.group_of_tensor.size
        assert self.lr_scale.size == self.weight_decay.size > int(self.group_of_tensor.max())


def adamw_step_groups(st, g, groups, lr, beta1, beta2, eps):
    """One AdamW step of one worker with per-tensor parameter groups, in place on st."""
    g = np.ascontiguousarray(g, dtype=st.dtype).reshape(-1)
    assert g.size == st.theta.size
    fn = (lib().oracle_adamw_step_groups_f32 if st.dtype == np.float32
          else lib().oracle_adamw_step_groups_f64)
    G = groups
    fn(_p(st.theta, st.dtype), _p(st.m, st.dtype), _p(st.v, st.dtype), _p(g, st.dtype),
       G.numel.size, _p(G.offsets, np.uint64), _p(G.numel, np.uint64),
       _p(G.group_of_tensor, np.uint8), _p(G.lr_scale, np.float64),
       _p(G.weight_decay, np.float64), lr, beta1, beta2, eps,
       C.addressof(st.p1), C.addressof(st.p2))
    st.t += 1


def lr_at(step, warmup_steps, total_steps, base_lr, final_ratio=1.0):
    return float(lib().oracle_lr_at(step, warmup_steps, total_steps, base_lr, final_ratio))


def unscale_f16(g16_bits, inv_scale):
    """widen(binary16 gradient) * inv_scale, as float32."""
    g16_bits = np.ascontiguousarray(g16_bits, dtype=np.uint16).reshape(-1)
    out = np.empty(g16_bits.size, dtype=np.float32)
    lib().oracle_unscale_f16(_p(g16_bits, np.uint16), inv_scale, _p(out, np.float32), out.size)
    return out


def unscale_f32(g, inv_scale):
    """float32 gradient * inv_scale, as float32."""
    g = np.ascontiguousarray(g, dtype=np.float32).reshape(-1)
    out = np.empty(g.size, dtype=np.float32)
    lib().oracle_unscale_f32(_p(g, np.float32), inv_scale, _p(out, np.float32), out.size)
    return out


def found_inf(g):
    """1 if any element of g (float32 array, or uint16 array of binary16 codes) is inf/NaN."""
    g = np.ascontiguousarray(g).reshape(-1)
    if g.dtype == np.uint16:
        return int(lib().oracle_found_inf_f16(_p(g, np.uint16), g.size))
    return int(lib().oracle_found_inf_f32(_p(g, np.float32), g.size))


# ---- outer step -------------------------------------------------------------
def pseudo_grad(theta0, theta_r):
    dt = theta0.dtype
    out = np.empty_like(theta0)
    fn = lib().oracle_pseudo_grad_f32 if dt == np.float32 else lib().oracle_pseudo_grad_f64
    fn(_p(theta0, dt), _p(theta_r, dt), _p(out, dt), theta0.size)
    return out


def round_through_f16(delta):
    lib().oracle_round_through_f16(_p(delta, np.float32), delta.size)
    return delta


def replica_mean(delta):
    """delta: [k][n] -> mean over k (sequential sum, then divide by k)."""
    k, n = delta.shape
    dt = delta.dtype
    out = np.empty(n, dtype=dt)
    fn = lib().oracle_replica_mean_f32 if dt == np.float32 else lib().oracle_replica_mean_f64
    fn(_p(delta, dt), k, n, _p(out, dt))
    return out


def nesterov_step(theta0, b, grad, lr, mu):
    dt = theta0.dtype
    fn = lib().oracle_nesterov_step_f32 if dt == np.float32 else lib().oracle_nesterov_step_f64
    fn(_p(theta0, dt), _p(b, dt), _p(grad, dt), theta0.size, lr, mu)


def outer_step(theta0, b, theta, outer_lr, mu, pg_f16, scratch=None, round_mean=False):
    """Whole outer step, float32, in place.  theta is [k][n].  pg_f16: False/True or a PG_* code
    (type the pseudo-gradients are rounded through); round_mean: also round the average.
    scratch: optional preallocated (delta[k][n], mean[n]) work arrays."""
    k, n = theta.shape
    d, mean = scratch if scratch is not None else (np.empty((k, n), dtype=np.float32),
                                                   np.empty(n, dtype=np.float32))
    lib().oracle_outer_step_f32(_p(theta0, np.float32), _p(b, np.float32), _p(theta, np.float32),
                                k, n, outer_lr, mu, _pg_code(pg_f16), 1 if round_mean else 0,
                                _p(d, np.float32), _p(mean, np.float32))
    return mean


# ---- delayed application of the outer step --------------------------------------
def outer_update_from_snapshot(theta0, b, snap, outer_lr, mu, pg=False, round_mean=False):
    """Outer update computed from the workers' snapshotted weights snap [k][n]: theta0 and b
    are updated in place, no worker is reset.  float32."""
    k, n = snap.shape
    d = np.empty((k, n), dtype=np.float32)
    mean = np.empty(n, dtype=np.float32)
    lib().oracle_outer_update_from_snapshot_f32(
        _p(theta0, np.float32), _p(b, np.float32), _p(snap, np.float32), k, n, outer_lr, mu,
        _pg_code(pg), 1 if round_mean else 0, _p(d, np.float32), _p(mean, np.float32))
    return mean


def merge_delayed(theta0, snap, theta):
    """theta_r <- theta0 - (snap_r - theta_r) in place for every worker; theta, snap [k][n]."""
    k, n = theta.shape
    dt = theta.dtype
    fn = lib().oracle_merge_delayed_f32 if dt == np.float32 else lib().oracle_merge_delayed_f64
    fn(_p(theta0, dt), _p(snap, dt), _p(theta, dt), k, n)


# ---- layout -------------------------------------------------------------------
def plan_layout(numel, align, tile):
    numel = np.ascontiguousarray(numel, dtype=np.uint64)
    off = np.empty(numel.size, dtype=np.uint64)
    n_pad = lib().oracle_plan_layout(_p(numel, np.uint64), numel.size, align, tile,
                                     _p(off, np.uint64))
    return off, int(n_pad)


def num_threads():
    return int(lib().oracle_num_threads())


# ---- the whole method over k workers (plain driver around the steps above) ----
class DiLoCoOracle:
    """k workers, each with its own AdamW state, plus the outer weights theta0 and the
    outer momentum buffer b.  float32 throughout.  A worker whose found_inf flag is set
    skips its inner step entirely (weights, moments and step count stay as they are)."""

    def __init__(self, theta_init, k, inner_lr, beta1, beta2, eps, weight_decay, outer_lr,
                 outer_momentum, pg_f16=False, round_mean=False):
        theta_init = np.ascontiguousarray(theta_init, dtype=np.float32).reshape(-1)
        self.k = k
        self.hp = (inner_lr, beta1, beta2, eps, weight_decay)
        self.outer_lr, self.mu, self.pg_f16 = outer_lr, outer_momentum, pg_f16
        self.round_mean = round_mean
        self.theta0 = theta_init.copy()
        self.b = np.zeros_like(self.theta0)
        self.workers = [AdamWState(theta_init) for _ in range(k)]
        self.groups = None   # optional ParamGroups

    def inner_step(self, grads, found_inf_flags=None, lr=None, inv_scale=None):
        """grads[r]: float32 array, or uint16 binary16 codes; inv_scale (the gradient scaler's
        unscale factor) is required with binary16 codes and optional with float32."""
        lr0, b1, b2, eps, wd = self.hp
        for r, st in enumerate(self.workers):
            if found_inf_flags is not None and found_inf_flags[r]:
                continue
            g = grads[r]
            if g.dtype == np.uint16:
                g = unscale_f16(g, inv_scale)
            elif inv_scale is not None:
                g = unscale_f32(g, inv_scale)
            if self.groups is not None:
                adamw_step_groups(st, g, self.groups, lr0 if lr is None else lr, b1, b2, eps)
            else:
                adamw_step(st, g, lr0 if lr is None else lr, b1, b2, eps, wd)

    def outer_begin(self):
        """Round boundary of the delayed outer step: snapshot every worker's weights and compute
        the outer update from the snapshots (theta0 and b change, the workers do not)."""
        self.snap = np.stack([st.theta for st in self.workers])
        return outer_update_from_snapshot(self.theta0, self.b, self.snap, self.outer_lr, self.mu,
                                          self.pg_f16, self.round_mean)

    def outer_finish(self):
        """Delayed application: every worker moves to the new outer weights, keeping what it did
        since the snapshot."""
        theta = np.stack([st.theta for st in self.workers])
        merge_delayed(self.theta0, self.snap, theta)
        for r, st in enumerate(self.workers):
            st.theta[:] = theta[r]
        self.snap = None

    def outer_step(self):
        theta = np.stack([st.theta for st in self.workers])
        mean = outer_step(self.theta0, self.b, theta, self.outer_lr, self.mu, self.pg_f16,
                          round_mean=self.round_mean)
        for r, st in enumerate(self.workers):
            st.theta[:] = theta[r]
        return mean
