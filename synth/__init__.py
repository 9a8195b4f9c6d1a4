"""Seeded synthetic inputs for the tests and the benchmark: workload shape lists and the
counter-based value generator (host twin for numpy arrays, device twin for GPU buffers).

This package serves both the CPU oracle's harness and the GPU path's harness and holds none
of the optimizer's arithmetic.  It imports neither of them.

The workloads stand in for the Llama models the paper trains on C4 (Appendix A, Table 3 gives
layers / hidden size / heads / vocabulary; FFN widths and KV-head counts are this build's
workload definition).  The optimizer path never looks at values except for the inf / NaN /
subnormal classes, so seeded bell-shaped numbers of the stated standard deviations replace
trained weights and real gradients.
"""
import ctypes as C
import os
import subprocess

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
HOST_LIB = os.path.join(HERE, "libsynth_host.so")
DEVICE_LIB = os.path.join(HERE, "libsynth_device.so")

SEED = 20240707
STREAM_WEIGHTS, STREAM_GRADS, STREAM_DELTA, STREAM_NONFINITE, STREAM_RAGGED = 0, 1, 2, 3, 4
IRWIN_HALL_SD = 37837.22723513447

KIND_PAD, KIND_NORMAL, KIND_ONE = 0, 1, 2

HIPCC_FLAGS = ["-O2", "-fPIC", "-shared", "--offload-arch=gfx950", "-ffp-contract=off",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# ------------------------------------------------------------------ building
def _stale(out, srcs):
    return (not os.path.exists(out)) or any(os.path.getmtime(s) > os.path.getmtime(out) for s in srcs)


def build_host(force=False):
    srcs = [os.path.join(HERE, "synth_host.c"), os.path.join(HERE, "synth_mix.h")]
    if force or _stale(HOST_LIB, srcs):
        tmp = HOST_LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                        srcs[0], "-o", tmp], check=True)
        os.replace(tmp, HOST_LIB)
    return HOST_LIB


def build_device(force=False):
    srcs = [os.path.join(HERE, "synth_device.hip"), os.path.join(HERE, "synth_mix.h")]
    if force or _stale(DEVICE_LIB, srcs):
        tmp = DEVICE_LIB + ".tmp.%d" % os.getpid()
        subprocess.run(["hipcc", *HIPCC_FLAGS, srcs[0], "-o", tmp], check=True)
        os.replace(tmp, DEVICE_LIB)
    return DEVICE_LIB


_host = None
_device = None


def host():
    global _host
    if _host is None:
        L = C.CDLL(build_host())
        vp, u64, sz, f32, i, u32 = C.c_void_p, C.c_uint64, C.c_size_t, C.c_float, C.c_int, C.c_uint32
        L.synth_host_fill_f32.argtypes = [vp, vp, u64, sz, u64, f32, i]
        L.synth_host_gather_f32.argtypes = [vp, vp, vp, sz, u64, f32, i]
        L.synth_host_fill_f16.argtypes = [vp, vp, u64, sz, u64, u64, u32]
        L.synth_host_gather_f16.argtypes = [vp, vp, vp, sz, u64, u64, u32]
        L.synth_host_key.argtypes = [u64, u64, u64, u64]
        L.synth_host_key.restype = u64
        L.synth_host_hash.argtypes = [u64, u64]
        L.synth_host_hash.restype = u64
        for n in ("synth_host_fill_f32", "synth_host_gather_f32", "synth_host_fill_f16",
                  "synth_host_gather_f16"):
            getattr(L, n).restype = None
        _host = L
    return _host


def device():
    """The device twin.  Import torch first so that the HIP runtime already in the process
    is the one this library binds to."""
    global _device
    if _device is None:
        import torch  # noqa: F401
        if not os.path.exists(DEVICE_LIB):
            build_device()
        L = C.CDLL(DEVICE_LIB)
        vp, u64, sz, f32, i, u32 = C.c_void_p, C.c_uint64, C.c_size_t, C.c_float, C.c_int, C.c_uint32
        L.synth_device_fill_f32.argtypes = [vp, vp, u64, sz, u64, f32, i, vp]
        L.synth_device_fill_f32.restype = i
        L.synth_device_fill_f16.argtypes = [vp, vp, u64, sz, u64, u64, u32, vp]
        L.synth_device_fill_f16.restype = i
        L.synth_device_copy.argtypes = [vp, vp, sz, vp]
        L.synth_device_copy.restype = i
        L.synth_device_stream_pattern.argtypes = [C.POINTER(vp), i, i, sz, i, vp, vp]
        L.synth_device_stream_pattern.restype = i
        _device = L
    return _device


# ------------------------------------------------------------------ workloads
class Workload:
    """A parameter tensor list: numel per tensor and whether a tensor is a norm vector
    (weights start at 1.0) or a matrix (weights ~ N(0, 0.02))."""

    def __init__(self, name, shapes):
        self.name = name
        self.shapes = [tuple(s) for s in shapes]
        self.numel = np.array([int(np.prod(s)) for s in self.shapes], dtype=np.uint64)
        self.is_vector = np.array([len(s) == 1 for s in self.shapes])
        self.n_params = int(self.numel.sum())

    def kind_map(self, offsets, n_pad):
        """uint8 [n_pad]: 0 pad, 1 matrix element, 2 norm-vector element."""
        kind = np.zeros(n_pad, dtype=np.uint8)
        for off, n, vec in zip(offsets, self.numel, self.is_vector):
            kind[int(off):int(off) + int(n)] = KIND_ONE if vec else KIND_NORMAL
        return kind


def tiny():
    return Workload("tiny", [(256, 1024), (1024, 512), (1024,)])


def llama(name, layers, hidden, ffn, kv_dim, vocab, tied):
    shapes = []
    for _ in range(layers):
        shapes += [(hidden, hidden), (kv_dim, hidden), (kv_dim, hidden), (hidden, hidden),   # q k v o
                   (ffn, hidden), (ffn, hidden), (hidden, ffn),                             # gate up down
                   (hidden,), (hidden,)]                                                     # 2 RMSNorm
    shapes.append((vocab, hidden))                                                           # embedding
    if not tied:
        shapes.append((vocab, hidden))                                                       # LM head
    return Workload(name, shapes)


def llama_150m():
    """12 layers, hidden 1024, FFN 4096, full-width K/V, vocabulary 32000, tied embeddings:
    109 tensors, 234 119 168 parameters (the paper's "150M" label, with this FFN width)."""
    return llama("llama150m", 12, 1024, 4096, 1024, 32000, True)


def llama_1_1b():
    """22 layers, hidden 2048, 32 heads / 4 KV heads of size 64 (K/V projections [256, 2048]),
    FFN 5632, untied embeddings: 200 tensors, 1 100 046 336 parameters."""
    return llama("llama1.1b", 22, 2048, 5632, 256, 32000, False)


def ragged_sizes(count=2000, seed=SEED):
    key = int(host().synth_host_key(seed, STREAM_RAGGED, 0, 0))
    return [1 + int(host().synth_host_hash(key, j)) % 4096 for j in range(count)]


def stress():
    """The 150M set followed by 2000 tiny tensors of 1..4096 elements (ragged multi-tensor)."""
    base = llama_150m()
    return Workload("llama150m+ragged2000", base.shapes + [(n,) if j % 2 else (1, n)
                                                           for j, n in enumerate(ragged_sizes())])


WORKLOADS = {"tiny": tiny, "llama150m": llama_150m, "llama1.1b": llama_1_1b, "stress": stress}


# ------------------------------------------------------------------ values
def key(stream, replica=0, step=0, seed=SEED):
    return int(host().synth_host_key(seed, stream, replica, step))


def scale_for(sigma):
    """The float32 multiplier c that gives the bell-shaped values standard deviation sigma."""
    return float(np.float32(sigma / IRWIN_HALL_SD))


def _np_ptr(a):
    return None if a is None else a.ctypes.data


def host_fill_f32(n, k, sigma, kind=None, first=0, ones_as_one=False):
    out = np.empty(n, dtype=np.float32)
    host().synth_host_fill_f32(out.ctypes.data, _np_ptr(kind), first, n, k, scale_for(sigma),
                               int(ones_as_one))
    return out


def host_gather_f32(idx, k, sigma, kind_at=None, ones_as_one=False):
    idx = np.ascontiguousarray(idx, dtype=np.uint64)
    out = np.empty(idx.size, dtype=np.float32)
    host().synth_host_gather_f32(out.ctypes.data, _np_ptr(kind_at), idx.ctypes.data, idx.size, k,
                                 scale_for(sigma), int(ones_as_one))
    return out


def host_fill_f16(n, k, kind=None, first=0, inject_key=0, inject_period=0):
    out = np.empty(n, dtype=np.uint16)
    host().synth_host_fill_f16(out.ctypes.data, _np_ptr(kind), first, n, k, inject_key,
                               inject_period)
    return out


def host_gather_f16(idx, k, kind_at=None, inject_key=0, inject_period=0):
    idx = np.ascontiguousarray(idx, dtype=np.uint64)
    out = np.empty(idx.size, dtype=np.uint16)
    host().synth_host_gather_f16(out.ctypes.data, _np_ptr(kind_at), idx.ctypes.data, idx.size, k,
                                 inject_key, inject_period)
    return out


def device_fill_f32(ptr, n, k, sigma, kind_ptr=None, first=0, ones_as_one=False, stream=None):
    """ptr / kind_ptr: device addresses (ints); stream: a hipStream_t handle (int) or None."""
    rc = device().synth_device_fill_f32(ptr, kind_ptr, first, n, k, scale_for(sigma),
                                        int(ones_as_one), stream)
    if rc != 0:
        raise RuntimeError("synth_device_fill_f32: hip error %d" % rc)


def device_fill_f16(ptr, n, k, kind_ptr=None, first=0, inject_key=0, inject_period=0, stream=None):
    rc = device().synth_device_fill_f16(ptr, kind_ptr, first, n, k, inject_key, inject_period,
                                        stream)
    if rc != 0:
        raise RuntimeError("synth_device_fill_f16: hip error %d" % rc)


def device_copy(dst_ptr, src_ptr, n_bytes, stream=None):
    """Plain device-to-device copy kernel of known size (reference for counter calibration)."""
    rc = device().synth_device_copy(dst_ptr, src_ptr, n_bytes, stream)
    if rc != 0:
        raise RuntimeError("synth_device_copy: hip error %d" % rc)


def device_stream_pattern(buf_ptrs, nr, nw, n_bytes, waves_per_cu, sink_ptr, stream=None):
    """One launch of the streaming reference pattern: nr read + nw write streams of n_bytes each
    (device addresses in buf_ptrs), residency capped at waves_per_cu waves per CU."""
    arr = (C.c_void_p * len(buf_ptrs))(*buf_ptrs)
    rc = device().synth_device_stream_pattern(arr, nr, nw, n_bytes, waves_per_cu, sink_ptr, stream)
    if rc != 0:
        raise RuntimeError("synth_device_stream_pattern: error %d" % rc)
