"""CPU-only checks of the product side: the shared library loads and exports every symbol the
header declares, the host-side layout planner agrees with the oracle's independent planner,
argument validation rejects bad problems without touching a GPU, and the input generator's
host twin matches a pure-Python restatement of its hash."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _D():
    import paper_2407_07852_amd as D
    return D


def test_library_exports_every_declared_symbol():
    D = _D()
    header = open(os.path.join(ROOT, "include", "diloco.h")).read()
    declared = sorted(set(re.findall(r"\b(diloco_[a-z0-9_]+)\s*\(", header)))
    assert len(declared) >= 12 and set(declared) == set(D.binding.EXPORTS)
    L = ctypes.CDLL(D.binding.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name


def test_header_constants_match_binding():
    D = _D()
    header = open(os.path.join(ROOT, "include", "diloco.h")).read()
    for name, val in (("DILOCO_MAX_WORKERS", D.MAX_WORKERS), ("DILOCO_TENSOR_ALIGN", D.TENSOR_ALIGN),
                      ("DILOCO_TILE", D.TILE)):
        assert int(re.search(name + r"\s+(\d+)", header).group(1)) == val
    for name in ("OK", "ROUND_COMPLETE", "ERR_INVALID_ARG", "ERR_ALIGN", "ERR_ARENA_TOO_SMALL",
                 "ERR_HIP", "ERR_STATE", "F32", "F16", "BF16", "BUF_THETA0", "BUF_MOM", "BUF_THETA",
                 "BUF_M", "BUF_V", "BUF_GRADS", "LAYOUT_AUTO", "LAYOUT_BUFFER_MAJOR",
                 "LAYOUT_WORKER_MAJOR"):
        assert int(re.search(r"DILOCO_" + name + r"\s*=\s*(-?\d+)", header).group(1)) == getattr(D, name)


def test_binding_structs_have_the_headers_sizes(tmp_path):
    """The ctypes mirrors of the header's structs against a C probe compiled from the header."""
    import subprocess
    D = _D()
    src = tmp_path / "probe.c"
    src.write_text('#include <stdio.h>\n#include "%s"\nint main(void) { printf("%%zu %%zu %%zu %%zu\\n", '
                   'sizeof(diloco_config), sizeof(diloco_layout), sizeof(diloco_inner_call), '
                   'sizeof(diloco_step_state)); return 0; }\n'
                   % os.path.join(ROOT, "include", "diloco.h"))
    exe = tmp_path / "probe"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", str(src), "-o", str(exe)], check=True)
    sizes = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True,
                                            text=True).stdout.split()]
    assert sizes == [ctypes.sizeof(D.Config), ctypes.sizeof(D.Layout), ctypes.sizeof(D.InnerCall),
                     D.STEP_STATE_BYTES]


def test_layout_agrees_with_oracle_planner():
    D = _D()
    rng = np.random.default_rng(0)
    cases = [synth.tiny().numel, synth.llama_150m().numel, synth.llama_1_1b().numel,
             synth.stress().numel, np.array([1], dtype=np.uint64)]
    for _ in range(50):
        cases.append(rng.integers(1, 20000, size=int(rng.integers(1, 60))).astype(np.uint64))
    for numel in cases:
        k = int(rng.integers(1, 9))
        for mode in (D.LAYOUT_AUTO, D.LAYOUT_BUFFER_MAJOR, D.LAYOUT_WORKER_MAJOR):
            lay, offs = D.diloco_query_layout(D.make_config(numel, k, layout_mode=mode))
            want_off, want_pad = oracle.plan_layout(numel, D.TENSOR_ALIGN, D.TILE)
            assert offs == [int(o) for o in want_off] and lay.n_pad == want_pad
            assert lay.slot >= lay.n_pad and (lay.slot * 4) % (2 << 20) == 0
            assert lay.slot - lay.n_pad < (2 << 20) // 4
            assert lay.layout_mode in (D.LAYOUT_BUFFER_MAJOR, D.LAYOUT_WORKER_MAJOR)
            if mode != D.LAYOUT_AUTO:
                assert lay.layout_mode == mode
            assert lay.stride == (4 * lay.slot if lay.layout_mode == D.LAYOUT_WORKER_MAJOR
                                  else lay.slot)
            # all 2 + 4k buffers: 256-byte aligned, pairwise disjoint, inside the arena
            starts = [lay.off_theta0, lay.off_mom]
            for off in (lay.off_theta, lay.off_m, lay.off_v, lay.off_grads):
                starts += [off + r * lay.stride * 4 for r in range(k)]
            assert all(s % 256 == 0 for s in starts)
            ordered = sorted(starts)
            assert len(set(ordered)) == 2 + 4 * k
            assert all(b - a >= lay.slot * 4 for a, b in zip(ordered, ordered[1:]))
            assert ordered[-1] + lay.slot * 4 <= lay.arena_bytes == (2 + 4 * k) * lay.slot * 4
            if lay.layout_mode == D.LAYOUT_WORKER_MAJOR:   # a worker's four buffers are adjacent
                assert (lay.off_m - lay.off_theta == lay.off_v - lay.off_m
                        == lay.off_grads - lay.off_v == lay.slot * 4)


def test_automatic_layout_choice_by_buffer_size():
    """Worker-major exactly when a slot holds 2 GiB or more (the 1.1B set: 4.1 GiB slots) or the
    arena exceeds 64 GiB."""
    D = _D()
    two_gib = (2 << 30) // 4   # elements
    for n, want in ((787456, D.LAYOUT_BUFFER_MAJOR), (234119168, D.LAYOUT_BUFFER_MAJOR),
                    (two_gib - 524288, D.LAYOUT_BUFFER_MAJOR), (two_gib - 524287, D.LAYOUT_WORKER_MAJOR),
                    (two_gib, D.LAYOUT_WORKER_MAJOR), (1100046336, D.LAYOUT_WORKER_MAJOR),
                    (1 << 32, D.LAYOUT_WORKER_MAJOR)):
        lay, _ = D.diloco_query_layout(D.make_config([n], 4))
        assert lay.layout_mode == want, (n, lay.layout_mode)
    # the 150M set (0.87 GiB slots): 34 slots at k = 8 and 70 at k = 17 fit 64 GiB, 74 at k = 18 do not
    for k, want in ((8, D.LAYOUT_BUFFER_MAJOR), (17, D.LAYOUT_BUFFER_MAJOR), (18, D.LAYOUT_WORKER_MAJOR),
                    (64, D.LAYOUT_WORKER_MAJOR)):
        lay, _ = D.diloco_query_layout(D.make_config([234119168], k))
        assert lay.layout_mode == want and (lay.arena_bytes > (64 << 30)) == (want == D.LAYOUT_WORKER_MAJOR)
    with pytest.raises(D.DilocoError):
        D.diloco_query_layout(D.make_config([4], 2, layout_mode=3))


def test_known_workload_sizes():
    assert synth.tiny().n_params == 787456
    assert synth.llama_150m().n_params == 234119168 and len(synth.llama_150m().shapes) == 109
    assert synth.llama_1_1b().n_params == 1100046336 and len(synth.llama_1_1b().shapes) == 200
    st = synth.stress()
    assert len(st.shapes) == 2109 and all(1 <= int(n) <= 4096 for n in st.numel[109:])


def test_bad_problems_are_rejected_on_the_host():
    D = _D()

    def code(cfg, init=False):
        with pytest.raises(D.DilocoError) as e:
            D.diloco_init(cfg) if init else D.diloco_query_layout(cfg)
        return e.value.code

    assert code(D.make_config([], 2)) == D.ERR_INVALID_ARG
    assert code(D.make_config([4, 0, 3], 2)) == D.ERR_INVALID_ARG
    assert code(D.make_config([4], 0)) == D.ERR_INVALID_ARG
    assert code(D.make_config([1 << 33, 1], 1)) == D.ERR_INVALID_ARG
    lay, _ = D.diloco_query_layout(D.make_config([1 << 33], 1))      # the largest accepted size
    assert lay.n_pad == 1 << 33
    assert code(D.make_config([4], D.MAX_WORKERS + 1)) == D.ERR_INVALID_ARG
    assert "k_workers" in D.diloco_last_error()
    for bad in (dict(beta1=1.0), dict(beta2=-0.1), dict(eps=0.0), dict(inner_lr=-1.0),
                dict(inner_lr=float("nan")), dict(weight_decay=-1.0), dict(outer_momentum=1.0),
                dict(outer_lr=float("inf")), dict(pg_dtype=5)):
        assert code(D.make_config([4], 2, arena=256, arena_bytes=1 << 30, **bad), init=True) \
            == D.ERR_INVALID_ARG, bad
    assert code(D.make_config([4], 2, arena=None, arena_bytes=1 << 30), init=True) == D.ERR_INVALID_ARG
    assert code(D.make_config([4], 2, arena=264, arena_bytes=1 << 30), init=True) == D.ERR_ALIGN
    assert code(D.make_config([4], 2, arena=256, arena_bytes=16), init=True) == D.ERR_ARENA_TOO_SMALL


def test_no_gpu_means_a_loud_error_not_a_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    D = _D()
    with pytest.raises(D.DilocoError) as e:
        D.diloco_init(D.make_config([4], 2, arena=256, arena_bytes=1 << 30))
    assert e.value.code == D.ERR_HIP


def test_noalloc_entry_point_validates_on_the_host_before_touching_the_gpu():
    """Argument errors of diloco_inner_step_noalloc are found on the host (the pointers are never
    dereferenced); valid arguments without a GPU end in a HIP error, not in a fallback."""
    import torch
    D = _D()
    base = dict(theta=4096, m=8192, v=12288, stride=8192, n_pad=8192, k_workers=2, grad_dtype=D.F32,
                grads=16384, grad_stride=8192, inv_scale=1.0, found_inf=None, step_state=256,
                lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, stream=None)

    def code(**kw):
        with pytest.raises(D.DilocoError) as e:
            D.diloco_inner_step_noalloc(**dict(base, **kw))
        return e.value.code, str(e.value)

    c, msg = code(k_workers=65)
    assert c == D.ERR_INVALID_ARG and "static step table" in msg
    assert code(k_workers=0)[0] == D.ERR_INVALID_ARG
    assert code(theta=None)[0] == D.ERR_INVALID_ARG
    assert code(n_pad=8191)[0] == D.ERR_INVALID_ARG
    assert code(stride=4096)[0] == D.ERR_INVALID_ARG
    assert code(grad_dtype=D.BF16)[0] == D.ERR_INVALID_ARG
    assert code(theta=4100)[0] == D.ERR_ALIGN
    assert code(grad_stride=8196)[0] == D.ERR_ALIGN
    assert code(beta1=1.0)[0] == D.ERR_INVALID_ARG
    assert code(eps=0.0)[0] == D.ERR_INVALID_ARG
    assert code(inv_scale=0.0)[0] == D.ERR_INVALID_ARG
    assert code(grad_dtype=D.F16)[0] == D.ERR_STATE          # binary16 gradients need flags
    if not torch.cuda.is_available():
        assert code()[0] == D.ERR_HIP


def _mix64(z):
    M = (1 << 64) - 1
    z ^= z >> 30
    z = (z * 0xBF58476D1CE4E5B9) & M
    z ^= z >> 27
    z = (z * 0x94D049BB133111EB) & M
    z ^= z >> 31
    return z


def test_generator_host_twin_against_python():
    M = (1 << 64) - 1
    seed, stream, replica, step = synth.SEED, 1, 5, 499
    k = _mix64((seed + 0x9E3779B97F4A7C15) & M)
    for x in (stream, replica, step):
        k = _mix64((k + x) & M)
    assert synth.key(stream, replica, step) == k
    c = np.float32(1e-3 / synth.IRWIN_HALL_SD)
    idx = np.array([0, 1, 2, 1000, 234119167, (1 << 33) + 5], dtype=np.uint64)
    got = synth.host_gather_f32(idx, k, 1e-3)
    got16 = synth.host_gather_f16(idx, k)
    for j, i in enumerate(idx.tolist()):
        u = _mix64((k + i * 0x9E3779B97F4A7C15) & M)
        s = sum((u >> sh) & 0xFFFF for sh in (0, 16, 32, 48)) - 131070
        assert got[j] == np.float32(s) * c
        assert np.array([got16[j]], dtype=np.uint16).view(np.float16)[0] == (s >> 6) / 8.0
    x = synth.host_fill_f32(1 << 20, k, 1e-3)
    assert abs(float(x.std()) - 1e-3) < 2e-5 and abs(float(x.mean())) < 5e-6
    assert np.array_equal(synth.host_fill_f32(1000, k, 1e-3, first=77), synth.host_gather_f32(
        np.arange(77, 1077, dtype=np.uint64), k, 1e-3))


def test_lr_schedule_matches_oracle():
    D = _D()
    for warm, total, ratio in ((1000, 0, 1.0), (1000, 88000, 0.1), (0, 100, 0.0), (5, 5, 0.5)):
        for step in list(range(0, 20)) + [999, 1000, 1001, 44000, 87999, 88000, 10 ** 7]:
            assert D.diloco_lr_at(step, warm, total, 4e-4, ratio) == oracle.lr_at(step, warm, total,
                                                                                  4e-4, ratio)
    assert np.isnan(D.diloco_lr_at(1, 10, 0, -1.0, 1.0))
    assert np.isnan(D.diloco_lr_at(1, 10, 0, float("inf"), 1.0))


def test_workload_shapes_follow_the_papers_model_table():
    """Layers / hidden size / vocabulary of the synthetic tensor lists are the ones the paper's
    model-configuration table prints (tests/golden/model_shapes.txt)."""
    rows = {}
    with open(os.path.join(ROOT, "tests", "golden", "model_shapes.txt")) as f:
        for line in f:
            line = line.split("#", 1)[0].split()
            if len(line) == 6:
                rows[line[0]] = [int(x) for x in line[1:]]
    for name, wl in (("llama_150m", synth.llama_150m()), ("llama_1_1b", synth.llama_1_1b())):
        layers, hidden, heads, kv_size, vocab = rows[name]
        norms = [s for s in wl.shapes if len(s) == 1]
        assert len(norms) == 2 * layers and all(s == (hidden,) for s in norms)
        assert wl.shapes[-1] == (vocab, hidden)
        square = [s for s in wl.shapes if s == (hidden, hidden)]
        assert len(square) >= 2 * layers                   # q and o projections
        assert hidden == heads * kv_size                   # head size as printed
        kv = [s for s in wl.shapes if len(s) == 2 and s[1] == hidden and s[0] % kv_size == 0]
        assert kv


def test_product_sources_never_reach_into_the_oracle():
    """The HIP path and its binding share nothing with the oracle: no import, include or path."""
    pkg = os.path.join(ROOT, "paper_2407_07852_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, fn)
    for fn in ("diloco_oracle.cpp", "__init__.py", "build.py"):
        text = open(os.path.join(ROOT, "oracle", fn)).read()
        assert "paper_2407_07852_amd" not in text and "csrc" not in text and "hip/" not in text
    header = open(os.path.join(ROOT, "include", "diloco.h")).read()
    assert "oracle" not in header.lower()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "single-GPU" in (r.stderr + r.stdout)
