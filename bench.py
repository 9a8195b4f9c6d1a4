#!/usr/bin/env python3
"""Benchmark of the DiLoCo optimizer hot path on one MI355X.

One "step" is one DiLoCo round over synthetic inputs already resident in HBM: H fused AdamW
inner steps of all k workers, then one fused outer step (pseudo-gradient, optional FP16
rounding, mean over k, Nesterov SGD, broadcast).  The headline value is the algorithmic HBM
traffic of the round divided by its wall time.  Per-kernel durations come from HIP events on
the stream the kernels are launched on.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload llama150m|llama1.1b]
                    [--h H] [--k K] [--pg f32|f16] [--no-also] [--no-cpu]

Prints ONE JSON line.  Everything on this path is single-GPU: --gpus above 1 is refused.
"""
import argparse
import json
import os
import sys
import time

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E peak


def inner_bytes(n, k, g16=False):
    """Algorithmic bytes of one inner step: per element and worker, read theta, m, v (12 B) and
    the gradient (4 B, or 2 B in binary16), write theta, m, v (12 B)."""
    return (26 if g16 else 28) * n * k


def outer_bytes(n, k):
    """Algorithmic bytes of one outer step: read theta0, mom and k worker weights, write theta0,
    mom and k worker weights: (16 + 8k) B per element."""
    return (16 + 8 * k) * n


def median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def run_workload(name, k, H, pg_f16, rounds, warmup, torch, D, synth, groups=False):
    wl = synth.WORKLOADS[name]()
    n = wl.n_params
    stream = torch.cuda.current_stream()

    def fill(theta0, layout, offsets):
        kind = torch.from_numpy(wl.kind_map(offsets, layout.n_pad)).to(theta0.device)
        synth.device_fill_f32(theta0.data_ptr(), layout.n_pad, synth.key(synth.STREAM_WEIGHTS),
                              0.02, kind.data_ptr(), ones_as_one=True, stream=stream.cuda_stream)
        fill.kind = kind

    dl = D.DiLoCo(wl.numel, k, fill_theta0=fill, h_inner_steps=H,
                  pg_dtype=D.F16 if pg_f16 else D.F32)
    if groups:
        # matrices decay 0.1; norm vectors and the embedding / LM head: no decay, and the
        # embeddings at half the learning rate
        grp = [1 if v else 0 for v in wl.is_vector]
        grp[-1] = 2
        if name == "llama1.1b":
            grp[-2] = 2
        dl.set_param_groups(grp, [1.0, 1.0, 0.5], [0.1, 0.0, 0.0])
    grads = dl.new_grads()
    for r in range(k):  # one seeded gradient set ~N(0, 1e-3), resident for the whole run
        synth.device_fill_f32(grads[r].data_ptr(), dl.layout.n_pad,
                              synth.key(synth.STREAM_GRADS, r, 0), 1e-3, fill.kind.data_ptr(),
                              stream=stream.cuda_stream)
    del fill.kind
    torch.cuda.synchronize()

    ev = lambda: torch.cuda.Event(enable_timing=True)  # noqa: E731

    def one_round(timed):
        marks = (ev(), ev(), ev()) if timed else None
        if timed:
            marks[0].record(stream)
        rc = 0
        for _ in range(H):
            rc = dl.inner_step(grads)
        assert rc == D.ROUND_COMPLETE
        if timed:
            marks[1].record(stream)
        dl.outer_step()
        if timed:
            marks[2].record(stream)
        return marks

    for _ in range(warmup):
        one_round(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    marks = [one_round(True) for _ in range(rounds)]
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    inner_ms = [m[0].elapsed_time(m[1]) / H for m in marks]
    outer_ms = [m[1].elapsed_time(m[2]) for m in marks]
    assert dl.steps() == [H * (rounds + warmup)] * k
    finite = bool(torch.isfinite(dl.theta0).all())
    dl.close()
    del dl, grads
    torch.cuda.empty_cache()

    ib, ob = inner_bytes(n, k), outer_bytes(n, k)
    im, om = sum(inner_ms) / len(inner_ms), sum(outer_ms) / len(outer_ms)
    round_ms = wall_ms / rounds
    return {
        "workload": name, "n_params": n, "k": k, "H": H, "pg_dtype": "f16" if pg_f16 else "f32",
        "finite": finite,
        "round_ms": round_ms,
        "round_GBps": (H * ib + ob) / round_ms / 1e6,
        "inner": {"ms": im, "ms_median_round": median(inner_ms), "bytes": ib,
                  "GBps": ib / im / 1e6, "frac_of_peak": ib / im / 1e6 / HBM_PEAK_GBS,
                  "launches_timed": H * rounds},
        "outer": {"ms": om, "ms_median": median(outer_ms), "bytes": ob,
                  "GBps": ob / om / 1e6, "frac_of_peak": ob / om / 1e6 / HBM_PEAK_GBS,
                  "launches_timed": rounds},
    }


def quick_measure(name, k, pg_dtype, round_mean, n_inner, n_outer, torch, D, synth):
    """Short timing of both kernels for one (workload, k, pseudo-gradient mode): n_inner inner
    launches and n_outer outer launches after two warm-up launches of each."""
    wl = synth.WORKLOADS[name]()
    n = wl.n_params
    stream = torch.cuda.current_stream()
    dl = D.DiLoCo(wl.numel, k, fill_theta0=lambda t, lay, off: t.normal_(0, 0.02),
                  pg_dtype=pg_dtype, pg_round_mean=round_mean)
    g = dl.new_grads()
    g.normal_(0, 1e-3)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    for _ in range(2):
        dl.inner_step(g)
        dl.outer_step()
    torch.cuda.synchronize()
    ev[0].record(stream)
    for _ in range(n_inner):
        dl.inner_step(g)
    ev[1].record(stream)
    for _ in range(n_outer):
        dl.outer_step()
    ev[2].record(stream)
    torch.cuda.synchronize()
    im, om = ev[0].elapsed_time(ev[1]) / n_inner, ev[1].elapsed_time(ev[2]) / n_outer
    dl.close()
    del dl, g
    torch.cuda.empty_cache()
    ib, ob = inner_bytes(n, k), outer_bytes(n, k)
    return {"inner_ms": im, "inner_GBps": ib / im / 1e6, "inner_frac": ib / im / 1e6 / HBM_PEAK_GBS,
            "outer_ms": om, "outer_GBps": ob / om / 1e6, "outer_frac": ob / om / 1e6 / HBM_PEAK_GBS}


def run_mixed_precision(k, reps, torch, D, synth):
    """Rows a1 + a2 in mixed precision: binary16 gradients scaled by 65536 on the 150M set plus
    2000 ragged tensors; the inf/NaN check, then the inner step with the unscale fused in."""
    wl = synth.WORKLOADS["stress"]()
    n = wl.n_params
    stream = torch.cuda.current_stream()
    holder = {}

    def fill(theta0, layout, offsets):
        holder["kind"] = torch.from_numpy(wl.kind_map(offsets, layout.n_pad)).to(theta0.device)
        synth.device_fill_f32(theta0.data_ptr(), layout.n_pad, synth.key(synth.STREAM_WEIGHTS),
                              0.02, holder["kind"].data_ptr(), ones_as_one=True,
                              stream=stream.cuda_stream)

    dl = D.DiLoCo(wl.numel, k, fill_theta0=fill)
    kind = holder["kind"]
    g = dl.new_grads(torch.float16)
    for r in range(k):
        synth.device_fill_f16(g[r].data_ptr(), dl.layout.n_pad, synth.key(synth.STREAM_GRADS, r, 0),
                              kind.data_ptr(), stream=stream.cuda_stream)
    flags = dl.new_flags()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * reps + 1)]
    dl.unscale_check(g, 1.0 / 65536, flags)
    dl.inner_step(g, flags=flags)
    torch.cuda.synchronize()
    ev[0].record(stream)
    for i in range(reps):
        dl.unscale_check(g, 1.0 / 65536, flags)
        ev[2 * i + 1].record(stream)
        dl.inner_step(g, flags=flags)
        ev[2 * i + 2].record(stream)
    torch.cuda.synchronize()
    chk = sum(ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(reps)) / reps
    inn = sum(ev[2 * i + 1].elapsed_time(ev[2 * i + 2]) for i in range(reps)) / reps
    assert flags.cpu().tolist() == [0] * k and dl.steps() == [reps + 1] * k
    dl.close()
    del dl, g, kind
    torch.cuda.empty_cache()
    cb, ib = 2 * n * k, inner_bytes(n, k, g16=True)
    return {"config": {"workload": "llama150m + 2000 ragged tensors x %d workers, FP16 gradients "
                                   "scaled by 65536" % k, "n_params": n, "n_tensors": len(wl.shapes)},
            "unscale_check": {"ms": chk, "bytes": cb, "GBps": cb / chk / 1e6,
                              "frac_of_peak": cb / chk / 1e6 / HBM_PEAK_GBS,
                              "note": "includes the flag-clearing launch"},
            "inner_step_fp16_grads": {"ms": inn, "bytes": ib, "GBps": ib / inn / 1e6,
                                      "frac_of_peak": ib / inn / 1e6 / HBM_PEAK_GBS},
            "launches_timed": reps}


def cpu_baseline(k, log2_slice=25, inner_reps=100, outer_reps=100):
    """The oracle as it stands, timed on this host's cores on a bounded sample of the workload:
    a contiguous slice of the flat buffers, k workers; its inner-step and outer-step loops are
    each repeated on preallocated arrays after one warm-up pass."""
    import numpy as np
    import oracle
    import synth
    n = 1 << log2_slice
    theta0 = synth.host_fill_f32(n, synth.key(synth.STREAM_WEIGHTS), 0.02)
    workers = [oracle.AdamWState(theta0) for _ in range(k)]
    g = [synth.host_fill_f32(n, synth.key(synth.STREAM_GRADS, r, 0), 1e-3) for r in range(k)]
    b = np.zeros(n, dtype=np.float32)
    theta = np.empty((k, n), dtype=np.float32)
    scratch = (np.zeros((k, n), dtype=np.float32), np.zeros(n, dtype=np.float32))
    hp = (4e-4, 0.9, 0.999, 1e-8, 0.1)

    def inner():
        for r in range(k):
            oracle.adamw_step(workers[r], g[r], *hp)

    def outer():
        oracle.outer_step(theta0, b, theta, 0.7, 0.9, False, scratch)

    inner()                                   # warm-up (pages in, threads up)
    for r in range(k):
        theta[r] = workers[r].theta
    outer()
    t0 = time.perf_counter()
    for _ in range(inner_reps):
        inner()
    t1 = time.perf_counter()
    for _ in range(outer_reps):
        outer()
    t2 = time.perf_counter()
    inner_s, outer_s = (t1 - t0) / inner_reps, (t2 - t1) / outer_reps
    total_bytes = inner_reps * inner_bytes(n, k) + outer_reps * outer_bytes(n, k)
    return {
        "value": total_bytes / (t2 - t0) / 1e9, "unit": "GB/s", "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": "2^%d-element slice of the flat buffers x %d workers: %d AdamW inner steps and "
                  "%d outer steps (FP32 pseudo-gradient) on preallocated arrays after one warm-up "
                  "pass; value = algorithmic bytes of all of them / their time"
                  % (log2_slice, k, inner_reps, outer_reps),
        "inner_step_GBps": inner_bytes(n, k) / inner_s / 1e9,
        "outer_step_GBps": outer_bytes(n, k) / outer_s / 1e9,
        "inner_step_ms_extrapolated_to_workload": None,
        "inner_ns_per_element_worker": inner_s / (n * k) * 1e9,
        "outer_ns_per_element": outer_s / n * 1e9,
        "seconds": t2 - t0,
        "host_cpus_visible": os.cpu_count(),
    }


def load_traffic(root, kernel, workload):
    """Measured HBM bytes per launch from the committed rocprofv3 --pmc summary, if present."""
    path = os.path.join(root, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            t = json.load(f)
        return t[workload][kernel]["bytes_per_launch"]
    except (OSError, KeyError, ValueError):
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3, help="timed rounds (H inner + 1 outer each)")
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llama150m", choices=["tiny", "llama150m", "llama1.1b"])
    ap.add_argument("--k", type=int, default=8)
    ap.add_argument("--h", type=int, default=500)
    ap.add_argument("--pg", default=None, choices=["f32", "f16"])
    ap.add_argument("--no-also", action="store_true", help="skip the second headline workload")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--calibration-copy", type=int, default=0, metavar="MIB",
                    help="first run a plain copy kernel of this many MiB three times (reference "
                         "for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this path is single-GPU (k worker replicas resident on one MI355X); "
                 "--gpus %d is not supported, run with --gpus 1" % args.gpus)

    root = os.path.dirname(os.path.abspath(__file__))
    sys.path.insert(0, root)
    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; the HIP path has no CPU fallback")
    import paper_2407_07852_amd as D
    import synth
    torch.cuda.set_device(0)

    if args.calibration_copy:
        nb = args.calibration_copy << 20
        a = torch.zeros(nb // 4, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            synth.device_copy(b.data_ptr(), a.data_ptr(), nb,
                              torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()

    pg = args.pg or ("f16" if args.workload == "llama1.1b" else "f32")
    main_res = run_workload(args.workload, args.k, args.h, pg == "f16", args.steps, args.warmup,
                            torch, D, synth)
    also = None
    if not args.no_also and args.workload == "llama150m":
        # the other configuration the metric is quoted on: 1.1B x 8, FP16 pseudo-gradient
        also = run_workload("llama1.1b", args.k, args.h, True, 1, 0, torch, D, synth)
        also["warmup_note"] = "no warm-up round; the first launches of 500 absorb it"

    def roof(res, which):
        r = res[which]
        kernel = "adamw_flat_kernel" if which == "inner" else "outer_fused_kernel"
        return {"bound": "hbm", "kernel": kernel, "achieved": r["GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": r["frac_of_peak"], "ms_per_launch": r["ms"],
                "algorithmic_bytes_per_launch": r["bytes"],
                "traffic": load_traffic(root, kernel, res["workload"])}

    out = {
        "metric": "inner/outer step HBM GB/s (% of peak) + outer-step ms",
        "value": main_res["round_GBps"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["round_ms"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32",
        "data": "synthetic (seeded bell-shaped weights ~N(0,0.02), norm vectors 1.0, one resident "
                "gradient set ~N(0,1e-3) per worker)",
        "config": {"workload": "%s x %d workers, H=%d AdamW inner steps + 1 outer step, %s "
                               "pseudo-gradient" % (main_res["workload"], args.k, args.h, pg),
                   "n_params": main_res["n_params"], "k_workers": args.k, "H": args.h,
                   "pg_dtype": pg, "step": "one round = H inner launches + 1 outer launch"},
        "inner_step": main_res["inner"], "outer_step": main_res["outer"],
        "outer_step_ms": main_res["outer"]["ms"],
        "roofline": roof(main_res, "inner"),
        "roofline_outer": roof(main_res, "outer"),
        "finite": main_res["finite"],
    }
    if also is not None:
        out["also"] = {"config": {"workload": "llama1.1b x %d workers, H=%d, f16 pseudo-gradient"
                                  % (args.k, args.h), "n_params": also["n_params"]},
                       "value": also["round_GBps"], "ms_per_step": also["round_ms"],
                       "inner_step": also["inner"], "outer_step": also["outer"],
                       "roofline": roof(also, "inner"), "roofline_outer": roof(also, "outer"),
                       "finite": also["finite"], "note": also["warmup_note"]}
    if not args.no_also and args.workload == "llama150m":
        out["mixed_precision"] = run_mixed_precision(4, 20, torch, D, synth)
        pgr = run_workload("llama150m", args.k, 100, False, 1, 0, torch, D, synth, groups=True)
        # worker-count sweep of the paper's ablation (1, 2, 4, 8 workers) and the
        # reduced-precision pseudo-gradient modes, short timings on the 150M set
        out["k_sweep"] = {"workload": "llama150m, FP32 pseudo-gradient, 40 inner + 20 outer launches",
                          **{"k=%d" % kk: quick_measure("llama150m", kk, D.F32, 0, 40, 20, torch, D, synth)
                             for kk in (1, 2, 4, 8)}}
        out["pg_modes"] = {"workload": "llama150m x 8 workers, outer step only, 20 launches",
                           **{nm: {kq: v for kq, v in quick_measure("llama150m", 8, pg, rm, 1, 20, torch, D,
                                                                     synth).items() if kq.startswith("outer")}
                              for nm, pg, rm in (("f32", D.F32, 0), ("f16", D.F16, 0),
                                                 ("f16+rounded_mean", D.F16, 1), ("bf16", D.BF16, 0),
                                                 ("bf16+rounded_mean", D.BF16, 1))}}
        out["param_groups"] = {
            "config": {"workload": "llama150m x %d workers, 100 inner steps, 3 parameter groups "
                                   "(norm vectors and embedding exempt from weight decay)" % args.k},
            "inner_step": pgr["inner"]}
    if not args.no_cpu:
        cb = cpu_baseline(args.k)
        n = main_res["n_params"]
        cb["inner_step_ms_extrapolated_to_workload"] = cb["inner_ns_per_element_worker"] * n * args.k / 1e6
        cb["outer_step_ms_extrapolated_to_workload"] = cb["outer_ns_per_element"] * n / 1e6
        out["cpu_baseline"] = cb
    print(json.dumps(out))


if __name__ == "__main__":
    main()
