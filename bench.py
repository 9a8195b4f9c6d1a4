#!/usr/bin/env python3
"""Benchmark of the DiLoCo optimizer hot path on one MI355X.

One "step" is one DiLoCo round over synthetic inputs already resident in HBM: H fused AdamW
inner steps of all k workers, then one fused outer step (pseudo-gradient, optional FP16
rounding, mean over k, Nesterov SGD, broadcast).  The headline value is the algorithmic HBM
traffic of the round divided by its wall time.  Every kernel launch of a timed region is
bracketed by HIP events on the stream it is launched on, so each kernel is reported with the
mean, median, minimum and maximum of its launch durations.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload tiny|llama150m|llama1.1b]
                    [--h H] [--k K] [--pg f32|f16] [--no-also] [--no-cpu] [--tune name=value ...]

Prints ONE JSON line.  Everything on this path is single-GPU: --gpus above 1 is refused.
"""
import argparse
import json
import os
import subprocess
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


def stats(ms, nbytes):
    """Launch-duration statistics and the bandwidth figures that follow from them."""
    s = sorted(ms)
    mean, med = sum(s) / len(s), s[len(s) // 2]
    return {"ms": mean, "ms_median": med, "ms_min": s[0], "ms_max": s[-1], "launches_timed": len(s),
            "bytes": nbytes, "GBps": nbytes / mean / 1e6, "frac_of_peak": nbytes / mean / 1e6 / HBM_PEAK_GBS,
            "frac_of_peak_median": nbytes / med / 1e6 / HBM_PEAK_GBS}


class Bench:
    """All device memory of the run comes out of ONE allocation made at start-up and is handed
    out again leg after leg.  The driver clears freed device memory in the background (measured
    here: about 34 GB/s, for as long as it takes), and while it does, every kernel loses 1-4 % of
    its bandwidth; a benchmark that frees and re-allocates its buffers between legs measures
    that, not the kernels."""

    def __init__(self, torch, D, synth, tune, pool_bytes):
        self.torch, self.D, self.synth, self.tune = torch, D, synth, tune
        self.stream = torch.cuda.current_stream()
        self.pool = torch.empty(pool_bytes, dtype=torch.uint8, device="cuda")
        self.base = 0       # offset of the current leg's first buffer (placement_spread moves it)
        self.cursor = 0

    def take(self, nbytes, dtype):
        """The next nbytes of the pool (2 MiB-aligned, as large allocations are) as a tensor."""
        start = (self.cursor + (1 << 21) - 1) >> 21 << 21
        assert start + nbytes <= self.pool.numel(), "benchmark pool too small"
        self.cursor = start + nbytes
        return self.pool[start:start + nbytes].view(dtype)

    def reset(self):
        self.cursor = self.base

    # ------------------------------------------------------------------ set-up
    def make(self, name, k, H=0, pg=0, round_mean=0, groups=False, g16=False, zeros=False,
             layout_mode=0):
        """A context on the named workload with seeded synthetic weights (matrices ~N(0, 0.02),
        norm vectors 1.0) and one resident seeded gradient set ~N(0, 1e-3) per worker."""
        torch, D, synth = self.torch, self.D, self.synth
        wl = synth.WORKLOADS[name]()
        holder = {}
        self.reset()
        lay, _ = D.diloco_query_layout(D.make_config(wl.numel, k, layout_mode=layout_mode))

        def fill(theta0, layout, offsets):
            holder["kind"] = self.take(layout.n_pad, torch.uint8)
            holder["kind"].copy_(torch.from_numpy(wl.kind_map(offsets, layout.n_pad)))
            synth.device_fill_f32(theta0.data_ptr(), layout.n_pad, synth.key(synth.STREAM_WEIGHTS),
                                  0.02, holder["kind"].data_ptr(), ones_as_one=True,
                                  stream=self.stream.cuda_stream)

        dl = D.DiLoCo(wl.numel, k, fill_theta0=fill, h_inner_steps=H, pg_dtype=pg,
                      pg_round_mean=round_mean, layout_mode=layout_mode,
                      arena=self.take(lay.arena_bytes, torch.float32))
        if self.tune:
            dl.set_tuning(**self.tune)
        if groups:
            # matrices decay 0.1; norm vectors and the embedding / LM head: no decay, and the
            # embeddings at half the learning rate
            grp = [1 if v else 0 for v in wl.is_vector]
            grp[-1] = 2
            if name == "llama1.1b":
                grp[-2] = 2
            dl.set_param_groups(grp, [1.0, 1.0, 0.5], [0.1, 0.0, 0.0])
        gdt = torch.float16 if g16 else torch.float32
        grads = dl.new_grads(gdt)   # the arena's own gradient slots
        for r in range(k):
            if g16:
                synth.device_fill_f16(grads[r].data_ptr(), dl.layout.n_pad,
                                      synth.key(synth.STREAM_GRADS, r, 0), holder["kind"].data_ptr(),
                                      stream=self.stream.cuda_stream)
            else:
                synth.device_fill_f32(grads[r].data_ptr(), dl.layout.n_pad,
                                      synth.key(synth.STREAM_GRADS, r, 0), 1e-3,
                                      holder["kind"].data_ptr(), stream=self.stream.cuda_stream)
        if zeros:   # all-zero weights and gradients: only for the data-dependence leg
            dl.theta0.zero_()
            dl.theta.zero_()
            grads.zero_()
        torch.cuda.synchronize()
        return wl, dl, grads

    def flush(self):
        pass  # nothing is freed between legs: see the class comment

    # ------------------------------------------------------------------ timing
    def time_sequence(self, fns):
        """Calls every function of the list in order, each bracketed by events on the launch
        stream, with no host synchronisation in between (so the queue never runs dry and no
        host launch latency lands inside a bracket); -> list of ms, one per call."""
        torch = self.torch
        n = len(fns)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        ev[0].record(self.stream)
        for i, fn in enumerate(fns):
            fn()
            ev[i + 1].record(self.stream)
        ev[n].synchronize()
        return [ev[i].elapsed_time(ev[i + 1]) for i in range(n)]

    def time_launches(self, fn, n):
        """n calls of fn, each bracketed by events on the launch stream; -> list of ms."""
        return self.time_sequence([fn] * n)

    def rounds(self, name, k, H, pg, rounds, warmup_rounds, warmup_inner=None, extra_outer=0,
               groups=False):
        """`warmup_rounds` untimed rounds (of warmup_inner inner steps each, default H), then
        `rounds` timed rounds of H inner steps + 1 outer step with every launch timed, then
        `extra_outer` more timed outer steps (rounds with no inner steps, which the method
        allows)."""
        torch, D = self.torch, self.D
        wl, dl, grads = self.make(name, k, H=H, pg=pg, groups=groups)
        n = wl.n_params
        for _ in range(warmup_rounds):
            for _ in range(H if warmup_inner is None else warmup_inner):
                dl.inner_step(grads)
            dl.outer_step()
        torch.cuda.synchronize()
        inner_ms, outer_ms = [], []
        t0 = time.perf_counter()
        step = lambda: dl.inner_step(grads)  # noqa: E731
        for _ in range(rounds):
            ms = self.time_sequence([step] * H + [dl.outer_step])
            inner_ms += ms[:H]
            outer_ms += ms[H:]
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        in_round_ms = list(outer_ms)
        batch_ms = None
        if extra_outer:
            outer_ms += self.time_launches(dl.outer_step, extra_outer)
            # the same number of launches once more between ONE pair of events: what a launch
            # takes when no event record sits between consecutive launches
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(self.stream)
            for _ in range(extra_outer):
                dl.outer_step()
            e1.record(self.stream)
            e1.synchronize()
            batch_ms = e0.elapsed_time(e1) / extra_outer
        done = (H if warmup_inner is None else warmup_inner) * warmup_rounds + H * rounds
        assert dl.steps() == [done] * k
        finite = bool(torch.isfinite(dl.theta0).all())
        dl.close()
        del dl, grads
        self.flush()
        ib, ob = inner_bytes(n, k), outer_bytes(n, k)
        round_ms = wall_ms / rounds
        res = {"workload": name, "n_params": n, "k": k, "H": H,
               "pg_dtype": {0: "f32", 1: "f16", 2: "bf16"}[pg], "finite": finite,
               "round_ms": round_ms, "round_GBps": (H * ib + ob) / round_ms / 1e6,
               "outer": stats(outer_ms, ob),
               "outer_in_rounds": stats(in_round_ms, ob)}
        if batch_ms is not None:
            res["outer"]["ms_back_to_back"] = batch_ms
            res["outer"]["frac_of_peak_back_to_back"] = ob / batch_ms / 1e6 / HBM_PEAK_GBS
            res["outer"]["note"] = ("ms / frac_of_peak: every launch between its own pair of events; "
                                    "back_to_back: %d launches between one pair" % extra_outer)
        if H:
            res["inner"] = stats(inner_ms, ib)
        return res

    def quick(self, name, k, pg=0, round_mean=0, n_inner=20, n_outer=20, groups=False, tune=None,
              zeros=False, layout_mode=0):
        """Short timing of both kernels: n_inner inner and n_outer outer launches after two
        warm-up launches of each."""
        wl, dl, grads = self.make(name, k, pg=pg, round_mean=round_mean, groups=groups, zeros=zeros,
                                  layout_mode=layout_mode)
        if tune:
            dl.set_tuning(**tune)
        n = wl.n_params
        for _ in range(2):
            dl.inner_step(grads)
            dl.outer_step()
        self.torch.cuda.synchronize()
        out = {}
        if n_inner:
            out["inner"] = stats(self.time_launches(lambda: dl.inner_step(grads), n_inner),
                                 inner_bytes(n, k))
        if n_outer:
            out["outer"] = stats(self.time_launches(dl.outer_step, n_outer), outer_bytes(n, k))
        dl.close()
        del dl, grads
        self.flush()
        return out

    def placement_spread(self, name, k, pg, n_inner, n_outer):
        """The same measurement with the arena and the gradients placed at three different
        offsets inside the pool (three different sets of physical pages)."""
        runs = []
        for spacer_mib in (0, 130, 1026):
            self.base = spacer_mib << 20
            q = self.quick(name, k, pg=pg, n_inner=n_inner, n_outer=n_outer)
            self.base = 0
            runs.append({"spacer_MiB": spacer_mib,
                         "inner_frac_median": q["inner"]["frac_of_peak_median"],
                         "outer_frac_median": q["outer"]["frac_of_peak_median"],
                         "inner_ms_median": q["inner"]["ms_median"],
                         "outer_ms_median": q["outer"]["ms_median"]})
        return {"workload": "%s x %d workers, %s pseudo-gradient; %d inner + %d outer launches per "
                            "placement (offsets 0, 130 and 1026 MiB inside the run's one device "
                            "allocation)" % (name, k, {0: "f32", 1: "f16"}[pg], n_inner, n_outer),
                "runs": runs,
                "inner_frac_min": min(r["inner_frac_median"] for r in runs),
                "inner_frac_max": max(r["inner_frac_median"] for r in runs),
                "outer_frac_min": min(r["outer_frac_median"] for r in runs),
                "outer_frac_max": max(r["outer_frac_median"] for r in runs)}

    def delayed_outer(self, name, k, pg, delay, reps):
        """The delayed application of the outer step (update on a side stream from a snapshot,
        merge later) next to the plain outer step: A = `delay` inner steps alone, B = begin +
        finish with nothing in between, C = begin, `delay` inner steps, finish.  What the overlap
        saves is A + B - C; both streams are HBM-bound, so it cannot be much."""
        torch = self.torch
        wl, dl, grads = self.make(name, k, pg=pg)
        n = wl.n_params
        snap = self.take(dl.grads_numel() * 4, torch.float32)
        side = torch.cuda.Stream()

        def seq_a():
            for _ in range(delay):
                dl.inner_step(grads)

        def seq_b():
            dl.outer_begin(snapshot=snap, side_stream=side)
            dl.outer_finish()

        def seq_c():
            dl.outer_begin(snapshot=snap, side_stream=side)
            for _ in range(delay):
                dl.inner_step(grads)
            dl.outer_finish()

        for fn in (seq_a, seq_b, seq_c, dl.outer_step):
            fn()
        torch.cuda.synchronize()
        med = lambda xs: sorted(xs)[len(xs) // 2]  # noqa: E731
        t_sync = med(self.time_launches(dl.outer_step, reps))
        t_a = med(self.time_launches(seq_a, reps))
        t_b = med(self.time_launches(seq_b, reps))
        halves = self.time_sequence([lambda: dl.outer_begin(snapshot=snap, side_stream=side),
                                     dl.outer_finish] * reps)
        t_snapshot, t_rest = med(halves[0::2]), med(halves[1::2])
        t_c = med(self.time_launches(seq_c, reps))
        dl.close()
        del dl, grads, snap
        bytes_delayed = (20 + 24 * k) * n   # snapshot 8k, update 16+4k, merge 4+12k bytes/element
        return {"config": "%s x %d workers, %s pseudo-gradient, %d inner steps between begin and "
                          "finish, medians of %d" % (name, k, {0: "f32", 1: "f16"}[pg], delay, reps),
                "outer_step_ms": t_sync, "inner_steps_alone_ms": t_a,
                "begin_finish_back_to_back_ms": t_b, "begin_inner_steps_finish_ms": t_c,
                "saved_by_overlap_ms": t_a + t_b - t_c,
                "extra_cost_over_plain_outer_step_ms": t_c - t_a - t_sync,
                "bytes_begin_finish": bytes_delayed,
                "begin_finish_GBps": bytes_delayed / t_b / 1e6,
                "begin_finish_frac_of_peak": bytes_delayed / t_b / 1e6 / HBM_PEAK_GBS,
                "snapshot_ms": t_snapshot,
                "snapshot_frac_of_peak": 8 * k * n / t_snapshot / 1e6 / HBM_PEAK_GBS,
                "update_plus_merge_ms": t_rest,
                "update_plus_merge_frac_of_peak": (20 + 16 * k) * n / t_rest / 1e6 / HBM_PEAK_GBS,
                "note": "snapshot 8k + update (16+4k) + merge (4+12k) = (20+24k) B/element against "
                        "(16+8k) for the plain outer step: on one GPU the delayed form costs more "
                        "traffic and the overlap buys little, because both streams compete for "
                        "the same HBM bandwidth"}

    def stream_patterns(self, mib=1024, reps=20):
        """What the machine sustains for plain streaming traffic of the same mixes and in the same
        launch shape as the optimizer kernels (no arithmetic): pure reads, pure writes, a copy,
        4 read + 3 write streams (the inner step's mix), 10 + 10 (the outer step's at k = 8).
        Separate 1 GiB buffers of seeded random data; best residency of a small sweep."""
        torch, synth = self.torch, self.synth
        self.reset()
        nbytes = mib << 20
        bufs = [self.take(nbytes, torch.float32) for _ in range(20)]
        for j, b in enumerate(bufs):
            synth.device_fill_f32(b.data_ptr(), b.numel(), synth.key(synth.STREAM_WEIGHTS, j), 0.02,
                                  stream=self.stream.cuda_stream)
        sink = self.take(1024, torch.float32)
        ptrs = [b.data_ptr() for b in bufs]
        out = {"buffer_MiB": mib, "launches_timed": reps,
               "note": "GB/s = (read + write streams) x buffer bytes / median launch time"}
        # (name, read streams, write streams, written in place?, residencies tried)
        cases = (("1R", 1, 0, False, (8, 16, 24, 32)),
                 ("4R", 4, 0, False, (6, 8, 12, 16, 24)),
                 ("10R", 10, 0, False, (3, 4, 5, 6, 8, 12, 24)),
                 ("10W", 0, 10, False, (2, 3, 4, 6, 8, 16)),
                 ("1R+1W", 1, 1, False, (8, 16, 24, 32)),
                 ("4R+3W", 4, 3, False, (8, 9, 10, 11, 12, 14)),
                 ("4R+3W_in_place", 4, 3, True, (8, 9, 10, 11, 12, 14)),
                 ("10R+10W", 10, 10, False, (2, 3, 4, 5, 6)),
                 ("10R+10W_in_place", 10, 10, True, (2, 3, 4, 5, 6)))
        for nm, nr, nw, in_place, waves in cases:
            # in place: the write streams are the first nw read streams, as in the optimizer
            # kernels (theta, m, v rewritten; theta0, mom and every worker's weights rewritten)
            use = ptrs[:nr] + (ptrs[:nw] if in_place else ptrs[nr:nr + nw])
            best = None
            for w in waves:
                go = lambda: synth.device_stream_pattern(use, nr, nw, nbytes, w, sink.data_ptr(),  # noqa: E731
                                                         self.stream.cuda_stream)
                go()
                go()
                ms = sorted(self.time_launches(go, reps))[reps // 2]
                gbps = (nr + nw) * nbytes / ms / 1e6
                if best is None or gbps > best["GBps"]:
                    best = {"GBps": gbps, "frac_of_peak": gbps / HBM_PEAK_GBS, "waves_per_cu": w,
                            "ms_median": ms}
            out[nm] = best
        return out

    def free_effect(self, gib, seconds=9.0):
        """What freeing device memory does to a kernel that runs afterwards: inner steps of the
        150M x 8 set are timed in bursts of 25 before, and for `seconds` after, a separate
        allocation of `gib` GiB is made and freed (the one thing in this benchmark that frees)."""
        torch = self.torch
        wl, dl, grads = self.make("llama150m", 8)
        ib = inner_bytes(wl.n_params, 8)

        def burst():
            ms = self.time_launches(lambda: dl.inner_step(grads), 25)
            return ib / (sum(ms) / len(ms)) / 1e6 / HBM_PEAK_GBS

        before = [burst() for _ in range(5)]
        t0 = time.perf_counter()
        big = torch.empty(gib << 30, dtype=torch.uint8, device="cuda")
        del big
        torch.cuda.empty_cache()
        t_free = time.perf_counter() - t0
        after = []
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            after.append((round(time.perf_counter() - t0, 2), burst()))
        dl.close()
        del dl, grads
        lo = min(f for _, f in after)
        recovered = next((t for t, f in after if f >= min(before) - 0.002 and
                          all(g >= min(before) - 0.002 for tt, g in after if tt >= t)), None)
        return {"freed_GiB": gib, "alloc_and_free_seconds": t_free,
                "inner_frac_before": before, "inner_frac_after": after,
                "inner_frac_lowest_after": lo, "seconds_until_back_to_normal": recovered}

    def tiny_graph(self, k, H, rounds):
        """Tiny is launch-bound (2 launches per inner step, 1 per outer step, a few microseconds
        of work each), which is what HIP graphs are for: one whole round (H inner steps + the
        outer step) captured once and replayed, against the same round launched eagerly.  The
        step state lives on the device, so the captured round replays correctly any number of
        times (tests/test_gpu_graph_capture.py checks replays against the oracle)."""
        torch = self.torch
        side = torch.cuda.Stream()
        main_stream = self.stream
        self.stream = side                       # the context borrows the capturing stream
        try:
            with torch.cuda.stream(side):
                wl, dl, grads = self.make("tiny", k, H=H)

                def one_round():
                    for _ in range(H):
                        dl.inner_step(grads)
                    dl.outer_step()

                one_round()
                side.synchronize()
                t0 = time.perf_counter()
                for _ in range(rounds):
                    one_round()
                side.synchronize()
                eager_us = (time.perf_counter() - t0) / rounds * 1e6
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    one_round()
                graph.replay()
                side.synchronize()
                t0 = time.perf_counter()
                for _ in range(rounds):
                    graph.replay()
                side.synchronize()
                graph_us = (time.perf_counter() - t0) / rounds * 1e6
                steps = dl.steps()
                dl.close()
                del graph, dl, grads
        finally:
            self.stream = main_stream
        assert steps == [H * (2 * rounds + 2)] * k, steps
        return {"config": "tiny x %d workers, one round = %d inner steps + 1 outer step (%d kernel "
                          "launches), wall time per round over %d rounds" % (k, H, 2 * H + 1, rounds),
                "eager_us_per_round": eager_us, "graph_replay_us_per_round": graph_us}

    def mixed_precision(self, k, reps):
        """Rows a1 + a2 in mixed precision: binary16 gradients scaled by 65536 on the 150M set
        plus 2000 ragged tensors; the inf/NaN check, then the inner step with the unscale fused."""
        torch = self.torch
        wl, dl, g = self.make("stress", k, g16=True)
        n = wl.n_params
        flags = dl.new_flags()
        dl.unscale_check(g, 1.0 / 65536, flags)
        dl.inner_step(g, flags=flags)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2 * reps + 1)]
        ev[0].record(self.stream)
        for i in range(reps):
            dl.unscale_check(g, 1.0 / 65536, flags)
            ev[2 * i + 1].record(self.stream)
            dl.inner_step(g, flags=flags)
            ev[2 * i + 2].record(self.stream)
        torch.cuda.synchronize()
        chk = [ev[2 * i].elapsed_time(ev[2 * i + 1]) for i in range(reps)]
        inn = [ev[2 * i + 1].elapsed_time(ev[2 * i + 2]) for i in range(reps)]
        assert flags.cpu().tolist() == [0] * k and dl.steps() == [reps + 1] * k
        dl.close()
        del dl, g
        self.flush()
        return {"config": {"workload": "llama150m + 2000 ragged tensors x %d workers, FP16 gradients "
                                       "scaled by 65536" % k, "n_params": n, "n_tensors": len(wl.shapes)},
                "unscale_check": dict(stats(chk, 2 * n * k), note="includes the flag-clearing launch"),
                "inner_step_fp16_grads": dict(stats(inn, inner_bytes(n, k, g16=True)),
                                              note="includes the step-prologue launch")}


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
        "inner_ns_per_element_worker": inner_s / (n * k) * 1e9,
        "outer_ns_per_element": outer_s / n * 1e9,
        "seconds": t2 - t0,
        "host_cpus_visible": os.cpu_count(),
    }


def load_traffic(root, kernel, workload):
    """Measured HBM bytes per launch of `kernel` on `workload` from the committed rocprofv3 --pmc
    summary, with where it comes from; (None, reason) when the file does not cover the case."""
    path = os.path.join(root, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            t = json.load(f)
        src = "profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, measured at commit %s)" \
            % t.get("measured_at_commit", "unknown")
        return t[workload][kernel]["bytes_per_launch"], src
    except (OSError, KeyError, ValueError):
        return None, "no committed counter summary covers this kernel and workload"


def git_head(root):
    try:
        return subprocess.run(["git", "-C", root, "rev-parse", "--short", "HEAD"], capture_output=True,
                              text=True, timeout=10).stdout.strip() or None
    except Exception:
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
    ap.add_argument("--no-also", action="store_true", help="only the main workload's rounds")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--tune", nargs="*", default=[], metavar="NAME=VALUE",
                    help="launch-shape knobs applied to every context (diloco_set_tuning)")
    ap.add_argument("--settle", type=float, default=10.0, metavar="SECONDS",
                    help="wait this long before the run's one device allocation is made.  The "
                         "driver clears device memory freed by earlier processes in the "
                         "background (about 34 GB/s, so up to 9 s for a whole GPU); an allocation "
                         "made meanwhile is placed elsewhere physically, and at the 1.1B size "
                         "that moves the kernels by up to 2 points either way")
    ap.add_argument("--free-effect", type=int, default=0, metavar="GIB",
                    help="instead of the benchmark: allocate and free this many GiB, and time the "
                         "inner step before and for 9 s afterwards (the driver clears freed "
                         "memory in the background)")
    ap.add_argument("--delayed-only", action="store_true",
                    help="only the delayed outer step's leg on --workload (for counter runs)")
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
    tune = {kv.split("=")[0]: int(kv.split("=")[1]) for kv in args.tune}
    # one device allocation for the whole run, sized for the largest leg (arena, which includes
    # the FP32 gradient slots, + the generator's kind map), the placement legs' largest offset
    # and alignment slack
    full = not args.no_also and args.workload == "llama150m" and not args.free_effect
    big = synth.WORKLOADS["llama1.1b" if full else args.workload]()
    kk = max(args.k, 8) if (full or args.free_effect) else args.k
    big_lay, _ = D.diloco_query_layout(D.make_config(big.numel, kk))
    # (the arena holds the gradients; the delayed outer step's snapshot is k slots more)
    pool_bytes = (big_lay.arena_bytes + kk * big_lay.slot * 4 + big_lay.n_pad + (1100 << 20))
    if args.settle > 0:
        torch.cuda.init()
        time.sleep(args.settle)
    B = Bench(torch, D, synth, tune, pool_bytes)

    if args.calibration_copy:
        nb = args.calibration_copy << 20
        a = torch.zeros(nb // 4, device="cuda")
        b = torch.empty_like(a)
        for _ in range(3):
            synth.device_copy(b.data_ptr(), a.data_ptr(), nb, B.stream.cuda_stream)
        torch.cuda.synchronize()
        del a, b
        torch.cuda.empty_cache()

    if args.free_effect:
        print(json.dumps({"free_effect": B.free_effect(args.free_effect)}))
        return
    if args.delayed_only:
        pgd = D.F16 if (args.pg or ("f16" if args.workload == "llama1.1b" else "f32")) == "f16" else D.F32
        print(json.dumps({"delayed_outer": B.delayed_outer(args.workload, args.k, pgd, 2, 20)}))
        return

    pgn = args.pg or ("f16" if args.workload == "llama1.1b" else "f32")
    pg = D.F16 if pgn == "f16" else D.F32
    # after the timed rounds, 50 more outer steps (rounds without inner steps) so that the outer
    # kernel's statistics rest on more than one launch per round
    main_res = B.rounds(args.workload, args.k, args.h, pg, args.steps, args.warmup, extra_outer=50)
    also = None
    if full:
        # the other configuration the metric is quoted on: 1.1B x 8, FP16 pseudo-gradient.  One
        # short warm-up round (10 inner steps + 1 outer step), one timed round of H inner steps,
        # then 20 more timed outer steps.
        also = B.rounds("llama1.1b", args.k, args.h, D.F16, 1, 1, warmup_inner=10, extra_outer=20)

    def roof(res, which):
        r = res[which]
        kernel = "adamw_flat_kernel" if which == "inner" else "outer_fused_kernel"
        traffic, src = load_traffic(root, kernel, res["workload"])
        return {"bound": "hbm", "kernel": kernel, "achieved": r["GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": r["frac_of_peak"], "ms_per_launch": r["ms"],
                "ms_per_launch_median": r["ms_median"], "launches_timed": r["launches_timed"],
                "algorithmic_bytes_per_launch": r["bytes"], "traffic": traffic,
                "traffic_source": src}

    out = {
        "metric": "inner/outer step HBM GB/s (% of peak) + outer-step ms",
        "value": main_res["round_GBps"], "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["round_ms"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32",
        "data": "synthetic (seeded bell-shaped weights ~N(0,0.02), norm vectors 1.0, one resident "
                "gradient set ~N(0,1e-3) per worker)",
        "config": {"workload": "%s x %d workers, H=%d AdamW inner steps + 1 outer step, %s "
                               "pseudo-gradient" % (main_res["workload"], args.k, args.h, pgn),
                   "n_params": main_res["n_params"], "k_workers": args.k, "H": args.h,
                   "pg_dtype": pgn, "step": "one round = H inner launches + 1 outer launch",
                   "tuning_overrides": tune, "commit": git_head(root),
                   "settle_seconds_before_allocating": args.settle},
        "outer_step": main_res["outer"], "outer_step_ms": main_res["outer"]["ms"],
        "outer_step_in_rounds": main_res["outer_in_rounds"],
        "finite": main_res["finite"],
    }
    if "inner" in main_res:
        out["inner_step"] = main_res["inner"]
        out["roofline"] = roof(main_res, "inner")
    out["roofline_outer"] = roof(main_res, "outer")
    if full:
        out["also"] = {"config": {"workload": "llama1.1b x %d workers, H=%d, f16 pseudo-gradient"
                                  % (args.k, args.h), "n_params": also["n_params"],
                                  "note": "one warm-up round of 10 inner steps + 1 outer step; one "
                                          "timed round; then 20 more timed outer steps (outer_step "
                                          "covers all 21, outer_step_in_rounds the one of the round)"},
                       "value": also["round_GBps"], "ms_per_step": also["round_ms"],
                       "inner_step": also["inner"], "outer_step": also["outer"],
                       "outer_step_in_rounds": also["outer_in_rounds"],
                       "roofline": roof(also, "inner"), "roofline_outer": roof(also, "outer"),
                       "finite": also["finite"]}
        out["placement_spread"] = {
            "llama150m": B.placement_spread("llama150m", args.k, pg, 20, 20),
            "llama1.1b": B.placement_spread("llama1.1b", args.k, D.F16, 20, 20)}
        out["mixed_precision"] = B.mixed_precision(4, 20)
        out["param_groups"] = {
            "config": {"workload": "llama150m and llama1.1b x %d workers, 3 parameter groups (norm "
                                   "vectors and embeddings exempt from weight decay), 50 / 20 inner "
                                   "launches" % args.k},
            "llama150m": B.quick("llama150m", args.k, n_inner=50, n_outer=0, groups=True)["inner"],
            "llama1.1b": B.quick("llama1.1b", args.k, n_inner=20, n_outer=0, groups=True)["inner"]}
        # the paper's ablations: 1, 2, 4, 8 workers; H = 50, 125 (and 500 above); 4 workers at 1.1B
        out["k_sweep"] = {"workload": "llama150m, FP32 pseudo-gradient, 30 inner + 20 outer launches",
                          **{"k=%d" % kk: B.quick("llama150m", kk, n_inner=30, n_outer=20)
                             for kk in (1, 2, 4, 8)}}
        out["h_sweep"] = {"workload": "llama150m x %d workers, one timed round after a short warm-up "
                                      "round, then 19 more outer steps" % args.k,
                          **{"H=%d" % h: B.rounds("llama150m", args.k, h, pg, 1, 1, warmup_inner=5,
                                                  extra_outer=19)
                             for h in (50, 125)}}
        out["llama1.1b_x4"] = dict(B.quick("llama1.1b", 4, pg=D.F16, n_inner=20, n_outer=20),
                                   config="llama1.1b x 4 workers (the paper's 1.1B run), f16 "
                                          "pseudo-gradient, 20 inner + 20 outer launches")
        out["pg_modes"] = {"workload": "llama150m x %d workers, outer step only, 20 launches" % args.k,
                           **{nm: B.quick("llama150m", args.k, pg=p, round_mean=rm, n_inner=0,
                                          n_outer=20)["outer"]
                              for nm, p, rm in (("f32", D.F32, 0), ("f16", D.F16, 0),
                                                ("f16+rounded_mean", D.F16, 1), ("bf16", D.BF16, 0),
                                                ("bf16+rounded_mean", D.BF16, 1))}}
        out["outer_template_vs_runtime_k"] = {
            "workload": "llama150m, FP32 pseudo-gradient, 20 outer launches; the kernel templated "
                        "on k against the run-time-k kernel at the same k",
            **{"k=%d" % kk: {"template": B.quick("llama150m", kk, n_inner=0, n_outer=20)["outer"],
                             "runtime_k": B.quick("llama150m", kk, n_inner=0, n_outer=20,
                                                  tune=dict(outer_anyk=1))["outer"]}
               for kk in (4, 8)}}
        out["data_dependence"] = {
            "workload": "llama150m x %d workers, FP32 pseudo-gradient, 20 + 20 launches: the same "
                        "kernels on all-zero weights and gradients against the synthetic values; "
                        "what the memory system sustains depends on the data" % args.k,
            "zeros": B.quick("llama150m", args.k, zeros=True),
            "synthetic": B.quick("llama150m", args.k)}
        out["layout_modes"] = {
            "workload": "k = %d, 20 inner + 20 outer launches per arena order; the automatic choice "
                        "is buffer-major for the 150M set (0.87 GiB slots) and worker-major for the "
                        "1.1B set (4.1 GiB slots)" % args.k,
            **{"%s_%s" % (nm, mode_name): B.quick(nm, args.k, pg=p, layout_mode=mode)
               for nm, p in (("llama150m", pg), ("llama1.1b", D.F16))
               for mode, mode_name in ((D.LAYOUT_BUFFER_MAJOR, "buffer_major"),
                                       (D.LAYOUT_WORKER_MAJOR, "worker_major"))}}
        out["stream_patterns"] = B.stream_patterns()
        out["delayed_outer"] = {"llama150m": B.delayed_outer("llama150m", args.k, pg, 4, 20),
                                "llama1.1b": B.delayed_outer("llama1.1b", args.k, D.F16, 2, 20)}
        out["tiny"] = dict(B.rounds("tiny", 2, 4, D.F32, 20, 2),
                           note="0.79M parameters x 2 workers: cache-resident and launch-bound, "
                                "reported for completeness, not roofline-meaningful")
        out["tiny_graph"] = B.tiny_graph(2, 4, 200)
    if not args.no_cpu:
        cb = cpu_baseline(args.k)
        n = main_res["n_params"]
        cb["inner_step_ms_extrapolated_to_workload"] = cb["inner_ns_per_element_worker"] * n * args.k / 1e6
        cb["outer_step_ms_extrapolated_to_workload"] = cb["outer_ns_per_element"] * n / 1e6
        out["cpu_baseline"] = cb
    print(json.dumps(out))


if __name__ == "__main__":
    main()
