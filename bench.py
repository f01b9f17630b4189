#!/usr/bin/env python3
"""Throughput of the batched joint CTC/attention beam-search path on one MI355X.

One benchmark "step" is one whole decode of one batch: ingest of the CTC posteriors
(ctcbs_create for the first batch, ctcbs_reset -- the same work without the allocations -- for
every later one) -> ctcbs_step until every utterance has finished -> ctcbs_finalize.  All inputs
are synthetic and already resident in HBM when the timed region starts: the CTC
log-posteriors come from the device generator, and the attention rows of every step are
recorded once, in an untimed decode with the same generator keyed by the hypotheses'
prefixes, and replayed from HBM in the timed decodes (decoding is deterministic, so every
timed decode takes the recorded path; this is checked).

Prints ONE JSON line (see the design doc for the fields).
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np  # noqa: E402

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--poll-every", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=24, help="utterances in the oracle's timed sample")
    ap.add_argument("--utts", type=int, default=0, help="override the workload's utterances per batch")
    ap.add_argument("--inflight", type=int, default=1,
                    help="batches decoded concurrently, each on its own handle and stream (offline decoding "
                         "always has more batches queued); the default 1 is the headline figure")
    ap.add_argument("--threads", type=int, default=1,
                    help="host threads that drive the batches in flight (ctcbs_run_many)")
    ap.add_argument("--no-offline", action="store_true",
                    help="skip the extra 'offline' figure (8 batches in flight, 4 host threads) of the default run")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the benchmark line: decode the workload under the paper's window "
                         "settings (Table 'batch decoding': M1 = 5, M2 in {inf, 60, 40, 20}), the per-hypothesis "
                         "and the batch-wide window, and print a table (terms, time, agreement with the "
                         "unrestricted decode)")
    ap.add_argument("--job", action="store_true",
                    help="instead of the benchmark line: decode a whole offline job shaped like the workload's "
                         "recordings (cfg3: 32 synthetic long recordings cut into segments, sorted by length, "
                         "batches of the workload's size, --inflight batches in flight on --threads host threads) "
                         "and print one JSON line for the job")
    ap.add_argument("--floor", action="store_true",
                    help="instead of the benchmark line: time the measurement kernels of csrc/probe.hip -- launches "
                         "with the score kernel's shape that perform its chain of dependent loads (record, "
                         "attention row, candidate columns) and next to no arithmetic -- and a sweep of empty launches")
    ap.add_argument("--floor-live", type=float, default=0.475,
                    help="--floor: fraction of the (utterance, beam) slots that hold a hypothesis (0.475 is the "
                         "average over a cfg2 decode, 0.86 its value at step 60)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (known traffic, for scaling rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class Batch:
    """Device-resident synthetic batch plus the recorded attention rows of its decode."""

    def __init__(self, w, poll_every, lens=None, t_max=None):
        import torch
        import gen
        import paper_2101_05600_amd as m
        self.torch, self.gen, self.m, self.w = torch, gen, m, w
        self.U, self.Wb, self.V = w["n_utt"], w["beam"], w["vocab"]
        self.lens = gen.workload_lengths(w) if lens is None else np.asarray(lens, np.int32)
        self.t_max = int(self.lens.max()) if t_max is None else int(t_max)
        self.poll_every = poll_every
        self.stream = torch.cuda.current_stream().cuda_stream
        self.d_lens = torch.from_numpy(self.lens).cuda()
        self.d_ctc = torch.empty((self.U, self.t_max, self.V), dtype=torch.float32, device="cuda")
        rc = gen.dev().gen_dev_ctc(w["seed"], self.U, self.d_lens.data_ptr(), self.t_max, self.V,
                                   w["blank_id"], w["blank_boost"], w["p_boost"], w["zipf_s"],
                                   self.d_ctc.data_ptr(), self.stream)
        assert rc == 0, f"gen_dev_ctc: hip error {rc}"
        torch.cuda.synchronize()
        # timed decodes keep the per-candidate arrays on chip; the recording decode leaves them in
        # device memory for an observer (the full-size parity tests read them with ctcbs_peek)
        kw = {k: v for k, v in w.items() if k not in ("n_utt", "stream", "keep_candidates")}
        self.cfg = m.make_config(n_utt=self.U, t_max=self.t_max, poll_every=poll_every,
                                 stream=self.stream, keep_candidates=0, **kw)
        self.cfg_rec = m.make_config(n_utt=self.U, t_max=self.t_max, poll_every=poll_every,
                                     stream=self.stream, keep_candidates=1, **kw)
        self.l_cap = int(max(self._cap(int(t)) for t in self.lens))
        self.att = None
        self.n_steps = 0
        self.h = None

    def _cap(self, T):
        w = self.w
        l = T
        if w["max_len_ratio"] > 0:
            l = min(l, int(np.floor(np.float32(w["max_len_ratio"]).astype(np.float64) * T)))
        if w["max_len_abs"] > 0:
            l = min(l, w["max_len_abs"])
        return max(l, 1)

    def record(self, observer=None):
        """Untimed decode that produces (and keeps) every step's attention rows.
        observer(step, att_rows_of_step, handle, step_out): optional hook after every step (tests)."""
        torch, m, gen, w = self.torch, self.m, self.gen, self.w
        U, Wb, V = self.U, self.Wb, self.V
        self.att = torch.empty((self.l_cap, U, Wb, V), dtype=torch.float32, device="cuda")
        hashes = [torch.zeros((U, Wb), dtype=torch.int64, device="cuda") for _ in range(2)]
        h = m.ctcbs_create(self.cfg_rec if observer is not None else self.cfg, self.d_ctc, self.lens)
        out = m.StepOut()
        G = gen.dev()
        step = 0
        try:
            while step < self.l_cap:
                step += 1
                rc = G.gen_dev_att_step(w["seed"], step, U, Wb, V, w["att_scale"],
                                        hashes[(step - 1) & 1].data_ptr(),
                                        out.d_parent if step > 1 else None,
                                        out.d_token if step > 1 else None,
                                        out.d_live if step > 1 else None,
                                        hashes[step & 1].data_ptr(), self.att[step - 1].data_ptr(),
                                        self.stream)
                assert rc == 0, f"gen_dev_att_step: hip error {rc}"
                if m.ctcbs_step(h, self.att[step - 1], out) == m.DONE:
                    step -= 1
                    break
                if observer is not None:
                    observer(step, self.att[step - 1], h, out)
                if m.ctcbs_poll(h) == U:           # untimed pass: blocking, exact
                    break
            self.n_steps = step
            self.att_ptr = [self.att[i].data_ptr() for i in range(self.l_cap)]
            res = m.ctcbs_finalize(h, U, self.l_cap, want_frames=observer is not None)
            stats = m.ctcbs_stats(h)
        finally:
            m.ctcbs_destroy(h)
        self.ref = res
        self.cells, self.groups, _ = stats
        return res

    def decode(self, profile=False):
        """One timed-style decode replaying the recorded rows; returns (result, handle stats)."""
        m, U = self.m, self.U
        # one handle serves every decode: the first call allocates, later ones re-initialise it for
        # the next batch (ctcbs_reset: transposed ingest of the posteriors + empty beams, no allocation)
        if self.h is None:
            self.h = m.ctcbs_create(self.cfg, self.d_ctc, self.lens)
        else:
            m.ctcbs_reset(self.h, self.d_ctc, self.lens)
        h = self.h
        out = m.StepOut()
        try:
            if profile:
                m.ctcbs_profile(h, True)
            # the loop a caller without foreknowledge runs: step until the library reports that every
            # utterance has finished (it looks every poll_every steps without draining the stream)
            for step in range(1, self.l_cap + 1):
                if m.ctcbs_step(h, self.att_ptr[min(step, self.n_steps) - 1], out) == m.DONE:
                    break
                if out.n_finished == U:
                    break
            res = m.ctcbs_finalize(h, U, self.l_cap)
            prof = m.ctcbs_profile_read(h) if profile else None
        except Exception:
            m.ctcbs_destroy(h)
            self.h = None
            raise
        return res, prof

    def close(self):
        if self.h is not None:
            self.m.ctcbs_destroy(self.h)
            self.h = None
        for h in getattr(self, "hs", []):
            self.m.ctcbs_destroy(h)
        self.hs = []

    def decode_queue(self, n_slots, n_jobs, threads=1):
        """n_jobs decodes of the same batch, n_slots of them in flight at once (one handle and one
        stream each), driven by the library's own executor (ctcbs_run_queue: `threads` host threads
        share the handles; every job re-ingests the posteriors with ctcbs_reset, is stepped with the
        recorded rows served by ctcbs_att_replay, and ends with ctcbs_finalize)."""
        m, torch, U = self.m, self.torch, self.U
        if len(getattr(self, "hs", [])) != n_slots:
            for h in getattr(self, "hs", []):
                m.ctcbs_destroy(h)
            self.streams = [torch.cuda.Stream() for _ in range(n_slots)]
            self.hs = []
            for st in self.streams:
                cfg = m.make_config(n_utt=self.U, t_max=self.t_max, poll_every=self.poll_every,
                                    stream=st.cuda_stream, keep_candidates=0,
                                    **{k: v for k, v in self.w.items() if k not in ("n_utt", "stream")})
                self.hs.append(m.ctcbs_create(cfg, self.d_ctc, self.lens))
        results = [None] * n_jobs

        def job_fn(job, slot, h, phase):
            if phase == m.JOB_LOAD:
                m.ctcbs_reset(h, self.d_ctc, self.lens)
            else:
                results[job] = m.ctcbs_finalize(h, U, self.l_cap)
        m.ctcbs_run_queue(self.hs, n_jobs, job_fn, replay=[self.att_ptr[:self.n_steps]] * n_jobs,
                          n_threads=threads)
        return results


def cpu_baseline(batch, n_sample):
    """The oracle, free-running, on the first n_sample utterances of the same batch (their CTC
    posteriors are the device bytes copied back); only oracle calls are timed."""
    import gen
    import oracle
    w = batch.w
    n = min(n_sample, batch.U)
    x = batch.d_ctc[:n].cpu().numpy()
    kw = {k: w[k] for k in (
        "vocab", "beam", "blank_id", "eos_id", "cand_k", "win_m1", "win_m2", "ctc_weight",
        "length_bonus", "max_len_ratio", "max_len_abs", "end_flags", "end_m", "end_d", "end_c",
        "eos_run")}
    kw["win_union"] = w.get("win_union", 0)
    for k in ("ctc_weight", "length_bonus", "max_len_ratio", "end_d"):
        kw[k] = float(np.float32(kw[k]))          # the values the fp32 fields of the C ABI carry
    cfg = oracle.make_cfg(**kw)
    L = oracle.lib()
    # every host core this job may use: the GPU machine hands each job a share of its cores and says so through
    # OMP_NUM_THREADS; without that, all the cores the OS shows
    host_cpus = os.cpu_count() or 1
    share = int(os.environ.get("OMP_NUM_THREADS", "0")) or host_cpus
    cores = max(1, min(host_cpus, share, n))
    cpu_model = "unknown"
    try:
        for ln in open("/proc/cpuinfo"):
            if ln.startswith("model name"):
                cpu_model = ln.split(":", 1)[1].strip()
                break
    except OSError:
        pass

    def run(utt_ids, threads):
        os.environ["OMP_NUM_THREADS"] = str(threads)
        utts = [oracle.OracleUtt(x[u, :batch.lens[u]], cfg) for u in utt_ids]
        arr = (ctypes.c_void_p * len(utts))(*[o.h for o in utts])
        fin = np.zeros(len(utts), np.int32)
        Wb, V = w["beam"], w["vocab"]
        basis = gen.prefix_hash([])
        t_or = 0.0
        step = 0
        while not all(o.finished for o in utts):
            step += 1
            ids, hs = [], []
            for i, o in enumerate(utts):
                for j in range(Wb):
                    hyp = o.hyp(j) if not o.finished else None
                    ids.append(utt_ids[i])
                    hs.append(gen.prefix_hash(hyp["labels"]) if hyp and hyp["live"] else basis)
            att = gen.att_rows(w["seed"], ids, step, hs, V, w["att_scale"])
            t0 = time.perf_counter()
            L.orc_batch_step_auto(arr, len(utts), att.ctypes.data_as(ctypes.c_void_p),
                                  fin.ctypes.data_as(ctypes.c_void_p))
            t_or += time.perf_counter() - t0
        return sum(o.cells for o in utts), t_or, len(utts)

    L.orc_set_threads.argtypes = [ctypes.c_int]
    L.orc_set_threads(1)
    c1, t1, n1 = run(list(range(min(3, n))), 1)
    L.orc_set_threads(cores)
    cN, tN, nN = run(list(range(n)), cores)
    return {"value": cN / tN, "unit": "cells/s", "cores": cores, "kind": "oracle",
            "cpu_model": cpu_model, "host_cpus": host_cpus,
            "cores_note": "all cores of this job's share of the host (OMP_NUM_THREADS as set on the box, "
                          "else every core the OS shows), capped by the utterances in the sample",
            "sample": f"first {nN} of {batch.U} utterances of the same batch, whole decodes, "
                      f"free-running with host-generated attention rows; oracle calls only "
                      f"({tN:.2f} s on {cores} threads)",
            "utterances_per_sec": nN / tN,
            "single_thread": {"value": c1 / t1, "utterances_per_sec": n1 / t1, "utterances": n1,
                              "seconds": t1}}


def sweep(a):
    """Window ablation on the synthetic stand-in workload (no transcripts exist, so agreement with the
    unrestricted decode takes the place of the paper's CER column)."""
    import torch
    import gen
    rows = []
    ref = None
    variants = [("unrestricted", -1, -1, 0), ("M1=5, M2=inf", 5, -1, 0), ("M1=5, M2=60", 5, 60, 0),
                ("M1=5, M2=40", 5, 40, 0), ("M1=5, M2=20", 5, 20, 0), ("M1=M2=50", 50, 50, 0),
                ("M1=5, M2=60, batch-wide window", 5, 60, 1), ("M1=M2=50, batch-wide window", 50, 50, 1)]
    for name, m1, m2, uni in variants:
        w = gen.workload(a.workload)
        if a.utts > 0:
            w["n_utt"] = a.utts
        w.update(win_m1=m1, win_m2=m2, win_union=uni)
        b = Batch(w, a.poll_every)
        tok, nt, sc, _, _ = b.record()
        b.decode()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(max(a.steps // 4, 3)):
            b.decode()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / max(a.steps // 4, 3) * 1e3
        if ref is None:
            ref = (tok, nt, sc)
        same = [int(nt[u] == ref[1][u] and np.array_equal(tok[u, :nt[u]], ref[0][u, :nt[u]])) for u in range(b.U)]
        dsc = [abs(float(sc[u]) - float(ref[2][u])) for u in range(b.U) if same[u]]
        rows.append((name, b.cells, b.n_steps, ms, sum(same) / b.U, max(dsc) if dsc else float("nan")))
        b.close()
        del b
        torch.cuda.empty_cache()
    print(f"| window ({a.workload}) | prefix-score terms per decode | steps | ms per decode | same transcript as "
          f"unrestricted | max score difference (same transcript) |")
    print("|---|---|---|---|---|---|")
    for r in rows:
        print(f"| {r[0]} | {r[1]:.3e} | {r[2]} | {r[3]:.2f} | {100 * r[4]:.1f} % | {r[5]:.2e} |")


def run_job(a):
    """A whole offline job (Sec. 4.2 / 4.4 of the paper: segments sorted by length, decoded batch by
    batch, several batches in flight).  Segment lengths come from the synthetic recordings of the
    workload; every batch has its own posteriors and its own recorded attention rows, all resident in
    HBM before the timed region; the last batch is filled up with unused slots (length 0)."""
    import torch
    import gen
    import paper_2101_05600_amd as m
    w = gen.workload(a.workload)
    if a.utts > 0:
        w["n_utt"] = a.utts
    U = w["n_utt"]
    seg = gen.segments(w["seed"])
    order, begin = m.ctcbs_plan_batches(seg, U)
    t_max = int(seg.max())
    batches = []
    for j in range(len(begin) - 1):
        ids = order[begin[j]:begin[j + 1]]
        lens = np.zeros(U, np.int32)
        lens[:len(ids)] = seg[ids]
        b = Batch(dict(w, seed=w["seed"] + 7919 * (j + 1)), a.poll_every, lens=lens, t_max=t_max)
        b.record()
        batches.append(b)
    n_slots = max(a.inflight, 1)
    l_cap = max(b.l_cap for b in batches)
    streams = [torch.cuda.Stream() for _ in range(n_slots)]
    hs = []
    for st in streams:
        cfg = m.make_config(n_utt=U, t_max=t_max, poll_every=a.poll_every, stream=st.cuda_stream, keep_candidates=0,
                            **{k: v for k, v in w.items() if k not in ("n_utt", "stream")})
        hs.append(m.ctcbs_create(cfg, batches[0].d_ctc, batches[0].lens))
    results = [None] * len(batches)

    def job_fn(job, slot, h, phase):
        if phase == m.JOB_LOAD:
            m.ctcbs_reset(h, batches[job].d_ctc, batches[job].lens)
        else:
            results[job] = m.ctcbs_finalize(h, U, l_cap)

    def one_pass():
        m.ctcbs_run_queue(hs, len(batches), job_fn, replay=[b.att_ptr[:b.n_steps] for b in batches],
                          n_threads=a.threads)
    try:
        for _ in range(max(a.warmup, 1)):
            one_pass()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            one_pass()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / a.steps
    finally:
        for h in hs:
            m.ctcbs_destroy(h)
    for b, r in zip(batches, results):
        n = int((b.lens > 0).sum())
        c = min(r[0].shape[1], b.ref[0].shape[1])            # token capacity differs (job-wide / the batch's own)
        same = (np.array_equal(r[0][:n, :c], b.ref[0][:n, :c]) and np.array_equal(r[1][:n], b.ref[1][:n])
                and np.array_equal(r[2][:n], b.ref[2][:n]))
        assert same, "a queued decode did not reproduce the lone decode of its batch"
    cells = sum(b.cells for b in batches)
    frames = int(seg.sum())
    audio_s = frames * 4 / 100.0                  # 4x-subsampled 100 frames/s features
    print(json.dumps({
        "metric": "whole offline job: segments/s and prefix-score cells/s", "value": len(seg) / dt,
        "unit": "segments/s", "cells_per_sec": cells / dt, "job_seconds": dt, "n_gpus": 1, "steps": a.steps,
        "warmup": max(a.warmup, 1), "higher_is_better": True, "dtype": "f32", "data": "synthetic",
        "audio_hours": audio_s / 3600.0, "audio_seconds_per_second": audio_s / dt,
        "config": {"workload": f"{a.workload} job: {len(seg)} segments of {int(seg.min())}-{t_max} frames from 32 "
                               f"synthetic recordings, sorted by length, {len(batches)} batches of {U} (last one "
                               f"{int((batches[-1].lens > 0).sum())} used slots), V={w['vocab']}, beam {w['beam']}, "
                               f"top-{w['cand_k']}, window {w['win_m1']}/{w['win_m2']}; decoding path only "
                               f"(posteriors and recorded attention rows resident in HBM)",
                   "batches_in_flight": n_slots, "host_threads": a.threads,
                   "decode_steps_total": sum(b.n_steps for b in batches), "cells_per_job": cells}}))


def read_profile_summary(path):
    """(HBM bytes per launch, the kernel's own average duration in us, when and on what it was measured) from a
    committed counter summary under profiles/, None for what the file does not hold."""
    traffic, prof_us, prof_when = None, None, None
    if os.path.exists(path):
        for ln in open(path):
            if ln.startswith("traffic_bytes_per_launch:"):
                traffic = float(ln.split(":")[1].split()[0])
            elif ln.startswith("rocprof_avg_launch_us:"):
                prof_us = float(ln.split(":")[1].split()[0])
            elif ln.startswith("measured:"):
                prof_when = ln.split(":", 1)[1].strip()
    return traffic, prof_us, prof_when


def floor(a):
    """Latency floor of one score launch at the headline shape (U=64, beam 10, V=5000, top-40, window
    50/50): the chain of dependent loads alone.  Synthetic buffers of the real sizes; every repetition
    reads attention rows and candidate columns it has not touched before, and the records are rewritten by
    a small kernel between launches (as the select kernel does in a decode).  Prints a table: average
    launch-to-launch period of back-to-back dependent launches on one stream (HIP events around the
    whole series), which is what a decode pays per launch.  Per-kernel durations come from running this
    under rocprofv3 --kernel-trace (the kernels of each level have their own names)."""
    import torch
    import paper_2101_05600_amd as m
    P = m.probe_lib()
    w = __import__("gen").workload(a.workload)
    U, Wb, V, K = (a.utts or w["n_utt"]), w["beam"], w["vocab"], w["cand_k"]
    T = 875
    Tp = ((T + 5 + 31) // 32) * 32
    G = U * Wb
    reps = 24
    st = torch.cuda.current_stream().cuda_stream
    gcpu = torch.Generator().manual_seed(1234)
    att = torch.randn((8, G, V), device="cuda")
    xT = torch.empty((U, V, Tp), device="cuda").normal_()
    cand = torch.randint(1, V - 1, (reps, G, K), generator=gcpu, dtype=torch.int32).cuda()
    sink = torch.zeros(G * 4, device="cuda")
    out = []
    for live_frac in (a.floor_live,):
        rec = np.zeros((G, 16), np.int32)                # 64-byte records: live, last, rs, re, tau, tau_end, ref, pad, 4 doubles
        rng = np.random.default_rng(7)
        rec[:, 0] = rng.random(G) < live_frac
        tau = rng.integers(60, T - 60, G)
        rec[:, 2] = 0; rec[:, 3] = T; rec[:, 4] = tau; rec[:, 5] = tau + 2; rec[:, 6] = tau
        rec_src = torch.from_numpy(rec).cuda()
        rec_dst = torch.empty_like(rec_src)
        for level in range(4):
            def series(n):
                for r in range(n):
                    P.probe_touch(rec_src.data_ptr(), rec_dst.data_ptr(), G, st)
                    rc = P.probe_chain(level, rec_dst.data_ptr(), att[r % 8].data_ptr(), xT.data_ptr(),
                                       cand[r % reps].data_ptr(), sink.data_ptr(), U, Wb, V, Tp, K,
                                       w["win_m1"], w["win_m2"], 15 * 1024, st)
                    assert rc == 0, rc
            series(4)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); series(reps); e1.record()
            torch.cuda.synchronize()
            pair_us = e0.elapsed_time(e1) * 1e3 / reps
            e0.record()
            for r in range(reps):
                P.probe_touch(rec_src.data_ptr(), rec_dst.data_ptr(), G, st)
            e1.record()
            torch.cuda.synchronize()
            touch_us = e0.elapsed_time(e1) * 1e3 / reps
            out.append((live_frac, level, pair_us - touch_us))
    print("| live groups | level | launch-to-launch period, us (touch kernel's own period taken out) |")
    print("|---|---|---|")
    names = ["0 nothing", "1 + record", "2 + attention row", "3 + candidate columns"]
    for lf, lv, us in out:
        print(f"| {int(round(lf * G))} of {G} | {names[lv]} | {us:.2f} |")
    print()
    print("| empty launch: work-groups x threads, LDS bytes, argument bytes | period, us |")
    print("|---|---|")
    for groups, threads, lds, big in ((G, 256, 15 * 1024, 1), (G, 256, 0, 1), (G, 256, 0, 0), (G, 64, 0, 0),
                                      (U, 256, 0, 0), (U, 1024, 0, 0), (8 * G, 256, 15 * 1024, 1), (1, 64, 0, 0)):
        for _ in range(4):
            P.probe_empty(groups, threads, lds, big, st)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(200):
            P.probe_empty(groups, threads, lds, big, st)
        e1.record()
        torch.cuda.synchronize()
        print(f"| {groups} x {threads}, {lds}, {704 if big else 12} | {e0.elapsed_time(e1) * 1e3 / 200:.2f} |")


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this path runs on ONE GPU (utterances are independent; several GPUs would "
              "each run their own batches with nothing exchanged) -- use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import gen
    import paper_2101_05600_amd as m
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    m.lib()
    if a.floor:
        floor(a)
        return
    if a.sweep:
        sweep(a)
        return
    if a.job:
        run_job(a)
        return
    w = gen.workload(a.workload)
    if a.utts > 0:
        w["n_utt"] = a.utts
    b = Batch(w, a.poll_every)
    ref = b.record()
    if a.calib_copy:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)                       # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    if a.inflight > 1:
        b.decode_queue(a.inflight, a.inflight * max(a.warmup, 1), a.threads)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        many = b.decode_queue(a.inflight, a.inflight * a.steps, a.threads)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / a.inflight      # a.steps batches per slot: dt / a.steps = per batch
        res = many[-1]
        for r in many:
            for x, y in zip(r[:3], ref[:3]):
                assert np.array_equal(x, y), "a concurrent decode did not reproduce the recorded decode"
    else:
        for _ in range(a.warmup):
            b.decode()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(a.steps):
            res, _ = b.decode()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
    for x, y in zip(res[:3], ref[:3]):
        assert np.array_equal(x, y), "timed decode did not reproduce the recorded decode"
    ms = dt / a.steps * 1e3
    # dominant kernel: score kernel, HIP events on its own stream, one extra decode
    _, prof = b.decode(profile=True)
    score_ms, select_ms, n_prof = prof
    K = int(w["cand_k"]) if 0 < w["cand_k"] < w["vocab"] - 2 else w["vocab"] - 2
    restricted = 0 < w["cand_k"] < w["vocab"] - 2
    # algorithmic bytes of the score kernel over the decode: candidate columns 4 B per term,
    # the parent's two forward variables 8 B per window frame, the attention row 4V per group
    bytes_score = 4.0 * b.cells + 8.0 * b.cells / K + (4.0 * w["vocab"] * b.groups if restricted else 0.0)
    ach = bytes_score / (score_ms * 1e-3) / 1e9
    # measured HBM bytes per launch of the same kernel (rocprofv3 FETCH_SIZE / WRITE_SIZE, scaled by a
    # plain copy): taken from the committed counter summary, not measurable from inside this process
    tname = f"k_score_{a.workload}_traffic.txt"
    traffic, prof_us, prof_when = (read_profile_summary(os.path.join(ROOT, "profiles", tname))
                                   if a.utts == 0 else (None, None, None))   # read at the workload's own size
    if restricted:
        roof = {"bound": "hbm", "kernel": "k_score", "achieved": ach, "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": ach / HBM_PEAK_GBS, "traffic": traffic,
                "avg_launch_us": score_ms * 1e3 / max(n_prof, 1),
                "avg_launch_us_how": "HIP events on the library's stream around every launch of one extra decode "
                                     "(spans the dispatch gap before the kernel: reads about 2 us more than the "
                                     "kernel's own duration)",
                "algorithmic_bytes_per_launch": bytes_score / max(n_prof, 1),
                "select_kernel_avg_us": select_ms * 1e3 / max(n_prof, 1),
                # from the committed rocprofv3 summary (a profiler cannot run inside this process): the
                # kernel's own average duration, the fraction of the roof it gives, and what the HBM counters read
                "rocprof": {"avg_launch_us": prof_us,
                            "frac": (bytes_score / max(n_prof, 1) / (prof_us * 1e-6) / 1e9 / HBM_PEAK_GBS) if prof_us else None,
                            "traffic_bytes_per_launch": traffic, "source": "profiles/" + tname,
                            "measured": prof_when}}
    else:
        # every id a candidate: the beam slots of an utterance share each posterior column, bytes fall
        # to 4/Wb per term and the bound is the plain ALUs.  Per term one fused multiply-add, one
        # exp2, one add = 4 flop; the exp2 issues at quarter rate, so the three instructions take 6
        # issue slots: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz / 6 = 6.55e12 terms/s = 26.2 TFLOP/s is
        # the most this instruction mix can reach (the chip's 157.3 TFLOP/s needs an FMA in every slot)
        tf = 4.0 * b.cells / (score_ms * 1e-3) / 1e12
        peak = 256 * 4 * 16 * 2.4e9 / 6.0 * 4.0 / 1e12
        terms_per_s = b.cells / (score_ms * 1e-3)
        roof = {"bound": "alu", "kernel": "k_score_dense", "achieved": tf, "peak": peak, "unit": "TFLOP/s",
                "frac": tf / peak, "traffic": None, "avg_launch_us": score_ms * 1e3 / max(n_prof, 1),
                "flop_per_term": 4, "select_kernel_avg_us": select_ms * 1e3 / max(n_prof, 1),
                "peak_how": "instruction-mix ceiling derived from the unit counts, not a published chip peak: "
                            "256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz / 6 issue slots per term x 4 flop",
                # the same rate against the chip's own figures: one exp2 per term against the transcendental
                # rate (quarter rate: 256 x 4 x 16 x 2.4e9 / 4 per second), and 4 flop per term against the
                # published fp32 vector peak
                "frac_of_transcendental_rate": terms_per_s / (256 * 4 * 16 * 2.4e9 / 4.0),
                "frac_of_fp32_vector_peak": tf / 157.3}
    line = {
        "metric": "CTC prefix-score cells/sec (utt·beam·cand·frame) + utterances/sec at B=64",
        "value": b.cells / (dt / a.steps), "unit": "cells/s",
        "utterances_per_sec": b.U / (dt / a.steps),
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{a.workload}: U={b.U} utterances, T in [{int(b.lens.min())},{int(b.lens.max())}], "
                               f"V={b.V}, beam {b.Wb}, top-{K} candidates, window M1={w['win_m1']} "
                               f"M2={w['win_m2']}, end_flags={w['end_flags']}; one step = one whole "
                               f"batch decode (create + {b.n_steps} beam-search steps + finalize)",
                   "decode_steps": b.n_steps, "cells_per_decode": b.cells,
                   "poll_every": a.poll_every, "batches_in_flight": a.inflight,
                   "host_threads": a.threads if a.inflight > 1 else 1},
        "roofline": roof,
    }
    if a.inflight == 1 and not a.no_offline and a.utts == 0 and restricted and w["n_utt"] <= 64:
        # the same work when several such batches are decoded as ONE batch of n x U utterances on one handle (one
        # launch per step over all their groups): the lone batch above stays the headline, these say what
        # the score kernel does as the launch grows from latency-bound towards memory-bound
        def multi(n):
            wm = dict(w, n_utt=n * w["n_utt"])
            bm = Batch(wm, a.poll_every)
            bm.record()
            for _ in range(2):
                bm.decode()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                bm.decode()
            torch.cuda.synchronize()
            dtm = (time.perf_counter() - t0) / 5
            _, pm = bm.decode(profile=True)
            bytes_m = 4.0 * bm.cells + 8.0 * bm.cells / K + 4.0 * w["vocab"] * bm.groups
            ach_m = bytes_m / (pm[0] * 1e-3) / 1e9
            out = {"utterances": bm.U, "how": "one handle, one batch of %d x %d utterances of the same recipe" % (n, w["n_utt"]),
                   "ms_per_decode": dtm * 1e3, "utterances_per_sec": bm.U / dtm, "value": bm.cells / dtm,
                   "unit": "cells/s", "decode_steps": bm.n_steps,
                   "roofline": {"bound": "hbm", "kernel": "k_score", "achieved": ach_m, "peak": HBM_PEAK_GBS,
                                "unit": "GB/s", "frac": ach_m / HBM_PEAK_GBS,
                                "avg_launch_us": pm[0] * 1e3 / max(pm[2], 1),
                                "algorithmic_bytes_per_launch": bytes_m / max(pm[2], 1),
                                "select_kernel_avg_us": pm[1] * 1e3 / max(pm[2], 1)}}
            bm.close()
            del bm
            torch.cuda.empty_cache()
            return out
        line["multi_batch"] = multi(8)
        line["multi_batch_32"] = multi(32)
    if a.inflight == 1 and not a.no_offline:
        # context, not the headline: a queue of copies of the same batch, 8 in flight (own handle and
        # stream each), driven by the library's executor on 4 host threads -- what an offline run with a queue of
        # batches gets out of the chip
        nf, nt, reps = 8, 4, max(2, a.steps // 4)
        b.decode_queue(nf, nf, nt)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        many = b.decode_queue(nf, nf * reps, nt)
        torch.cuda.synchronize()
        dto = (time.perf_counter() - t0) / (reps * nf)
        for r in many:
            for x, y in zip(r[:3], ref[:3]):
                assert np.array_equal(x, y), "a concurrent decode did not reproduce the recorded decode"
        line["offline"] = {"batches_in_flight": nf, "host_threads": nt, "ms_per_batch": dto * 1e3,
                           "utterances_per_sec": b.U / dto, "value": b.cells / dto, "unit": "cells/s"}
    if not a.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(b, a.cpu_sample)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
