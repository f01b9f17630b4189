"""Child process of tests/test_cpu_emulation.py: decodes small batches with the CPU build of the
kernels (argv[1] = its shared library), every step compared with the oracle exactly as the GPU
tests do.  Prints "emu ok <name>" per case; any sanitizer report or mismatch ends it with a non-zero
status."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import numpy as np  # noqa: E402

import paper_2101_05600_amd as m  # noqa: E402

m._SO = sys.argv[1]          # the binding loads this instead of the GPU library (tests only)

import gen  # noqa: E402
from helpers import EmuDecoder, lockstep_decode  # noqa: E402

CASES = {
    # split select kernel, 16-lane score kernel, eos-run rule, an unused slot
    "windowed": (dict(n_utt=3, vocab=40, beam=3, cand_k=6, win_m1=5, win_m2=5, end_flags=7, eos_run=2,
                      max_len_ratio=0.4), [12, 0, 18]),
    # per-utterance select kernel (batch-wide window), 64-lane score kernel (no end margin)
    "batch_window": (dict(n_utt=2, vocab=36, beam=2, cand_k=5, win_m1=4, win_m2=-1, win_union=1, end_flags=3,
                          max_len_ratio=0.4), [15, 10]),
    # every id a candidate: all-candidates score kernel, list builder from registers
    "all_candidates": (dict(n_utt=1, vocab=12, beam=2, cand_k=0, win_m1=-1, win_m2=-1, end_flags=3,
                            max_len_ratio=0.4), [11]),
    # fewer ids than beam slots: most slots never hold a hypothesis, their records are never written
    "all_candidates_few_ids": (dict(n_utt=2, vocab=6, beam=6, cand_k=0, win_m1=-1, win_m2=-1, end_flags=3,
                                    max_len_ratio=0.4), [9, 7]),
    # a vocabulary large enough for the register-resident candidate selection to succeed (pivot, per-wave
    # stretches of the short list, ranking), eos-run rule armed, list ranked by one wave
    "pivot": (dict(n_utt=1, vocab=2048, beam=2, cand_k=12, win_m1=6, win_m2=6, end_flags=7, eos_run=3,
                   max_len_ratio=0.3), [16]),
    # more than 64 candidates per hypothesis: the group's list is ranked by the whole work-group
    "pivot_k80": (dict(n_utt=1, vocab=1024, beam=2, cand_k=80, win_m1=-1, win_m2=-1, end_flags=3,
                       max_len_ratio=0.3), [12]),
    # eos-run rule armed with more candidates than one wave ranks: the kernel form that carries the rule's
    # work-group-wide path (second sum in the column pass, test across all waves)
    "k80_eos_run": (dict(n_utt=2, vocab=1024, beam=2, cand_k=80, win_m1=6, win_m2=6, end_flags=7, eos_run=3,
                         max_len_ratio=0.4), [14, 9]),
    # a vocabulary beyond 65535 whose attention rows are constant: the radix selection meets more equal keys
    # than 16 bits count, and the K smallest ids must come out
    "radix_wide_ties": (dict(n_utt=1, vocab=66000, beam=1, cand_k=3, win_m1=-1, win_m2=-1, end_flags=3,
                             max_len_abs=3, max_len_ratio=0.0), [5]),
    # window margins beyond 128 frames: the score kernel's form with four float4 per lane in flight, eos-run
    # rule armed (its one-wave walk through the last frames after a two-part sum whose second part is empty)
    "wide_window_eos_run": (dict(n_utt=2, vocab=40, beam=2, cand_k=6, win_m1=70, win_m2=70, end_flags=7, eos_run=3,
                                 max_len_ratio=0.4), [22, 15]),
    # logits in, odd vocabulary (radix selection), one candidate per hypothesis
    "logits_odd_vocab": (dict(n_utt=1, vocab=33, beam=2, cand_k=1, win_m1=3, win_m2=8, end_flags=2, att_is_logits=1,
                              max_len_ratio=0.4), [13]),
}


def executor_case():
    """The job queue on two handles driven by two host threads (ctcbs_run_queue with the replay provider):
    three small batches, each first decoded alone against the oracle; the queue must return the same.
    Under ThreadSanitizer this is the check of the executor's own host code."""
    ws, data, singles, recs = [], [], [], []
    for j, lens in enumerate([[14, 9], [11, 0], [8, 13]]):
        w = gen.workload("cfg1")
        w.update(n_utt=2, vocab=24, beam=2, cand_k=4, win_m1=4, win_m2=4, end_flags=7, eos_run=2,
                 max_len_ratio=0.4, seed=500 + j)
        w["eos_id"] = w["vocab"] - 1
        lens = np.asarray(lens, np.int32)
        g = gen.workload_ctc(w, np.maximum(lens, 1))
        ctc = np.full((2, 14, 24), np.nan, np.float32)
        for u in range(2):
            ctc[u, :lens[u]] = g[u, :lens[u]]
        rows = []
        rep, res = lockstep_decode(w, ctc, lens, check_utts=[u for u in range(2) if lens[u] > 0],
                                   decoder_cls=EmuDecoder, gpu_att_fn=lambda a, rows=rows: rows.append(a.copy()) or a)
        assert rep["max_score_err"] < 1e-4, rep
        ws.append(w); data.append((np.ascontiguousarray(ctc), lens)); singles.append(res); recs.append(rows)
    decs = [EmuDecoder(ws[0], data[0][0], data[0][1], poll_every=2) for _ in range(2)]
    got = [None] * 3
    cap = max(r["tokens"].shape[1] for r in singles)

    def job_fn(job, slot, h, phase):
        if phase == m.JOB_LOAD:
            m.ctcbs_reset(h, data[job][0].ctypes.data, data[job][1])
        else:
            got[job] = m.ctcbs_finalize(h, 2, cap)
    keep = [[np.ascontiguousarray(r) for r in rows] for rows in recs]
    m.ctcbs_run_queue([d.h for d in decs], 3, job_fn, replay=[[r.ctypes.data for r in rows] for rows in keep],
                      n_threads=2)
    for j in range(3):
        tok, nt, sc, frm, fl = got[j]
        c = singles[j]["tokens"].shape[1]
        assert np.array_equal(tok[:, :c], singles[j]["tokens"]) and np.array_equal(nt, singles[j]["ntok"]), j
        assert np.array_equal(sc, singles[j]["score"]), j
    for d in decs:
        d.close()
    print("emu ok executor", flush=True)


def static_step_case():
    """ctcbs_step_static (per-step scratch in the library's fixed array) decodes like ctcbs_step."""
    plain = m.ctcbs_step
    m.ctcbs_step = m.ctcbs_step_static
    try:
        over, lens = CASES["windowed"]
        w = gen.workload("cfg1")
        w.update(over)
        w["eos_id"] = w["vocab"] - 1
        lens = np.asarray(lens, np.int32)
        ctc = gen.workload_ctc(w, np.maximum(lens, 1))
        rep, res = lockstep_decode(w, ctc, lens, check_utts=[u for u in range(len(lens)) if lens[u] > 0],
                                   decoder_cls=EmuDecoder)
        assert rep["max_score_err"] < 1e-4 and res["cells"] == int(res["oracle_cells"]), rep
    finally:
        m.ctcbs_step = plain
    print("emu ok static_step", flush=True)


def main():
    names = sys.argv[2:] or list(CASES)
    if "static_step" in names:
        names.remove("static_step")
        static_step_case()
    if "executor" in names:
        names.remove("executor")
        executor_case()
    for name in names:
        max_steps = None
        if name.startswith("random:"):      # random:<seed of the list>:<case>[:<steps>], tests/random_cases.py
            import random_cases
            parts = name.split(":")
            seed0, case = parts[1], parts[2]
            max_steps = int(parts[3]) if len(parts) > 3 else None
            mode, w, lens = random_cases.case_params(int(case), int(seed0))
            print(random_cases.describe(int(seed0), int(case), mode, w, lens), flush=True)
        else:
            over, lens = CASES[name]
            w = gen.workload("cfg1")
            w.update(over)
            w["eos_id"] = w["vocab"] - 1
        lens = np.asarray(lens, np.int32)
        ctc = gen.workload_ctc(w, np.maximum(lens, 1))
        used = [u for u in range(len(lens)) if lens[u] > 0]
        kw = {}
        if name == "radix_wide_ties":
            flat = lambda a: np.where(np.isnan(a), a, np.float32(-11.0)).astype(np.float32)
            kw = dict(att_fn=flat, gpu_att_fn=flat)
        if w.get("att_is_logits"):
            # the library takes unnormalised scores; the oracle takes their log_softmax
            def to_logits(a):
                return (a * 1.7 + 0.3).astype(np.float32)

            def normalised(a):
                z = to_logits(a).astype(np.float64)
                mx = np.nanmax(z, axis=-1, keepdims=True)
                return (z - (mx + np.log(np.nansum(np.exp(z - mx), axis=-1, keepdims=True)))).astype(np.float32)
            kw = dict(att_fn=normalised, gpu_att_fn=to_logits)
        rep, res = lockstep_decode(w, ctc, lens, check_utts=used, decoder_cls=EmuDecoder, max_steps=max_steps, **kw)
        tol = 2e-4 if w.get("att_is_logits") else 1e-4
        assert rep["max_score_err"] < tol and rep["max_ctc_err"] < tol, (name, rep)
        if max_steps is None:
            assert res["cells"] == int(res["oracle_cells"]), (name, res["cells"], res["oracle_cells"])
        print(f"emu ok {name} steps={rep['utt_steps']} score_err={rep['max_score_err']:.2e}", flush=True)


if __name__ == "__main__":
    main()
