"""Parity at the benchmark's full size and launch configuration (cfg2: U=64, V=5000, beam 10, top-40,
window 50/50, all end rules), on sampled utterances that the oracle follows step by step.

Inputs are the device generator's bytes (the same ones bench.py times), copied back for the oracle."""
import os
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import gen
from helpers import orc_cfg_from
from oracle.lockstep import Lockstep

pytestmark = pytest.mark.gpu


def run_sampled(workload, sample, over=None):
    import bench
    import paper_2101_05600_amd as m
    w = gen.workload(workload)
    if over:
        w.update(over)
    b = bench.Batch(w, poll_every=8)
    U, Wb = b.U, b.Wb
    K = w["cand_k"] if 0 < w["cand_k"] < w["vocab"] - 2 else w["vocab"] - 2
    xs = [b.d_ctc[u, :b.lens[u]].cpu().numpy() for u in sample]
    ls = Lockstep(xs, orc_cfg_from(w), utt_ids=sample)
    g = lambda p, shape, dt: m.view(p, shape, dt).cpu().numpy()

    def observer(step, att_step, h, o):
        out = dict(parent=g(o.d_parent, (U, Wb), np.int32), token=g(o.d_token, (U, Wb), np.int32),
                   score=g(o.d_score, (U, Wb), np.float32), live=g(o.d_live, (U, Wb), np.uint8),
                   finished=g(o.d_finished, (U,), np.uint8), tau=g(o.d_tau, (U, Wb), np.int32),
                   tau_end=g(o.d_tau_end, (U, Wb), np.int32),
                   eos_added=g(o.d_eos_added, (U, Wb), np.uint8),
                   stopped=g(o.d_stopped, (U, Wb), np.uint8))
        pk = lambda what: m.ctcbs_peek(h, what)
        peek = dict(cand_id=pk(m.PEEK_CAND_ID).reshape(U, Wb, K),
                    cand_ctc=pk(m.PEEK_CAND_CTC).reshape(U, Wb, K),
                    cand_joint=pk(m.PEEK_CAND_JOINT).reshape(U, Wb, K),
                    win_s=pk(m.PEEK_WIN_S).reshape(U, Wb), win_e=pk(m.PEEK_WIN_E).reshape(U, Wb),
                    ctc_eos=pk(m.PEEK_CTC_EOS).reshape(U, Wb), joint_eos=pk(m.PEEK_JOINT_EOS).reshape(U, Wb))
        att = {u: att_step[u].cpu().numpy() for u in sample if not ls.utts[sample.index(u)].finished}
        for u in sample:
            att.setdefault(u, None)
        ls.step(att, out, peek)
        if step % 50 == 0:
            print(f"step {step}: {ls.report}", flush=True)

    tok, nt, sc, frm, fl = b.record(observer)
    ls.check_results(tok, nt, sc, fl, frames=frm)
    # the timed path (recorded rows replayed, polling every 8 steps) reproduces the recorded decode
    (tok2, nt2, sc2, _, fl2), _ = b.decode()
    assert np.array_equal(tok, tok2) and np.array_equal(nt, nt2) and np.array_equal(sc, sc2)
    assert all(o.finished for o in ls.utts)
    return ls.report, b


def test_cfg2_full_size_sampled_utterances():
    w = gen.workload("cfg2")
    lens = gen.workload_lengths(w)
    order = np.argsort(lens)
    # a quarter of the batch: the shortest, the longest, the median and every fourth by length in between
    sample = sorted({int(order[0]), int(order[-1]), int(order[len(order) // 2])} | {int(u) for u in order[2::4]})
    assert len(sample) >= 16
    rep, b = run_sampled("cfg2", sample)
    print(rep, "decode steps", b.n_steps, "cells", b.cells)
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4
    assert rep["utt_steps"] > 1500


def test_cfg2_recipe_as_one_batch_of_512_utterances():
    """The multi-batch launch shape of bench.py (eight cfg2 batches as ONE batch: 5120 score work-groups per
    launch, per-utterance select kernel with eight waves per utterance): six utterances followed by the
    oracle through every step."""
    w = gen.workload("cfg2")
    w["n_utt"] = 512
    lens = gen.workload_lengths(w)
    order = np.argsort(lens)
    sample = sorted({int(order[0]), int(order[-1]), int(order[255]), 0, 301, 511})
    rep, b = run_sampled("cfg2", sample, over=dict(n_utt=512))
    print(rep, "decode steps", b.n_steps, "cells", b.cells)
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4
    assert rep["utt_steps"] > 400


def test_cfg3_one_batch_of_meeting_segments():
    """One batch of 128 Korean-meeting-like segments (V=2300), the four longest and shortest followed."""
    seg = gen.segments(2101)
    assert seg.max() <= 500
    w = gen.workload("cfg3")
    lens = seg[-128:]                       # the batch of the 128 longest segments (sorted by length)
    import bench
    orig = gen.workload_lengths
    try:
        gen.workload_lengths = lambda _w: np.ascontiguousarray(lens, dtype=np.int32)
        rep, b = run_sampled("cfg3", [0, 1, 126, 127])
    finally:
        gen.workload_lengths = orig
    print(rep)
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4


def _cfg3_batch(lens, sample):
    orig = gen.workload_lengths
    try:
        gen.workload_lengths = lambda _w: np.ascontiguousarray(lens, dtype=np.int32)
        return run_sampled("cfg3", sample)
    finally:
        gen.workload_lengths = orig


def test_cfg3_short_segment_batch_and_the_last_batch_that_is_not_full():
    """The other ends of the cfg3 job: the batch of the 128 shortest segments, and the job's last batch,
    which holds fewer segments than slots (unused slots have length 0 and stay inert)."""
    import paper_2101_05600_amd as m
    seg = gen.segments(2101)
    rep, b = _cfg3_batch(seg[:128], [0, 1, 64, 127])
    print("shortest", rep)
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4
    order, begin = m.ctcbs_plan_batches(seg, 128)
    ids = order[begin[-2]:begin[-1]]
    assert 0 < len(ids) < 128
    lens = np.zeros(128, np.int32)
    lens[:len(ids)] = seg[ids]
    n = len(ids)
    rep, b = _cfg3_batch(lens, [0, n // 2, n - 1])
    print("last batch", n, "of 128 slots used", rep)
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4
    tok, nt, sc = b.ref[0], b.ref[1], b.ref[2]
    assert (nt[n:] == 0).all() and (sc[n:] < -1e29).all()          # unused slots: no tokens, score log0


def test_cfg4b_full_size_sampled_utterances():
    """U=256 utterances of 1500 frames, beam 20, top-60, window 80/80: the throughput-bound launch
    shape (5120 score work-groups, one-work-group-per-utterance select), two utterances followed
    through all of their ~350 steps."""
    rep, b = run_sampled("cfg4b", [0, 201])
    print(rep, "decode steps", b.n_steps, "cells", b.cells)
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4
    assert rep["utt_steps"] > 500


def test_cfg4a_shape_followed_deep_into_the_utterance():
    """Eq. (3) as it stands at cfg4a's sizes (T = 1500 frames, all 4998 ids, whole-utterance windows): one
    utterance at beam 4 followed for 120 steps, every candidate's prefix score compared at 1e-4.  This is
    the regime in which a candidate's own prefix score lies hundreds of nats below its hypothesis's."""
    rep, b = run_sampled("cfg4a", [0], over=dict(n_utt=2, beam=4, max_len_ratio=0.0, max_len_abs=120))
    print(rep, "decode steps", b.n_steps, "cells", b.cells)
    assert b.n_steps == 120 and rep["utt_steps"] == 120
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4


def test_cfg4a_full_vocabulary_first_steps():
    """U=256, T=1500, beam 20, every id a candidate (4998 per hypothesis), no window: the shape whose
    bound is the ALUs.  The oracle needs seconds per step and utterance here, so one utterance is
    followed and the decode is capped at five steps (utterances are independent: the others run the
    same steps)."""
    rep, b = run_sampled("cfg4a", [77], over=dict(max_len_ratio=0.0, max_len_abs=5))
    print(rep, "decode steps", b.n_steps, "cells", b.cells)
    assert b.n_steps == 5 and rep["utt_steps"] == 5
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4
