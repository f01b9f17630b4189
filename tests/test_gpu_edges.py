"""GPU parity at the edges of the supported range: the smallest and the largest sizes the C ABI
accepts and the degenerate cases of the method, each checked step by step against the oracle
(same protocol and tolerances as test_gpu_parity.py)."""
import numpy as np
import pytest

import gen
from helpers import lockstep_decode
from test_gpu_parity import small, make_inputs

pytestmark = pytest.mark.gpu


def run(w, lens=None, eps=1e-4, **kw):
    if lens is None:
        lens, ctc = make_inputs(w)
    else:
        lens = np.asarray(lens, np.int32)
        ctc = gen.workload_ctc(w, lens)
    rep, res = lockstep_decode(w, ctc, lens, eps=eps, **kw)
    assert rep["max_score_err"] < eps and rep["max_ctc_err"] < eps, rep
    assert res["cells"] == int(res["oracle_cells"])
    return rep, res


def test_smallest_problem():
    """One utterance of one frame, three ids (blank, one label, eos), beam 1: one step."""
    w = small("cfg0", n_utt=1, vocab=3, beam=1, cand_k=0, max_len_abs=5)
    rep, res = run(w, lens=[1])
    assert res["steps"] == 1 and res["ntok"][0] <= 1


def test_one_to_four_frame_utterances_in_a_ragged_batch():
    """Utterances shorter than a float4 of frames beside long ones: the windows' aligned loads
    touch the zero padding, the step caps differ by two orders of magnitude."""
    w = small("cfg1", vocab=64, beam=3, cand_k=10, win_m1=4, win_m2=4, end_flags=7, eos_run=2,
              max_len_ratio=0.5)
    rep, res = run(w, lens=[1, 2, 3, 4, 5, 150, 7, 1, 96])
    assert rep["utt_steps"] > 60


def test_single_candidate_and_eos_only_competition():
    """K = 1: every hypothesis has one extension, the beam fills from different parents only."""
    w = small("cfg1", n_utt=3, t_lo=30, t_hi=60, vocab=200, beam=4, cand_k=1, win_m1=10, win_m2=10, end_flags=3)
    run(w)


def test_widest_beam():
    """Beam 32 (the maximum): 1024 list entries per utterance in the select kernel."""
    w = small("cfg1", n_utt=2, t_lo=40, t_hi=70, vocab=120, beam=32, cand_k=40, win_m1=20, win_m2=20,
              end_flags=7, eos_run=4, max_len_abs=14)
    rep, res = run(w)
    assert rep["utt_steps"] >= 20


def test_longest_utterance_unrestricted_window():
    """t_max at the limit of the ABI (6140 frames), whole-utterance windows (one wave per candidate,
    many passes), few steps.
    The eos score of a hypothesis of a handful of labels on 6140 frames (the probability that the WHOLE
    utterance is those labels) lies some 2000 nats below its prefix score: it only keeps the 1e-4 bar
    because the per-frame reference B_t is carried in fp64 outside the fp32 state."""
    w = small("cfg1", vocab=24, beam=2, cand_k=0, win_m1=-1, win_m2=-1, end_flags=0, max_len_ratio=0.0,
              max_len_abs=6)
    rep, res = run(w, lens=[6140, 517])
    assert res["steps"] == 6


def test_longest_utterance_windowed():
    w = small("cfg1", vocab=24, beam=2, cand_k=8, win_m1=60, win_m2=200, end_flags=4, eos_run=32,
              max_len_ratio=0.0, max_len_abs=6)
    run(w, lens=[6140, 6000])


def test_longest_end_detection_memory():
    """end_m = 8 (the maximum ring of Eq. (4)) and eos_run = 32 (the maximum run)."""
    w = small("cfg1", n_utt=4, t_lo=50, t_hi=120, vocab=300, beam=5, cand_k=12, win_m1=40, win_m2=40,
              end_flags=7, end_m=8, end_d=-3.0, eos_run=32)
    run(w)


def test_lambda_zero_and_one():
    """ctc_weight 0 (attention only: Eq. (1) without its first term) and 1 (CTC only)."""
    for lam in (0.0, 1.0):
        w = small("cfg1", n_utt=2, t_lo=40, t_hi=80, vocab=150, beam=3, cand_k=9, win_m1=15, win_m2=15,
                  end_flags=3, ctc_weight=lam)
        run(w)


def test_degenerate_posteriors():
    """Posteriors that put all mass on blank at every frame (nothing but the empty output has
    probability) and rows with exact -inf entries: log0 bookkeeping on both sides."""
    w = small("cfg1", n_utt=2, t_lo=20, t_hi=30, vocab=40, beam=3, cand_k=6, win_m1=5, win_m2=5, end_flags=7,
              eos_run=3, max_len_abs=8)
    lens, ctc = make_inputs(w)
    ctc = ctc.copy()
    ctc[0, :lens[0], :] = -np.inf
    ctc[0, :lens[0], w["blank_id"]] = 0.0                   # utterance 0: blank with probability one
    ctc[1, :lens[1], 5] = -np.inf                           # utterance 1: one label impossible everywhere
    rep, res = lockstep_decode(w, ctc, lens)
    assert rep["max_score_err"] < 1e-4
    assert res["ntok"][0] == 0                              # the empty transcript


def test_very_large_unrestricted_vocabulary():
    """Every id a candidate on a vocabulary beyond what the register-resident list builder holds
    (more than 8192 candidates per hypothesis): the all-candidates score kernel with the
    block-wide arg-max list builder."""
    w = small("cfg1", n_utt=2, t_lo=25, t_hi=40, vocab=9001, beam=3, cand_k=0, win_m1=-1, win_m2=-1,
              end_flags=3, max_len_abs=7)
    rep, res = run(w)
    assert rep["utt_steps"] >= 8


@pytest.mark.parametrize("variant", ["windowed", "batch_window", "all_candidates"])
def test_unused_slots_of_a_batch(variant):
    """Length 0 marks an unused slot (a last batch that is not full): it is finished from the
    start, holds no hypothesis, costs nothing and reports an empty result; the other utterances
    decode exactly as they do in a full batch (every step against the oracle)."""
    kw = dict(windowed=dict(cand_k=10, win_m1=6, win_m2=6, end_flags=7, eos_run=3),
              batch_window=dict(cand_k=10, win_m1=6, win_m2=6, end_flags=7, eos_run=3, win_union=1),
              all_candidates=dict(cand_k=0, win_m1=-1, win_m2=-1, end_flags=3))[variant]
    w = small("cfg1", vocab=48, beam=3, max_len_ratio=0.4, **kw)
    lens = np.asarray([0, 37, 0, 0, 90, 12, 0], np.int32)
    ctc = gen.workload_ctc(w, np.maximum(lens, 1))          # the rows of an unused slot are never read
    ctc[lens == 0] = np.nan
    used = [u for u in range(len(lens)) if lens[u] > 0]
    seen_live = []
    rep, res = lockstep_decode(w, ctc, lens, check_utts=used,
                               progress=lambda step, out: seen_live.append(out["live"][lens == 0].any()
                                                                           or not out["finished"][lens == 0].all()))
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4, rep
    assert res["cells"] == int(res["oracle_cells"])
    assert not any(seen_live)
    empty = lens == 0
    assert (res["ntok"][empty] == 0).all() and (res["flags"][empty] == 1).all() and (res["score"][empty] < -1e29).all()


def test_batch_of_unused_slots_only():
    import torch
    import paper_2101_05600_amd as m
    w = small("cfg1", vocab=48, beam=3, cand_k=10, win_m1=6, win_m2=6, end_flags=7, eos_run=3)
    cfg = m.make_config(n_utt=3, t_max=20, **{k: v for k, v in w.items() if k != "n_utt"})
    d_ctc = torch.full((3, 20, 48), float("nan"), device="cuda")
    h = m.ctcbs_create(cfg, d_ctc, np.zeros(3, np.int32))
    try:
        att = torch.full((3, 3, 48), float("nan"), device="cuda")
        assert m.ctcbs_step(h, att, m.StepOut()) == m.DONE
        tok, nt, sc, frm, fl = m.ctcbs_finalize(h, 3, 4)
        assert (nt == 0).all() and (fl == 1).all() and (sc < -1e29).all()
    finally:
        m.ctcbs_destroy(h)
