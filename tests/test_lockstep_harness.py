"""The lock-step validator itself, exercised on the CPU with a stand-in decoder built from a
second oracle instance: a faithful stand-in passes, near-tie swaps are adopted, real
deviations raise."""
import numpy as np
import pytest

import gen
import oracle
from oracle import OracleUtt, make_cfg
from oracle.lockstep import Lockstep, ParityError


def stand_in_step(o, att, B, perturb=None):
    """One step of a free-running oracle, reported in the step-output layout of the C ABI."""
    live_old = [o.hyp(j)["live"] for j in range(B)]
    o.score(att)
    el, fire, margin = o.e2()
    o.rank()
    S_all = o.sorted_cands()
    S = S_all[:B]
    best, je, forced = o.best, o.joint_eos(), (o.step + 1 == o.lmax)
    out = dict(parent=np.full((1, B), -1, np.int32), token=np.full((1, B), -1, np.int32),
               score=np.full((1, B), -1e30, np.float32), live=np.zeros((1, B), np.uint8),
               finished=np.zeros(1, np.uint8), tau=np.zeros((1, B), np.int32),
               tau_end=np.zeros((1, B), np.int32), eos_added=np.zeros((1, B), np.uint8),
               stopped=np.zeros((1, B), np.uint8))
    par, tok, sc = S["parent"].copy(), S["token"].copy(), S["joint"].copy()
    if perturb:
        perturb(par, tok, sc, S_all)
    for j in range(B):
        if live_old[j]:
            out["stopped"][0, j] = fire[j]
            out["eos_added"][0, j] = forced or fire[j] or je[j] > best
    fin = o.commit(par, tok, out["eos_added"][0].astype(np.int32), out["stopped"][0].astype(np.int32))
    n = len(par)
    out["parent"][0, :n], out["token"][0, :n], out["score"][0, :n] = par, tok, sc
    out["finished"][0] = fin
    for j in range(n):
        h = o.hyp(j)
        out["live"][0, j] = 0 if fin else 1
        out["tau"][0, j], out["tau_end"][0, j] = h["tau"], h["tau_end"]
    return out


def run(perturb_at=None, perturb=None, cfg_over=None):
    kw = dict(vocab=40, beam=4, cand_k=10, win_m1=10, win_m2=10, ctc_weight=0.3, max_len_abs=14,
              end_flags=7, eos_run=5, length_bonus=0.5)
    kw.update(cfg_over or {})
    cfg = make_cfg(**kw)
    x = gen.ctc_utt(4, 0, 70, 40)
    ls = Lockstep([x], cfg)
    o = OracleUtt(x, cfg)
    B = cfg.beam
    while not o.finished:
        step = o.step + 1
        hyps = [o.hyp(j) for j in range(B)]
        att = np.stack([gen.att_row(1, 0, step, gen.prefix_hash(h["labels"]), 40) if h["live"]
                        else np.full(40, np.nan, np.float32) for h in hyps])
        out = stand_in_step(o, att, B, perturb if step == perturb_at else None)
        ls.step(att[None], out)
    return ls, o


def test_faithful_stand_in_passes_and_results_agree():
    ls, o = run()
    lab, sc, fb = o.result()
    tok = np.full((1, 20), -1, np.int32); tok[0, :len(lab)] = lab
    ls.check_results(tok, np.array([len(lab)]), np.array([sc], np.float32), np.array([int(fb)]))
    assert ls.report["adopted_sel"] == 0 and ls.report["exact_sel_steps"] == ls.report["utt_steps"]
    # the per-label time stamps are part of the result: the stand-in's own pass, a wrong frame is caught
    lab2, frm, _, _ = o.result_frames()
    assert len(lab) > 1 and list(lab2) == list(lab)
    frames = np.full((1, 20), -1, np.int32); frames[0, :len(lab)] = frm
    ls.check_results(tok, np.array([len(lab)]), np.array([sc], np.float32), np.array([int(fb)]), frames=frames)
    frames[0, len(lab) // 2] += 1
    with pytest.raises(ParityError, match="time stamps"):
        ls.check_results(tok, np.array([len(lab)]), np.array([sc], np.float32), np.array([int(fb)]), frames=frames)


def test_wrong_token_is_caught():
    def p(par, tok, sc, S_all):
        # a candidate of the same parent that is far down the ranking
        worst = [c for c in S_all if c["parent"] == par[0]][-1]
        tok[0] = worst["token"]
    with pytest.raises(ParityError):
        run(perturb_at=3, perturb=p)


def test_wrong_time_index_is_caught():
    """A time index that is not a maximiser of the oracle's forward variable (within the tolerance) fails."""
    cfg = make_cfg(vocab=40, beam=4, cand_k=10, win_m1=10, win_m2=10, ctc_weight=0.3, max_len_abs=14,
                   end_flags=7, eos_run=5, length_bonus=0.5)
    x = gen.ctc_utt(4, 0, 70, 40)
    ls = Lockstep([x], cfg)
    o = OracleUtt(x, cfg)
    with pytest.raises(ParityError, match="tau of new slot"):
        while not o.finished:
            step = o.step + 1
            hyps = [o.hyp(j) for j in range(4)]
            att = np.stack([gen.att_row(1, 0, step, gen.prefix_hash(h["labels"]), 40) if h["live"]
                            else np.full(40, np.nan, np.float32) for h in hyps])
            out = stand_in_step(o, att, 4)
            if step == 5:
                out["tau"][0, 0] += 7
            ls.step(att[None], out)


def test_score_error_is_caught():
    def p(par, tok, sc, S_all):
        sc[1] += 5e-4
    with pytest.raises(ParityError):
        run(perturb_at=2, perturb=p)


def test_swapped_order_outside_tolerance_is_caught():
    def p(par, tok, sc, S_all):
        par[[0, 1]], tok[[0, 1]], sc[[0, 1]] = par[[1, 0]], tok[[1, 0]], sc[[1, 0]]
    with pytest.raises(ParityError):
        run(perturb_at=4, perturb=p)


def test_dropping_the_best_candidate_is_caught():
    def p(par, tok, sc, S_all):
        # the last slot takes the first candidate that did not make the beam, the best is lost
        par[:-1], tok[:-1], sc[:-1] = par[1:].copy(), tok[1:].copy(), sc[1:].copy()
        par[-1], tok[-1], sc[-1] = S_all[len(par)]["parent"], S_all[len(par)]["token"], S_all[len(par)]["joint"]
    with pytest.raises(ParityError):
        run(perturb_at=2, perturb=p)
