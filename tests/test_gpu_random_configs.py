"""GPU parity on seeded random small configurations: combinations of beam width, vocabulary,
candidate count, window form (per hypothesis, batch-wide, none; one-sided), end rules, batch shape
(ragged, unused slots) that the hand-written tests do not spell out, each decoded step by step against
the oracle.  All cases run in ONE process, handle after handle, as a long-running service would: device
memory that a new handle gets is whatever earlier handles left there (a kernel that lets a never-written
value steer an access shows up here and nowhere in a fresh process; tests/cpu_emu hunts the same on the
CPU with poisoned memory)."""
import random

import numpy as np
import pytest

import gen
from helpers import lockstep_decode
from test_gpu_parity import small

pytestmark = pytest.mark.gpu

RUNS = [(1, 60), (2, 40), (3, 30)]          # (seed of the list, cases): every case ran on the CPU build first


def case_params(case, seed0=1):
    rng = random.Random(seed0 * 1000 + case)
    beam = rng.choice([1, 2, 3, 4, 6, 10, 16, 20, 32])
    vocab = rng.choice([12, 40, 64, 129, 300, 700, 1000])
    mode = rng.choice(["win", "win", "win_e2", "union", "unres", "full", "full_win"])
    n_utt = rng.choice([1, 2, 3, 5, 9])
    t_lo = rng.choice([5, 20, 60])
    t_hi = t_lo + rng.choice([0, 30, 150, 320])
    kw = dict(n_utt=n_utt, t_lo=t_lo, t_hi=t_hi, vocab=vocab, beam=beam, seed=rng.randrange(1 << 30),
              max_len_ratio=rng.choice([0.2, 0.3, 0.5]), length_bonus=rng.choice([0.0, 0.5, 1.0]),
              ctc_weight=rng.choice([0.1, 0.3, 0.5, 0.9]), end_flags=rng.choice([1, 2, 3]))
    K = min(rng.choice([1, 4, 10, 24, 40, 60]), vocab - 3)
    m1, m2 = rng.choice([(3, 3), (5, 20), (12, 12), (50, 50), (80, 80), (5, 200)])
    if mode == "win":
        kw.update(cand_k=K, win_m1=m1, win_m2=m2)
    elif mode == "win_e2":
        kw.update(cand_k=K, win_m1=m1, win_m2=m2, end_flags=kw["end_flags"] | 4, eos_run=rng.choice([1, 3, 10]))
    elif mode == "union":
        kw.update(cand_k=K, win_m1=m1, win_m2=rng.choice([m2, -1]), win_union=1)
    elif mode == "unres":
        kw.update(cand_k=K, win_m1=-1, win_m2=-1)
    elif mode == "full":
        kw.update(cand_k=0, win_m1=-1, win_m2=-1)
    else:
        kw.update(cand_k=0, win_m1=m1, win_m2=m2)
    if mode in ("full", "full_win") and vocab > 300:
        kw["vocab"] = 300
    w = small("cfg1", **kw)
    lens = gen.workload_lengths(w)
    if rng.random() < 0.3 and n_utt > 1:
        lens[rng.randrange(n_utt)] = 0                      # an unused slot
    return mode, w, lens


@pytest.mark.parametrize("seed0,n_cases", RUNS)
def test_random_small_configurations_one_process(seed0, n_cases):
    bad = []
    for case in range(n_cases):
        mode, w, lens = case_params(case, seed0)
        used = [u for u in range(len(lens)) if lens[u] > 0]
        if not used:
            continue
        print(f"case {seed0}/{case}: {mode} U={len(lens)} beam={w['beam']} V={w['vocab']} K={w['cand_k']} "
              f"M=({w['win_m1']},{w['win_m2']}) union={w.get('win_union', 0)} end={w['end_flags']} lens={list(lens)}",
              flush=True)
        ctc = gen.workload_ctc(w, np.maximum(lens, 1))
        rep, res = lockstep_decode(w, ctc, lens, check_utts=used)
        ok = (rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4
              and res["cells"] == int(res["oracle_cells"]))
        if not ok:
            bad.append((case, mode, rep))
    assert not bad, bad
