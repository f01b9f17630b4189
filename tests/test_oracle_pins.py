"""Pins of the CPU oracle against things it did not compute itself.

Each test names the passage of the paper (arXiv 2101.05600) whose content it fixes:
brute-force enumeration of CTC alignments (Sec. 2.1 rules + Eq. 3), the prefix-sum
invariant, the full-sequence forward probability (textbook lattice and torch's CTC loss),
closed forms, window properties (Eq. 5), Algorithm 2/3 behaviour on constructed inputs.
"""
import itertools
import math

import numpy as np
import pytest
import torch

import gen
import oracle
from oracle import OracleUtt, make_cfg, prefix_and_full, end_detect

NEG = -np.inf


def lse(v):
    v = np.asarray(v, dtype=np.float64)
    if v.size == 0 or np.all(np.isneginf(v)):
        return NEG
    m = v.max()
    return m + math.log(np.exp(v - m).sum())


def rand_logp(rng, T, V, peaky=0.0):
    z = rng.normal(size=(T, V)) * (1.0 + peaky)
    z = z - np.log(np.exp(z).sum(1, keepdims=True))
    return z.astype(np.float32)


def collapse(path, blank=0):
    out, prev = [], None
    for z in path:
        if z != prev and z != blank:
            out.append(z)
        prev = z
    return tuple(out)


def brute_tables(x, blank=0):
    """log-prob of every collapsed output, by enumerating all V^T frame paths."""
    T, V = x.shape
    table = {}
    for path in itertools.product(range(V), repeat=T):
        lp = sum(float(x[t, z]) for t, z in enumerate(path))
        y = collapse(path, blank)
        table.setdefault(y, []).append(lp)
    return {y: lse(v) for y, v in table.items()}


# --------------------------------------------------------------------------------------
# P1: Sec. 2.1 alignment rules + Eq. (3) by brute force, T <= 6, V <= 3
# --------------------------------------------------------------------------------------
@pytest.mark.parametrize("T,V,blank", [(1, 2, 0), (3, 3, 0), (5, 3, 0), (6, 3, 0), (5, 3, 1), (4, 4, 0)])
def test_prefix_and_full_match_brute_force(T, V, blank):
    rng = np.random.default_rng(100 * T + V + blank)
    x = rand_logp(rng, T, V)
    full = brute_tables(x, blank)           # log P(output == y)
    labels = [k for k in range(V) if k != blank]
    for n in range(0, T + 2):
        for g in itertools.product(labels, repeat=n):
            # prefix probability = total mass of outputs that start with g
            want_psi = lse([lp for y, lp in full.items() if y[:n] == g])
            want_phi = full.get(g, NEG)
            got_psi, got_phi = prefix_and_full(x, list(g), blank_id=blank)
            # Eq. (3) takes the frames after the prefix's completion to sum to one; rows of
            # fp32 log-probs do so only to ~1e-8 each, hence the looser bound on psi.
            for got, want, tol in ((got_psi, want_psi, 1e-6), (got_phi, want_phi, 1e-9)):
                if want == NEG:
                    assert got == NEG, (g, got)
                else:
                    assert abs(got - want) < tol, (g, got, want)


# --------------------------------------------------------------------------------------
# P2 / P4: psi(g) = sum_c psi(g.c) + phi_T(g); psi(empty) = 1
# --------------------------------------------------------------------------------------
def test_prefix_sum_invariant():
    rng = np.random.default_rng(7)
    T, V = 40, 7
    x = rand_logp(rng, T, V, peaky=1.0)
    for g in ([], [3], [3, 3], [1, 2, 3, 4, 5, 6], [2, 2, 2, 5, 1], [6, 1, 6, 1, 6]):
        psi, phi = prefix_and_full(x, g)
        parts = [phi] + [prefix_and_full(x, g + [c])[0] for c in range(1, V)]
        # the identity holds up to the rows' own normalisation error: fp32 log-prob rows sum to
        # one only to ~1e-8 each
        assert abs(lse(parts) - psi) < 1e-6, g
    assert abs(prefix_and_full(x, [])[0]) < 1e-12
    # the empty prefix's "whole output" probability is the all-blank path
    assert abs(prefix_and_full(x, [])[1] - float(x[:, 0].astype(np.float64).sum())) < 1e-9


# --------------------------------------------------------------------------------------
# P3: phi_T(y) = CTC forward probability (textbook 2|y|+1 lattice; torch's CTC loss)
# --------------------------------------------------------------------------------------
def lattice_forward(x, y, blank=0):
    T = x.shape[0]
    ext = [blank]
    for k in y:
        ext += [k, blank]
    S = len(ext)
    a = np.full(S, NEG)
    a[0] = x[0, blank]
    if S > 1:
        a[1] = x[0, ext[1]]
    for t in range(1, T):
        b = np.full(S, NEG)
        for s in range(S):
            terms = [a[s]]
            if s >= 1:
                terms.append(a[s - 1])
            if s >= 2 and ext[s] != blank and ext[s] != ext[s - 2]:
                terms.append(a[s - 2])
            b[s] = lse(terms) + x[t, ext[s]]
        a = b
    return lse([a[S - 1], a[S - 2]] if S > 1 else [a[S - 1]])


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_full_sequence_probability_matches_ctc_forward(seed):
    rng = np.random.default_rng(seed)
    T, V = 50, 9
    x = rand_logp(rng, T, V, peaky=0.5)
    for y in ([1], [4, 4], [1, 2, 2, 3], [8, 7, 6, 5, 4, 3, 2, 1], [5] * 10, list(rng.integers(1, V, 20))):
        y = [int(k) for k in y]
        _, phi = prefix_and_full(x, y)
        assert abs(phi - lattice_forward(x.astype(np.float64), y)) < 1e-9
        loss = torch.nn.functional.ctc_loss(
            torch.from_numpy(x.astype(np.float64)).unsqueeze(1), torch.tensor([y]),
            torch.tensor([T]), torch.tensor([len(y)]), blank=0, reduction="sum", zero_infinity=False)
        assert abs(phi + float(loss)) < 1e-8


# --------------------------------------------------------------------------------------
# P10: closed forms of the repeat rule (third alignment rule)
# --------------------------------------------------------------------------------------
def test_repeat_label_closed_forms():
    rng = np.random.default_rng(3)
    x3 = rand_logp(rng, 3, 3)
    psi, phi = prefix_and_full(x3, [1, 1])
    want = float(x3[0, 1]) + float(x3[1, 0]) + float(x3[2, 1])   # only a-blank-a fits in 3 frames
    assert abs(psi - want) < 1e-12 and abs(phi - want) < 1e-12
    x2 = rand_logp(rng, 2, 3)
    assert prefix_and_full(x2, [1, 1]) == (NEG, NEG)
    # different labels need no blank: psi(a.b) over 2 frames = x1(a)+x2(b)
    psi, _ = prefix_and_full(x2, [1, 2])
    assert abs(psi - (float(x2[0, 1]) + float(x2[1, 2]))) < 1e-12
    # single label, T=2: prefix a = a? + blank,a ; full = aa + a,blank + blank,a
    psi, phi = prefix_and_full(x2, [1])
    a1, a2, b1, b2 = (float(x2[0, 1]), float(x2[1, 1]), float(x2[0, 0]), float(x2[1, 0]))
    assert abs(psi - lse([a1, b1 + a2])) < 1e-12
    assert abs(phi - lse([a1 + a2, a1 + b2, b1 + a2])) < 1e-12


# --------------------------------------------------------------------------------------
# Search-level helpers
# --------------------------------------------------------------------------------------
def att_table_rows(seed, utt, step, hyps, V, scale=2.0):
    hs = [gen.prefix_hash(h) for h in hyps]
    return gen.att_rows(seed, [utt] * len(hs), step, hs, V, scale)


def run_free(x, cfg, seed=5, max_steps=None, record=None):
    """Free-running oracle decode with generator-keyed attention rows."""
    o = OracleUtt(x, cfg)
    B, V = cfg.beam, cfg.vocab
    while not o.finished and (max_steps is None or o.step < max_steps):
        hyps = [o.hyp(j) for j in range(B)]
        att = np.full((B, V), np.nan, dtype=np.float32)
        for j, h in enumerate(hyps):
            if h["live"]:
                att[j] = gen.att_row(seed, 0, o.step + 1, gen.prefix_hash(h["labels"]), V)
        o.score(att)
        if record is not None:
            record(o, att)
        o.commit()
    return o


def small_workload(T=60, V=12, seed=11, zipf=0.0):
    return gen.ctc_utt(seed, 0, T, V, zipf_s=zipf)


# --------------------------------------------------------------------------------------
# Step-level consistency with the stand-alone definition (Eq. 3 inside Algorithm 2)
# --------------------------------------------------------------------------------------
def test_step_scores_equal_definition_along_a_decode():
    x = small_workload()
    cfg = make_cfg(vocab=12, beam=3, cand_k=0, ctc_weight=0.4, max_len_abs=12, end_flags=0)
    seen = []

    def rec(o, att):
        ids, ctc, joint, attc = o.cand_id(), o.cand_ctc(), o.cand_joint(), o.cand_att()
        l = o.step + 1
        for j in range(o.B):
            h = o.hyp(j)
            if not h["live"]:
                continue
            a_cum = 0.0
            for i, k in enumerate(ids[j]):
                psi, _ = prefix_and_full(x, list(h["labels"]) + [int(k)])
                assert (psi == ctc[j, i]) or abs(psi - ctc[j, i]) < 1e-9
                want = 0.4 * psi + 0.6 * (h["att"] + float(att[j, k]))
                assert abs(want - joint[j, i]) < 1e-9 or (want == NEG and joint[j, i] == NEG)
            _, phi = prefix_and_full(x, list(h["labels"]))
            assert abs(phi - o.ctc_eos()[j]) < 1e-9
            seen.append(l)

    run_free(x, cfg, record=rec)
    assert max(seen) >= 8


# --------------------------------------------------------------------------------------
# P5: window (Eq. 5): huge margins == unrestricted; windowed <= full; monotone in M1, M2
# --------------------------------------------------------------------------------------
def test_window_properties():
    x = small_workload(T=80, V=10, seed=21)
    base = dict(vocab=10, beam=4, cand_k=0, ctc_weight=0.3, max_len_abs=25, end_flags=0)
    full = run_free(x, make_cfg(**base))
    huge = run_free(x, make_cfg(win_m1=1000, win_m2=1000, **base))
    assert np.array_equal(full.result()[0], huge.result()[0])
    assert abs(full.result()[1] - huge.result()[1]) < 1e-12
    # same parent state, different windows: drive a full decode, re-score each step with windows
    cfgs = [make_cfg(win_m1=m1, win_m2=m2, **base) for (m1, m2) in
            [(2, 2), (5, 2), (5, 8), (20, 8), (20, 30), (1000, 1000)]]
    o = OracleUtt(x, make_cfg(**base))
    for step in range(12):
        hyps = [o.hyp(j) for j in range(o.B)]
        att = np.stack([gen.att_row(5, 0, step + 1, gen.prefix_hash(h["labels"]), 10) for h in hyps])
        o.score(att)
        ref = o.cand_ctc()
        # replay the same hypotheses through windowed scorers: rebuild them by forcing the selection
        o.commit()
    # windowed decoders forced along the unrestricted decoder's trajectory
    traj = OracleUtt(x, make_cfg(**base))
    wins = [OracleUtt(x, c) for c in cfgs]
    for step in range(15):
        hyps = [traj.hyp(j) for j in range(traj.B)]
        att = np.stack([gen.att_row(5, 0, step + 1, gen.prefix_hash(h["labels"]), 10)
                        if h["live"] else np.zeros(10, np.float32) for h in hyps])
        traj.score(att)
        traj.rank()
        sel = traj.sorted_cands()[:traj.B]
        full_ctc = traj.cand_ctc()
        prev = None
        for w in wins:
            w.score(att)
            c = w.cand_ctc()
            live = np.array([h["live"] for h in hyps], bool)
            assert np.all(c[live] <= full_ctc[live] + 1e-9)
            if prev is not None:
                assert np.all(c[live] >= prev[live] - 1e-9)      # wider window never loses mass
            prev = c
        assert np.allclose(prev[live], full_ctc[live], atol=1e-9)
        z = np.zeros(traj.B, np.int32)
        traj.commit(sel["parent"], sel["token"], z, z)
        for w in wins:
            w.commit(sel["parent"], sel["token"], z, z)
            # keep every scorer's time indices on the reference trajectory so windows nest
            w.override([traj.hyp(j)["tau"] for j in range(traj.B)],
                       [traj.hyp(j)["tau_end"] for j in range(traj.B)], -1)


def test_window_formula_and_empty_window():
    x = small_workload(T=30, V=8, seed=4)
    cfg = make_cfg(vocab=8, beam=2, cand_k=0, win_m1=3, win_m2=4, max_len_abs=40, end_flags=0)
    o = OracleUtt(x, cfg)
    for step in range(1, 31):
        hyps = [o.hyp(j) for j in range(2)]
        att = np.stack([gen.att_row(9, 0, step, gen.prefix_hash(h["labels"]), 8) for h in hyps])
        o.score(att)
        s, e = o.windows()
        for j, h in enumerate(hyps):
            if h["live"]:
                assert s[j] == max(h["tau"] - 3, step, 1)
                assert e[j] == min(h["tau_end"] + 4, 30)
                if e[j] < s[j]:
                    assert np.all(np.isneginf(o.cand_ctc()[j]))
        if o.commit():
            break
    assert o.finished


# --------------------------------------------------------------------------------------
# P6: K >= V-2 is the unrestricted candidate set; a small K is the top-K by attention
# --------------------------------------------------------------------------------------
def test_candidate_restriction():
    x = small_workload(T=50, V=12, seed=2)
    base = dict(vocab=12, beam=3, ctc_weight=0.3, max_len_abs=15)
    a = run_free(x, make_cfg(cand_k=0, **base))
    b = run_free(x, make_cfg(cand_k=10, **base))
    c = run_free(x, make_cfg(cand_k=99, **base))
    assert np.array_equal(a.result()[0], b.result()[0]) and np.array_equal(a.result()[0], c.result()[0])
    att = np.zeros((3, 12), np.float32)
    att[0] = [9, 1, 5, 5, 2, 5, 0, 5, 3, 1, 1, 9]        # blank=0 and eos=11 hold the largest values
    o = OracleUtt(x, make_cfg(cand_k=3, **base))
    o.score(att)
    assert list(o.cand_id()[0]) == [2, 3, 5]              # four ids hold 5.0: the largest id (7) loses
    o = OracleUtt(x, make_cfg(cand_k=5, **base))
    o.score(att)
    assert list(o.cand_id()[0]) == [2, 3, 5, 7, 8]        # then the 3.0 at id 8
    # ascending order and exclusion of blank/eos
    assert 0 not in o.cand_id()[0] and 11 not in o.cand_id()[0]


# --------------------------------------------------------------------------------------
# P7 / P9: lambda = 0 is attention-only search; beam 1 is greedy (Algorithm 2, TopB)
# --------------------------------------------------------------------------------------
def test_attention_only_scores_are_path_sums_and_beam_is_exhaustive():
    V, T = 5, 12            # ids: 0 blank, 1..3 labels, 4 eos
    x = small_workload(T=T, V=V, seed=8)
    cfg = make_cfg(vocab=V, beam=27, cand_k=0, ctc_weight=0.0, length_bonus=0.25, max_len_abs=4,
                   end_flags=0)
    o = OracleUtt(x, cfg)
    table = {}

    def row(prefix, step):
        return gen.att_row(77, 0, step, gen.prefix_hash(list(prefix)), V)

    step = 0
    while not o.finished:
        step += 1
        hyps = [o.hyp(j) for j in range(27)]
        att = np.stack([row(h["labels"], step) if h["live"] else np.zeros(V, np.float32) for h in hyps])
        o.score(att)
        o.commit()
        # beam = every label sequence of this length, ordered by its path sum (3^step <= 27)
        seqs = {}
        for g in itertools.product([1, 2, 3], repeat=step):
            sc = sum(float(row(g[:i], i + 1)[g[i]]) for i in range(step)) + 0.25 * step
            seqs[g] = sc
        if step < 4:
            want = sorted(seqs.items(), key=lambda kv: (-kv[1],))
            got = [(tuple(o.hyp(j)["labels"]), o.hyp(j)["joint"]) for j in range(len(want))]
            assert [g for g, _ in got] == [g for g, _ in want]
            assert np.allclose([s for _, s in got], [s for _, s in want], atol=1e-9)
    labels, score, fb = o.result()
    # lambda = 0: ctc_eos = -inf rows are excluded; every ended entry scored by its own path sum
    for e in o.ended():
        assert e["len"] <= 4


def test_beam_one_is_greedy():
    x = small_workload(T=40, V=9, seed=13)
    cfg = make_cfg(vocab=9, beam=1, cand_k=0, ctc_weight=0.5, max_len_abs=10, end_flags=0)
    o = OracleUtt(x, cfg)
    while not o.finished:
        h = o.hyp(0)
        att = gen.att_row(3, 0, o.step + 1, gen.prefix_hash(h["labels"]), 9)[None]
        o.score(att)
        J, ids = o.cand_joint()[0], o.cand_id()[0]
        k = int(ids[int(np.argmax(J))])
        o.commit()
        if o.hyp(0)["live"]:
            assert o.hyp(0)["labels"][-1] == k


# --------------------------------------------------------------------------------------
# Algorithm 2's eos rule and the final argmax, on a hand-made two-step case
# --------------------------------------------------------------------------------------
def test_eos_rule_strict_and_final_argmax():
    V, T = 4, 3            # 0 blank, 1 a, 2 b, 3 eos
    x = np.log(np.array([[0.1, 0.8, 0.05, 0.05], [0.8, 0.1, 0.05, 0.05], [0.9, 0.04, 0.03, 0.03]],
                        np.float32))
    cfg = make_cfg(vocab=V, beam=2, cand_k=0, ctc_weight=0.5, max_len_abs=3, end_flags=0,
                   length_bonus=0.7)
    o = OracleUtt(x, cfg)
    att1 = np.log(np.array([[0.01, 0.9, 0.05, 0.04], [0.25] * 4], np.float32))
    o.score(att1)
    o.commit()
    assert list(o.hyp(0)["labels"]) == [1] and list(o.hyp(1)["labels"]) == [2]
    assert o.ended() == []                                   # phi_T(empty) is tiny: eos not confident
    att2 = np.log(np.array([[0.01, 0.02, 0.02, 0.95], [0.01, 0.4, 0.4, 0.19]], np.float32))
    o.score(att2)
    je, best = o.joint_eos(), None
    o.rank()
    best = o.best
    o.commit()
    ended = o.ended()
    assert je[0] > best and len(ended) >= 1 and ended[0]["slot"] == 0 and ended[0]["len"] == 2
    _, phi_a = prefix_and_full(x, [1])
    want = 0.5 * phi_a + 0.5 * (math.log(0.9) + math.log(0.95)) + 0.7 * 2   # bonus counts eos
    assert abs(ended[0]["score"] - want) < 1e-6
    # forced ending at the cap adds every live hypothesis and finishes
    att3 = np.log(np.full((2, 4), 0.25, np.float32))
    o.score(att3)
    assert o.commit() == 1 and o.finished
    lab, sc, fb = o.result()
    assert list(lab) == [1] and abs(sc - want) < 1e-6 and not fb


# --------------------------------------------------------------------------------------
# Eq. (4) and Algorithm 3 on plain lists
# --------------------------------------------------------------------------------------
def test_end_detection_rules():
    cfg = make_cfg(vocab=5, beam=2, end_flags=3, end_m=3, end_d=-10.0, end_c=2)
    T = 50
    # best ended hyp long ago; the last three lengths all ended >10 below it -> stop
    assert end_detect(cfg, T, 9, [4, 7, 8, 9], [10, 20, 22, 25], [-5.0, -16.0, -17.0, -15.5])[0]
    # one of the three within 10 of the best -> go on
    assert not end_detect(cfg, T, 9, [4, 7, 8, 9], [10, 20, 22, 25], [-5.0, -16.0, -14.9, -15.5])[0]
    # a length with no ended hypothesis does not count -> go on (also: empty set never stops)
    assert not end_detect(cfg, T, 9, [4, 7, 9], [10, 20, 25], [-5.0, -16.0, -15.5])[0]
    assert not end_detect(cfg, T, 1, [], [], [])[0]
    # per length the best hypothesis is the one compared
    assert not end_detect(cfg, T, 9, [4, 7, 7, 8, 9], [1, 2, 3, 4, 5], [-5.0, -16.0, -14.0, -17.0, -15.5])[0]
    # exactly at the threshold is not below it
    assert not end_detect(cfg, T, 3, [1, 2, 3, 0], [1, 1, 1, 1], [-15.0, -16.0, -17.0, -5.0])[0]
    # tau-count rule: more than C ended hypotheses whose tau equals T
    assert not end_detect(cfg, T, 9, [5, 6], [T, T], [-1.0, -2.0])[0]
    assert end_detect(cfg, T, 9, [5, 6, 7], [T, T, T], [-1.0, -2.0, -3.0])[0]
    assert not end_detect(cfg, T, 9, [5, 6, 7], [T, T - 1, T], [-1.0, -2.0, -3.0])[0]
    only_base = make_cfg(vocab=5, beam=2, end_flags=1)
    assert not end_detect(only_base, T, 9, [5, 6, 7], [T, T, T], [-1.0, -2.0, -3.0])[0]
    only_tau = make_cfg(vocab=5, beam=2, end_flags=2)
    assert not end_detect(only_tau, T, 9, [4, 7, 8, 9], [10, 20, 22, 25], [-5.0, -16.0, -17.0, -15.5])[0]


# --------------------------------------------------------------------------------------
# tau / tau~ (Sec. 3.2.2) on constructed, sharply peaked posteriors; P11
# --------------------------------------------------------------------------------------
def peaky_posteriors(T, V, emits, p=0.98):
    """Blank everywhere except frames in `emits` {t: label}, 1-based."""
    x = np.full((T, V), (1.0 - p) / (V - 1), np.float64)
    for t in range(1, T + 1):
        x[t - 1, emits.get(t, 0)] = p
    return np.log(x).astype(np.float32)


def follow(o, x, seq, V, eos_logp=-8.0):
    """Drive the oracle with attention rows that strongly prefer the labels in seq, then eos."""
    taus = []
    step = 0
    while not o.finished and step < 200:
        att = np.full((o.B, V), -6.0, np.float32)
        att[:, V - 1] = eos_logp
        want = seq[step] if step < len(seq) else None
        if want is not None:
            att[:, want] = -0.05
        else:
            att[:, V - 1] = -0.05
        o.score(att)
        o.commit()
        step += 1
        if o.hyp(0)["live"]:
            taus.append((list(o.hyp(0)["labels"]), o.hyp(0)["tau"], o.hyp(0)["tau_end"]))
    return taus


def test_time_indices_land_on_the_emitting_frames():
    T, V = 60, 6
    emits = {5: 1, 17: 2, 18: 2, 30: 3, 44: 1}
    x = peaky_posteriors(T, V, emits)
    cfg = make_cfg(vocab=V, beam=2, cand_k=0, ctc_weight=0.5, max_len_abs=10, end_flags=0)
    o = OracleUtt(x, cfg)
    taus = follow(o, x, [1, 2, 3, 1], V)
    got = {tuple(l): (a, b) for l, a, b in taus}
    assert got[(1,)][0] == 5 and got[(1, 2)][0] in (17, 18) and got[(1, 2, 3)][0] == 30
    assert got[(1, 2, 3, 1)][0] == 44
    # tau~ (blank after the label): first frame after the label's last emitting frame
    assert got[(1,)][1] == 6 and got[(1, 2)][1] == 19 and got[(1, 2, 3)][1] == 31
    lab, sc, fb = o.result()
    assert list(lab) == [1, 2, 3, 1]


def test_time_index_search_starts_at_the_parents_tau():
    """The argmax range of tau^l begins at tau^(l-1), not at the window start (Sec. 3.2.2)."""
    hits = 0
    for seed in range(40):
        rng = np.random.default_rng(seed)
        T, V = 14, 5
        x = rand_logp(rng, T, V, peaky=2.0)
        cfg = make_cfg(vocab=V, beam=3, cand_k=0, ctc_weight=0.6, max_len_abs=6, end_flags=0)
        o = OracleUtt(x, cfg)
        while not o.finished:
            parents = [o.hyp(j) for j in range(o.B)]
            att = np.stack([gen.att_row(seed, 0, o.step + 1, gen.prefix_hash(h["labels"]), V)
                            for h in parents])
            o.score(att)
            o.rank()
            sel = o.sorted_cands()[:o.B]
            s_win, e_win = o.windows()
            o.commit()
            for j in range(len(sel)):
                h = o.hyp(j)
                if not h["live"]:
                    continue
                g = parents[int(sel["parent"][j])]
                gn, gb = o.hyp_gamma(j)
                s, e = s_win[sel["parent"][j]], e_win[sel["parent"][j]]
                lo = max(s, g["tau"])
                assert h["tau"] >= g["tau"]
                if lo <= e and np.isfinite(gn[lo:e + 1].max()):
                    assert h["tau"] == lo + int(np.argmax(gn[lo:e + 1]))
                    assert h["tau_end"] == lo + int(np.argmax(gb[lo:e + 1]))
                    if s + int(np.argmax(gn[s:e + 1])) != h["tau"]:
                        hits += 1
    assert hits > 0        # the restriction mattered somewhere, so dropping it would be noticed


def test_overlong_hypotheses_peg_tau_at_T_and_algorithm3_stops():
    """Fig. 2(b): labels beyond what the audio holds get tau = T; more than C of them end decoding."""
    T, V = 30, 5
    x = peaky_posteriors(T, V, {4: 1, 12: 2}, p=0.9)
    cfg = make_cfg(vocab=V, beam=1, cand_k=0, ctc_weight=0.3, max_len_abs=25, end_flags=2, end_c=2)
    o = OracleUtt(x, cfg)
    step = 0
    pegged = 0
    while not o.finished:
        step += 1
        att = np.full((1, V), -5.0, np.float32)
        att[0, 3] = -0.2                      # the decoder keeps repeating label 3 (never in the audio)
        att[0, V - 1] = -0.1                  # ... and eos always looks attractive
        if step == 1:
            att[0, 1], att[0, 3] = -0.2, -5.0
        if step == 2:
            att[0, 2], att[0, 3] = -0.2, -5.0
        o.score(att)
        o.commit()
        if o.hyp(0)["live"] and o.hyp(0)["tau"] == T:
            pegged += 1
    n_T = sum(1 for e in o.ended() if e["tau"] == T)
    assert n_T == 3 and o.step < 25          # stopped by the count rule, not by the length cap
    assert pegged >= 3


def test_eos_run_rule_fires_at_true_length():
    """[brief] E2: with >= R trailing blank frames the finished transcript is stopped at once."""
    T, V = 50, 6
    x = peaky_posteriors(T, V, {6: 1, 15: 2, 27: 3})
    cfg = make_cfg(vocab=V, beam=1, cand_k=0, ctc_weight=0.5, max_len_abs=20, end_flags=4, eos_run=10)
    o = OracleUtt(x, cfg)
    fired_at = None
    for step, want in enumerate([1, 2, 3, 4, 4, 4], start=1):
        att = np.full((1, V), -4.0, np.float32)
        att[:, want] = -0.1
        att[:, V - 1] = -9.0                  # attention alone would never end the hypothesis
        o.score(att)
        el, fire, margin = o.e2()
        if fire[0] and fired_at is None:
            fired_at = step
            assert el[0] and margin[0] > 0
        if o.commit():
            break
    assert fired_at == 4                      # prefix (1,2,3) is complete: stop when extending it
    lab, sc, fb = o.result()
    assert list(lab) == [1, 2, 3] and o.finished
    # without the rule the same inputs keep going
    o2 = OracleUtt(x, make_cfg(vocab=V, beam=1, cand_k=0, ctc_weight=0.5, max_len_abs=20, end_flags=0))
    for step, want in enumerate([1, 2, 3, 4, 4, 4], start=1):
        att = np.full((1, V), -4.0, np.float32)
        att[:, want] = -0.1
        att[:, V - 1] = -9.0
        o2.score(att)
        o2.commit()
    assert not o2.finished


def test_eos_run_not_eligible_when_window_misses_the_tail():
    T, V = 50, 6
    x = peaky_posteriors(T, V, {6: 1})
    cfg = make_cfg(vocab=V, beam=1, cand_k=0, win_m1=5, win_m2=5, ctc_weight=0.5, max_len_abs=20,
                   end_flags=4, eos_run=10)
    o = OracleUtt(x, cfg)
    att = np.full((1, V), -4.0, np.float32)
    att[0, 1] = -0.1
    o.score(att); o.commit()
    o.score(att)
    el, fire, _ = o.e2()
    assert not el[0] and not fire[0]          # stored range [1, 5] does not reach T


def test_cells_count_is_K_times_window():
    x = small_workload(T=40, V=10, seed=6)
    cfg = make_cfg(vocab=10, beam=3, cand_k=5, win_m1=4, win_m2=6, max_len_abs=8, end_flags=0)
    total = 0

    def rec(o, att):
        nonlocal total
        s, e = o.windows()
        for j in range(o.B):
            if o.hyp(j)["live"] and e[j] >= s[j]:
                total += 5 * (e[j] - s[j] + 1)

    o = run_free(x, cfg, record=rec)
    assert o.cells == total and total > 0


def test_lmax():
    L = oracle.lib()
    import ctypes
    assert L.orc_lmax(ctypes.byref(make_cfg(vocab=5, beam=1, max_len_ratio=0.3)), 875) == 262
    assert L.orc_lmax(ctypes.byref(make_cfg(vocab=5, beam=1, max_len_abs=20)), 100) == 20
    assert L.orc_lmax(ctypes.byref(make_cfg(vocab=5, beam=1)), 7) == 7
    assert L.orc_lmax(ctypes.byref(make_cfg(vocab=5, beam=1, max_len_ratio=0.3)), 2) == 1


# --------------------------------------------------------------------------------------
# Batch-wide window (last two equations of Sec. 3.2.3)
# --------------------------------------------------------------------------------------
def test_union_window_is_min_start_max_end_over_the_batch():
    xs = [small_workload(T=70, V=9, seed=31), small_workload(T=45, V=9, seed=32)]
    base = dict(vocab=9, beam=3, cand_k=0, win_m1=4, win_m2=6, max_len_abs=12, end_flags=0)
    us = [OracleUtt(x, make_cfg(win_union=1, **base)) for x in xs]
    for step in range(1, 11):
        shares = [o.union_contrib() for o in us]
        live = [c for c in shares if c is not None]
        tmin, emax = min(c[0] for c in live), max(c[1] for c in live)
        # each share is (min tau, max min(tau~ + M2, T)) over that utterance's live hypotheses
        for o, c in zip(us, shares):
            hyps = [o.hyp(j) for j in range(3) if o.hyp(j)["live"]]
            assert c == (min(h["tau"] for h in hyps), max(min(h["tau_end"] + 6, o.T) for h in hyps))
        for i, o in enumerate(us):
            o.set_union(tmin, emax)
            hyps = [o.hyp(j) for j in range(3)]
            att = np.stack([gen.att_row(7, i, step, gen.prefix_hash(h["labels"]), 9) for h in hyps])
            o.score(att)
            s, e = o.windows()
            for j, h in enumerate(hyps):
                if h["live"]:
                    assert s[j] == max(tmin - 4, step, 1) and e[j] == min(emax, o.T)
                    # never narrower than the hypothesis's own window
                    assert s[j] <= max(h["tau"] - 4, step, 1) and e[j] >= min(h["tau_end"] + 6, o.T)
            o.commit()


# --------------------------------------------------------------------------------------
# Per-label time stamps (Sec. 3.2.2, Fig. 2(a)): the tau found when each label was appended
# --------------------------------------------------------------------------------------
def test_result_carries_the_time_stamp_of_every_label():
    T, V = 60, 6
    emits = {5: 1, 17: 2, 18: 2, 30: 3, 44: 1}
    x = peaky_posteriors(T, V, emits)
    cfg = make_cfg(vocab=V, beam=2, cand_k=0, ctc_weight=0.5, max_len_abs=10, end_flags=0)
    o = OracleUtt(x, cfg)
    follow(o, x, [1, 2, 3, 1], V)
    lab, frm, sc, fb = o.result_frames()
    assert list(lab) == [1, 2, 3, 1] and not fb
    assert frm[0] == 5 and frm[1] in (17, 18) and frm[2] == 30 and frm[3] == 44
    # the tau kept with an ended hypothesis g.<eos> is that of g's last label, and every ended entry
    # carries the stamps of its own labels
    for e in o.ended():
        assert len(e["taus"]) == len(e["labels"])
        if len(e["labels"]):
            assert e["tau"] == e["taus"][-1]
        assert list(e["taus"]) == sorted(e["taus"])          # time stamps never run backwards
    # an adopted tau (lock-step tolerance) replaces the stamp of the label it belongs to
    o2 = OracleUtt(x, cfg)
    att = np.full((2, V), -6.0, np.float32); att[:, 1] = -0.05
    o2.score(att); o2.commit()
    assert o2.hyp(0)["taus"].tolist() == [5]
    o2.override(np.array([6, -1], np.int32), None, -1)
    assert o2.hyp(0)["tau"] == 6 and o2.hyp(0)["taus"].tolist() == [6]


# --------------------------------------------------------------------------------------
# [brief] eos-run rule E2 against its definition evaluated another way: with unrestricted windows
# phi_t(g) is the full-sequence probability of g on the first t frames and the running prefix score
# of g.c up to t is the prefix probability of g.c on the first t frames -- both from the stand-alone
# routine that the brute-force enumeration pins
# --------------------------------------------------------------------------------------
def e2_by_definition(x, labels, cands, R, t_first=None):
    T = x.shape[0]
    t_first = T - R + 1 if t_first is None else t_first
    margin = np.inf
    for t in range(t_first, T + 1):
        _, E = prefix_and_full(x[:t], labels)
        X = max(prefix_and_full(x[:t], list(labels) + [c])[0] for c in cands)
        d = -np.inf if E == NEG else (np.inf if X == NEG else E - X)
        margin = min(margin, d)
    return margin


def test_eos_run_rule_equals_its_definition_and_the_frame_range_matters():
    fires = quiet = early_differs = late_differs = 0
    for seed in range(60):
        rng = np.random.default_rng(1000 + seed)
        T, V, R = 11, 4, 4
        x = rand_logp(rng, T, V, peaky=2.5)
        cfg = make_cfg(vocab=V, beam=2, cand_k=0, ctc_weight=0.5, max_len_abs=5, end_flags=4, eos_run=R)
        o = OracleUtt(x, cfg)
        while not o.finished:
            hyps = [o.hyp(j) for j in range(o.B)]
            att = np.stack([gen.att_row(seed, 0, o.step + 1, gen.prefix_hash(h["labels"]), V) for h in hyps])
            o.score(att)
            el, fire, margin = o.e2()
            s_win, _ = o.windows()
            for j, h in enumerate(hyps):
                if not h["live"]:
                    continue
                # unrestricted: eligible iff the window and the stored range start early enough
                assert bool(el[j]) == (max(s_win[j], h["rs"]) <= T - R + 1)
                if not el[j]:
                    continue
                cands = [c for c in range(V) if c not in (0, V - 1)]
                want = e2_by_definition(x, h["labels"], cands, R)
                assert (np.isinf(want) and margin[j] == want) or abs(margin[j] - want) < 1e-9
                assert bool(fire[j]) == (want > 0.0)
                fires += int(fire[j]); quiet += int(not fire[j])
                # one frame more, one frame fewer: would the outcome change?
                if s_win[j] <= T - R:
                    early_differs += int((e2_by_definition(x, h["labels"], cands, R, T - R) > 0) != bool(fire[j]))
                late_differs += int((e2_by_definition(x, h["labels"], cands, R, T - R + 2) > 0) != bool(fire[j]))
            o.commit()
    assert fires > 5 and quiet > 5
    assert early_differs > 0 and late_differs > 0      # so a frame range off by one would have been noticed


def test_eos_run_eligibility_boundary_and_strict_comparison():
    # eligibility: the window must start at T - R + 1 at the latest
    T, V, R = 30, 4, 10
    x = peaky_posteriors(T, V, {26: 1})
    for m1, want in ((5, 1), (4, 0)):                  # s = tau - M1 = 21 = T - R + 1, or 22
        cfg = make_cfg(vocab=V, beam=1, cand_k=0, win_m1=m1, win_m2=-1, ctc_weight=0.5, max_len_abs=9,
                       end_flags=4, eos_run=R)
        o = OracleUtt(x, cfg)
        att = np.full((1, V), -4.0, np.float32); att[0, 1] = -0.1
        o.score(att); o.commit()
        assert o.hyp(0)["tau"] == 26
        o.score(att)
        s_win, e_win = o.windows()
        assert s_win[0] == 26 - m1 and e_win[0] == T
        assert o.e2()[0][0] == want
    # strictness: E_t == X_t on the deciding frame is not "exceeds".  T = 2, R = 1, g = (1), and log values
    # (not normalised: the oracle takes any) chosen so that a single path carries each side and no rounding
    # occurs: label 1 is impossible at frame 2, hence phi_2(g) = x_1(1) + x_2(blank), and the best
    # extension is psi(g.2) = phi_1(g) + x_2(2) = x_1(1) + x_2(2); with x_2(blank) = x_2(2) they are equal
    xs = np.array([[-1.0, -0.5, -2.0, -2.0], [-1.0, -np.inf, -1.0, -2.0]], np.float32)
    cfg = make_cfg(vocab=4, beam=1, cand_k=0, ctc_weight=0.5, max_len_abs=2, end_flags=4, eos_run=1)
    o = OracleUtt(xs, cfg)
    att = np.full((1, 4), -4.0, np.float32); att[0, 1] = -0.1
    o.score(att); o.commit()
    o.score(att)
    el, fire, margin = o.e2()
    assert el[0] and margin[0] == 0.0 and not fire[0]
    xs2 = xs.copy(); xs2[1, 2] = np.nextafter(xs2[1, 2], np.float32(-2.0))      # X a hair smaller: exceeds
    o = OracleUtt(xs2, cfg)
    o.score(att); o.commit(); o.score(att)
    el, fire, margin = o.e2()
    assert el[0] and margin[0] > 0.0 and fire[0]


# --------------------------------------------------------------------------------------
# Algorithm 2: "p > best_score" is strict; equal joint scores are ordered by (parent slot, token);
# the final argmax over the ended set keeps the entry added first among equals
# --------------------------------------------------------------------------------------
def test_equal_scores_strictness_and_tie_breaks():
    V, T = 6, 8
    x = rand_logp(np.random.default_rng(3), T, V)
    # lambda = 0: joint scores are sums of attention values, so equal inputs give exactly equal scores
    cfg = make_cfg(vocab=V, beam=3, cand_k=0, ctc_weight=0.0, max_len_abs=4, end_flags=0)
    o = OracleUtt(x, cfg)
    a1 = np.full((3, V), -5.0, np.float32)
    a1[0, 2] = a1[0, 4] = -1.0                        # two labels with the same score
    a1[0, 3] = -2.0
    o.score(a1); o.rank()
    S = o.sorted_cands()
    assert [(int(c["parent"]), int(c["token"])) for c in S[:3]] == [(0, 2), (0, 4), (0, 3)]   # equal: token ascending
    o.commit()
    assert [list(o.hyp(j)["labels"]) for j in range(3)] == [[2], [4], [3]]
    # step 2: the two equal hypotheses get identical rows -> equal candidates from different parents
    a2 = np.full((3, V), -5.0, np.float32)
    a2[0, 1] = a2[1, 1] = -0.5
    a2[0, 3] = a2[1, 3] = -0.75
    a2[:, V - 1] = -0.5                               # eos exactly as good as the best extension
    o.score(a2); o.rank()
    S = o.sorted_cands()
    assert [(int(c["parent"]), int(c["token"])) for c in S[:4]] == [(0, 1), (1, 1), (0, 3), (1, 3)]   # equal: parent ascending
    je, best = o.joint_eos(), o.best
    assert je[0] == best and je[1] == best            # equal is not greater: nothing enters the ended set
    o.commit()
    assert o.ended() == []
    # step 3: eos a hair better than every extension for the two equal hypotheses -> two entries of equal score
    a3 = np.full((3, V), -5.0, np.float32)
    a3[0, 2] = a3[1, 2] = -0.5
    a3[0, V - 1] = a3[1, V - 1] = np.nextafter(np.float32(-0.5), np.float32(0.0))
    hyp0, hyp1 = list(o.hyp(0)["labels"]), list(o.hyp(1)["labels"])
    assert hyp0 == [2, 1] and hyp1 == [4, 1]
    o.score(a3); o.commit()
    ended = o.ended()
    assert len(ended) == 2 and ended[0]["score"] == ended[1]["score"]
    assert list(ended[0]["labels"]) == hyp0 and list(ended[1]["labels"]) == hyp1     # slot order
    while not o.finished:
        o.score(np.full((3, V), -9.0, np.float32)); o.commit()
    lab, sc, fb = o.result()
    assert list(lab) == hyp0 and sc == ended[0]["score"]      # the first of the equal entries
