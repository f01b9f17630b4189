"""ctcbs_step_static (the step whose scratch lies in the library's fixed array, for callers that cannot
allocate) against ctcbs_step, through the C ABI: two decodes in a row on one GPU, the second with a
smaller batch, every step's outputs and the results bit for bit; and the size limit."""
import numpy as np
import pytest

import gen
from helpers import host_att

pytestmark = pytest.mark.gpu


def _decode(w, ctc, lens, static):
    import torch
    import paper_2101_05600_amd as m
    U, Wb, V = len(lens), w["beam"], w["vocab"]
    cfg = m.make_config(n_utt=U, t_max=ctc.shape[1], keep_candidates=0,
                        **{k: v for k, v in w.items() if k not in ("n_utt", "keep_candidates")})
    d_ctc = torch.from_numpy(np.ascontiguousarray(ctc)).cuda()
    h = m.ctcbs_create(cfg, d_ctc, lens)
    step_fn = m.ctcbs_step_static if static else m.ctcbs_step
    out = m.StepOut()
    d_att = torch.empty((U, Wb, V), dtype=torch.float32, device="cuda")
    steps = []
    try:
        basis = gen.prefix_hash([])
        hashes = [[basis] * Wb for _ in range(U)]
        live = np.zeros((U, Wb), bool)
        live[:, 0] = True
        for step in range(1, 10000):
            d_att.copy_(torch.from_numpy(host_att(w, step, hashes, live, U)))
            if step_fn(h, d_att, out) == m.DONE:
                break
            g = lambda p, shape, dt: m.view(p, shape, dt).cpu().numpy()
            o = dict(parent=g(out.d_parent, (U, Wb), np.int32), token=g(out.d_token, (U, Wb), np.int32),
                     score=g(out.d_score, (U, Wb), np.float32), live=g(out.d_live, (U, Wb), np.uint8),
                     finished=g(out.d_finished, (U,), np.uint8), tau=g(out.d_tau, (U, Wb), np.int32),
                     tau_end=g(out.d_tau_end, (U, Wb), np.int32),
                     eos_added=g(out.d_eos_added, (U, Wb), np.uint8), stopped=g(out.d_stopped, (U, Wb), np.uint8))
            if static:   # the windows and eos scores of the step come back from the fixed array
                o["win_s"] = m.ctcbs_peek(h, m.PEEK_WIN_S).copy()
                o["joint_eos"] = m.ctcbs_peek(h, m.PEEK_JOINT_EOS).copy()
            steps.append(o)
            new_hashes = [[basis] * Wb for _ in range(U)]
            for u in range(U):
                for n in range(Wb):
                    if o["live"][u, n]:
                        new_hashes[u][n] = gen.prefix_hash_extend(hashes[u][o["parent"][u, n]], o["token"][u, n])
            hashes, live = new_hashes, o["live"].astype(bool)
            if o["finished"].all():
                break
        res = m.ctcbs_finalize(h, U, 400, want_frames=True)
        stats = m.ctcbs_stats(h)
    finally:
        m.ctcbs_destroy(h)
    return steps, res, stats


def _same(a, b):
    sa, ra, ta = a
    sb, rb, tb = b
    assert len(sa) == len(sb) and len(sa) > 10
    for x, y in zip(sa, sb):
        for k in y:
            assert np.array_equal(x[k], y[k]), k
    for x, y in zip(ra, rb):
        assert np.array_equal(x, y)
    assert ta == tb


def test_static_step_equals_the_allocating_one_twice_in_a_row():
    big = gen.workload("cfg1")
    big.update(n_utt=6, t_lo=60, t_hi=180, vocab=1200, beam=8, cand_k=24, win_m1=15, win_m2=20, end_flags=7,
               eos_run=5)
    big["eos_id"] = big["vocab"] - 1
    small = dict(big, n_utt=2, beam=3, cand_k=10, t_lo=40, t_hi=90, seed=big["seed"] + 1)
    runs = []
    for w in (big, small):                     # the second, smaller decode finds the first one's leftovers in the array
        lens = gen.workload_lengths(w)
        ctc = gen.workload_ctc(w, lens, pad_value=np.nan)
        runs.append((w, ctc, lens, _decode(w, ctc, lens, static=True)))
    for w, ctc, lens, got in runs:
        _same(got, _decode(w, ctc, lens, static=False))


def test_static_step_rejects_what_does_not_fit():
    import torch
    import paper_2101_05600_amd as m
    L = m.lib()
    # 40*U*Wb + 24*U*Wb*Wb bytes beyond the 4 MiB array; and more than 256 candidates per hypothesis
    for kw in (dict(n_utt=2048, beam=10, cand_k=8), dict(n_utt=2, beam=2, cand_k=300)):
        w = gen.workload("cfg1")
        w.update(t_lo=8, t_hi=8, vocab=400, win_m1=4, win_m2=4, **kw)
        w["eos_id"] = w["vocab"] - 1
        U = w["n_utt"]
        lens = np.full(U, 8, np.int32)
        ctc = torch.zeros((U, 8, w["vocab"]), dtype=torch.float32, device="cuda")
        cfg = m.make_config(t_max=8, keep_candidates=0, **{k: v for k, v in w.items() if k != "keep_candidates"})
        h = m.ctcbs_create(cfg, ctc, lens)
        try:
            att = torch.zeros((U, w["beam"], w["vocab"]), dtype=torch.float32, device="cuda")
            assert L.ctcbs_step_static(h, att.data_ptr(), None) == m.EINVAL
            assert L.ctcbs_step(h, att.data_ptr(), None) == m.OK     # the handle itself is fine
        finally:
            m.ctcbs_destroy(h)
