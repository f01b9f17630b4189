"""GPU parity: libctcbs (through its C ABI) against the CPU oracle, step by step.

Tolerances (written out here): integer results (candidate ids, windows, selected parent/token,
time indices, flags, final labels) must be identical wherever the oracle's deciding margin
exceeds 1e-4; fused scores and CTC prefix scores within 1e-4 absolute (fp32 path, fp64 oracle).
"""
import numpy as np
import pytest

import gen
import oracle
from helpers import GpuDecoder, lockstep_decode, orc_cfg_from, host_att

pytestmark = pytest.mark.gpu


def small(name="cfg1", **over):
    w = gen.workload(name)
    w.update(over)
    w["eos_id"] = w["vocab"] - 1
    return w


def make_inputs(w, pad=np.nan):
    lens = gen.workload_lengths(w)
    return lens, gen.workload_ctc(w, lens, pad_value=pad)


def test_cfg0_full_vocabulary_single_utterance():
    w = gen.workload("cfg0")
    lens, ctc = make_inputs(w)
    rep, res = lockstep_decode(w, ctc, lens)
    print(rep, res["ntok"], res["score"])
    assert rep["utt_steps"] >= 5 and rep["max_score_err"] < 1e-4
    assert res["cells"] == int(res["oracle_cells"])


@pytest.mark.parametrize("variant", ["topk", "topk_window_e2", "topk_k80_window_e2", "fullv_window", "beam1", "wide_beam"])
def test_small_batches_ragged(variant):
    base = dict(n_utt=5, t_lo=37, t_hi=211, vocab=700, beam=6, cand_k=24, win_m1=-1, win_m2=-1,
                end_flags=3)
    if variant == "topk_window_e2":
        base.update(win_m1=12, win_m2=17, end_flags=7, eos_run=6)
    elif variant == "topk_k80_window_e2":              # more candidates than one wave ranks, eos-run rule armed
        base.update(cand_k=80, win_m1=12, win_m2=17, end_flags=7, eos_run=6)
    elif variant == "fullv_window":
        base.update(vocab=90, cand_k=0, win_m1=9, win_m2=30, end_flags=7, beam=5)
    elif variant == "beam1":
        base.update(beam=1, cand_k=300, vocab=421, end_flags=7, win_m1=25, win_m2=25)  # K > block size
    elif variant == "wide_beam":
        base.update(beam=17, cand_k=9, n_utt=3, win_m1=30, win_m2=30, end_flags=7)
    w = small("cfg1", **base)
    lens, ctc = make_inputs(w)
    rep, res = lockstep_decode(w, ctc, lens)
    print(variant, rep)
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4
    assert res["cells"] == int(res["oracle_cells"])
    assert rep["exact_sel_steps"] >= 0.9 * rep["utt_steps"]


def test_tied_attention_rows_take_the_radix_path():
    """Coarsely quantised attention rows: thousands of equal values, ties resolved to smaller ids."""
    w = small("cfg1", n_utt=3, t_lo=40, t_hi=90, vocab=3000, beam=4, cand_k=37, win_m1=20, win_m2=20,
              end_flags=3)
    lens, ctc = make_inputs(w)
    rep, res = lockstep_decode(w, ctc, lens, att_fn=lambda a: np.where(np.isnan(a), a, np.round(a / 4) * 4),
                               max_steps=12)
    print(rep)
    assert rep["utt_steps"] == 36 and rep["max_ctc_err"] < 1e-4
    w2 = small("cfg1", n_utt=2, t_lo=30, t_hi=50, vocab=900, beam=3, cand_k=300, end_flags=3)
    lens, ctc = make_inputs(w2)
    rep, res = lockstep_decode(w2, ctc, lens, att_fn=lambda a: np.where(np.isnan(a), a, -1.0), max_steps=6)
    assert rep["utt_steps"] == 12


def test_finalize_equals_backtrack_of_step_outputs():
    """Long utterance, wide beam: the trie walk that does not fit LDS; checked against the steps' own
    parent/token outputs (no oracle involved)."""
    w = small("cfg1", n_utt=2, t_lo=2300, t_hi=2400, vocab=64, beam=32, cand_k=0, win_m1=10, win_m2=10,
              end_flags=0, max_len_ratio=0.0, max_len_abs=2290)
    lens, ctc = make_inputs(w)
    dec = GpuDecoder(w, ctc, lens)
    rng = np.random.default_rng(1)
    hist = []
    att = rng.normal(size=(2, 32, 64)).astype(np.float32)
    att[:, :, 63] = -1e4
    for step in range(300):
        assert dec.step(att) == dec.m.OK
        if step % 50 == 49 or step < 3:
            pass
        out = dec.outputs()
        hist.append((out["parent"].copy(), out["token"].copy(), out["tau"].copy()))
    tok, nt, sc, frm, fl = dec.finalize(frames=True)
    dec.close()
    for u in range(2):
        assert nt[u] == 300 and fl[u] == 1          # nothing ended: best live hypothesis
        slot, want, want_f = 0, [], []
        for par, tk, tau in reversed(hist):
            want.append(tk[u, slot]); want_f.append(tau[u, slot]); slot = par[u, slot]
        assert tok[u, :300].tolist() == want[::-1] and frm[u, :300].tolist() == want_f[::-1]


def test_cfg1_shape_all_utterances():
    w = gen.workload("cfg1")
    lens, ctc = make_inputs(w)
    rep, res = lockstep_decode(w, ctc, lens, peek=True, max_steps=None)      # all 16 utterances
    print(rep)
    assert rep["utt_steps"] > 1200
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4


def test_batch_independence_and_padding_never_read():
    """An utterance decoded alone equals the same utterance inside a batch (padding NaN-poisoned)."""
    w = small("cfg1", n_utt=4, t_lo=50, t_hi=160, vocab=300, beam=4, cand_k=16, win_m1=15, win_m2=15,
              end_flags=7, eos_run=5)
    lens, ctc = make_inputs(w, pad=np.nan)

    def free_run(ctc_b, lens_b, utt_rows):
        dec = GpuDecoder(w, ctc_b, lens_b)
        U, Wb = len(lens_b), w["beam"]
        basis = gen.prefix_hash([])
        hashes = [[basis] * Wb for _ in range(U)]
        live = np.zeros((U, Wb), bool); live[:, 0] = True
        step = 0
        trace = []
        while True:
            step += 1
            # attention rows are keyed by the utterance's id in the full batch
            att = np.full((U, Wb, w["vocab"]), np.nan, np.float32)
            for i, u in enumerate(utt_rows):
                for j in range(Wb):
                    if live[i, j]:
                        att[i, j] = gen.att_row(w["seed"], u, step, hashes[i][j], w["vocab"])
            if dec.step(att) == dec.m.DONE:
                break
            out = dec.outputs()
            trace.append({k: v.copy() for k, v in out.items()})
            nh = [[basis] * Wb for _ in range(U)]
            for i in range(U):
                for n in range(Wb):
                    if out["live"][i, n]:
                        nh[i][n] = gen.prefix_hash_extend(hashes[i][out["parent"][i, n]], out["token"][i, n])
            hashes, live = nh, out["live"].astype(bool)
            if out["finished"].all():
                break
        r = dec.finalize(frames=True)
        dec.close()
        return trace, r

    tr_all, (tok, nt, sc, frm, fl) = free_run(ctc, lens, [0, 1, 2, 3])
    for u in (1, 3):
        t1 = int(lens[u])
        tr_one, (tok1, nt1, sc1, frm1, fl1) = free_run(ctc[u:u + 1, :t1], lens[u:u + 1], [u])
        assert nt1[0] == nt[u] and np.array_equal(tok1[0, :nt1[0]], tok[u, :nt[u]])
        assert sc1[0] == sc[u] and np.array_equal(frm1[0, :nt1[0]], frm[u, :nt[u]])
        for a, b in zip(tr_one, tr_all):
            for k in ("parent", "token", "score", "tau", "tau_end"):
                assert np.array_equal(a[k][0], b[k][u]), k
    # reversed batch order gives the same hypotheses
    tr_rev, (tokr, ntr, scr, _, _) = free_run(ctc[::-1].copy(), lens[::-1].copy(), [3, 2, 1, 0])
    for u in range(4):
        assert ntr[3 - u] == nt[u] and np.array_equal(tokr[3 - u, :nt[u]], tok[u, :nt[u]]) and scr[3 - u] == sc[u]


def test_constructed_eos_run_stop_and_time_stamps():
    """Sharply peaked posteriors with a blank tail: the eos-run rule stops the finished transcript,
    and the per-label frames returned by finalize are the emitting frames."""
    T, V = 50, 6
    x = np.full((T, V), 0.02 / (V - 1), np.float64)
    emits = {6: 1, 15: 2, 27: 3}
    for t in range(1, T + 1):
        x[t - 1, emits.get(t, 0)] = 0.98
    x = np.log(x).astype(np.float32)[None]
    w = small("cfg0", n_utt=1, vocab=V, beam=1, cand_k=0, ctc_weight=0.5, max_len_abs=20, end_flags=4,
              eos_run=10, t_lo=T, t_hi=T)
    dec = GpuDecoder(w, x, [T])
    stopped_at = None
    for step, want in enumerate([1, 2, 3, 4, 4, 4], start=1):
        att = np.full((1, 1, V), -4.0, np.float32)
        att[0, 0, want] = -0.1
        att[0, 0, V - 1] = -9.0
        if dec.step(att) == dec.m.DONE:
            break
        out = dec.outputs()
        if out["stopped"][0, 0] and stopped_at is None:
            stopped_at = step
        if out["finished"][0]:
            break
    tok, nt, sc, frm, fl = dec.finalize(frames=True)
    dec.close()
    assert stopped_at == 4 and nt[0] == 3 and tok[0, :3].tolist() == [1, 2, 3]
    assert frm[0, :3].tolist() == [6, 15, 27] and fl[0] == 0


def test_stats_poll_and_done():
    w = small("cfg1", n_utt=3, t_lo=30, t_hi=60, vocab=200, beam=3, cand_k=8)
    lens, ctc = make_inputs(w)
    dec = GpuDecoder(w, ctc, lens, poll_every=2)
    m = dec.m
    att = np.zeros((3, 3, 200), np.float32)
    rng = np.random.default_rng(0)
    n = 0
    fin_hist = []
    while True:
        att[:] = rng.normal(size=att.shape).astype(np.float32)
        rc = dec.step(att)
        if rc == m.DONE:
            break
        n += 1
        assert dec.out.step == n
        if n % 2 == 0:
            # a lower bound that lags by at most two poll intervals (here: four steps)
            assert 0 <= dec.out.n_finished <= int(dec.outputs()["finished"].sum())
            fin_hist.append(int(dec.outputs()["finished"].sum()))
            if len(fin_hist) > 3:
                assert dec.out.n_finished >= fin_hist[-4]
        else:
            assert dec.out.n_finished == -1
        assert n <= 20
    assert m.ctcbs_poll(dec.h) == 3
    cells, groups, steps = m.ctcbs_stats(dec.h)
    assert steps == n and cells > 0
    assert dec.step(att) == m.DONE          # stays done, enqueues nothing
    assert m.ctcbs_stats(dec.h)[2] == n
    dec.close()


def test_reset_reuses_a_handle_for_the_next_batch():
    """Decoding batch B on a handle that already decoded batch A equals decoding B on a fresh handle."""
    wa = small("cfg1", n_utt=3, t_lo=40, t_hi=120, vocab=400, beam=4, cand_k=12, win_m1=20, win_m2=20,
               end_flags=7, eos_run=5)
    lens_a, ctc_a = make_inputs(wa)
    wb = dict(wa); wb["seed"] = wa["seed"] + 1
    lens_b = gen.workload_lengths(wb)
    ctc_b = gen.workload_ctc(wb, lens_b)
    t_max = max(ctc_a.shape[1], ctc_b.shape[1])

    def pad(c):
        out = np.full((c.shape[0], t_max, c.shape[2]), np.nan, np.float32)
        out[:, :c.shape[1]] = c
        return out

    def run(dec, w, lens):
        U, Wb, V = len(lens), w["beam"], w["vocab"]
        basis = gen.prefix_hash([])
        hashes = [[basis] * Wb for _ in range(U)]
        live = np.zeros((U, Wb), bool); live[:, 0] = True
        step, trace = 0, []
        while True:
            step += 1
            att = host_att(w, step, hashes, live, U)
            if dec.step(att) == dec.m.DONE:
                break
            out = dec.outputs()
            trace.append((out["parent"].copy(), out["token"].copy(), out["score"].copy()))
            nh = [[basis] * Wb for _ in range(U)]
            for i in range(U):
                for n in range(Wb):
                    if out["live"][i, n]:
                        nh[i][n] = gen.prefix_hash_extend(hashes[i][out["parent"][i, n]], out["token"][i, n])
            hashes, live = nh, out["live"].astype(bool)
            if out["finished"].all():
                break
        return trace, dec.finalize(frames=True)

    import torch
    dec = GpuDecoder(wa, pad(ctc_a), lens_a)
    run(dec, wa, lens_a)
    d_b = torch.from_numpy(pad(ctc_b)).cuda()
    dec.m.ctcbs_reset(dec.h, d_b, lens_b)
    dec.lens = np.asarray(lens_b, np.int32)
    tr1, r1 = run(dec, wb, lens_b)
    dec.close()
    fresh = GpuDecoder(wb, pad(ctc_b), lens_b)
    tr2, r2 = run(fresh, wb, lens_b)
    fresh.close()
    assert len(tr1) == len(tr2)
    for a, b in zip(tr1, tr2):
        for x, y in zip(a, b):
            assert np.array_equal(x, y)
    for x, y in zip(r1, r2):
        assert np.array_equal(x, y)
    # a length beyond t_max is refused and leaves the handle usable
    bad = GpuDecoder(wa, pad(ctc_a), lens_a)
    import ctypes
    too_long = np.array([t_max + 1] * 3, np.int32)
    assert bad.m.lib().ctcbs_reset(bad.h, d_b.data_ptr(), too_long.ctypes.data_as(ctypes.c_void_p)) == bad.m.EINVAL
    run(bad, wa, lens_a)
    bad.close()


def test_abi_rejects_bad_arguments():
    import ctypes
    import torch
    import paper_2101_05600_amd as m
    L = m.lib()
    good = dict(n_utt=2, t_max=20, vocab=50, beam=3, cand_k=5)
    x = torch.zeros((2, 20, 50), device="cuda")
    lens = np.array([20, 11], np.int32)

    def create(**over):
        kw = dict(good); kw.update(over)
        out = ctypes.c_void_p(123)
        rc = L.ctcbs_create(ctypes.byref(m.make_config(**kw)), x.data_ptr(),
                            lens.ctypes.data_as(ctypes.c_void_p), ctypes.byref(out))
        return rc, out.value

    for bad in (dict(n_utt=0), dict(beam=0), dict(beam=33), dict(vocab=2), dict(blank_id=50),
                dict(eos_id=0), dict(cand_k=-1), dict(ctc_weight=1.5), dict(t_max=7000),
                dict(end_flags=8), dict(end_m=9), dict(eos_run=0, end_flags=4),
                dict(max_len_ratio=-1.0)):
        rc, h = create(**bad)
        assert rc == m.EINVAL and h is None, bad
    out = ctypes.c_void_p()
    cfg = m.make_config(**good)
    assert L.ctcbs_create(None, x.data_ptr(), lens.ctypes.data_as(ctypes.c_void_p), ctypes.byref(out)) == m.EINVAL
    assert L.ctcbs_create(ctypes.byref(cfg), None, lens.ctypes.data_as(ctypes.c_void_p), ctypes.byref(out)) == m.EINVAL
    bad_lens = np.array([21, 5], np.int32)
    assert L.ctcbs_create(ctypes.byref(cfg), x.data_ptr(), bad_lens.ctypes.data_as(ctypes.c_void_p),
                          ctypes.byref(out)) == m.EINVAL
    rc, h = create()
    assert rc == m.OK and h
    assert L.ctcbs_step(h, None, None) == m.EINVAL
    assert L.ctcbs_step(None, x.data_ptr(), None) == m.EINVAL
    tok = np.zeros((2, 1), np.int32); nt = np.zeros(2, np.int32); sc = np.zeros(2, np.float32)
    vp = ctypes.c_void_p
    att = torch.randn((2, 3, 50), device="cuda")
    att[:, :, 49] = -1.0e4                  # eos never attractive: nothing enters the ended set
    for _ in range(4):
        assert L.ctcbs_step(h, att.data_ptr(), None) == m.OK
    # capacity too small for a 4-label hypothesis (nothing has ended: best live hypothesis is returned)
    assert L.ctcbs_finalize(h, tok.ctypes.data_as(vp), 1, nt.ctypes.data_as(vp), sc.ctypes.data_as(vp),
                            None, None) == m.ECAP
    assert L.ctcbs_peek(h, 99, None, 0, None) == m.EINVAL
    assert m.ctcbs_strerror(m.ECAP) and m.ctcbs_strerror(-77)
    L.ctcbs_destroy(h)
    L.ctcbs_destroy(None)


def test_full_vocabulary_large_v_matches_oracle():
    """The unrestricted stress shape in miniature: every one of V-2 = 4998 ids scored per hypothesis
    (whole-wave chains over the full frame range, group lists by repeated arg-max)."""
    w = small("cfg4a", n_utt=2, t_lo=70, t_hi=131, beam=3, max_len_ratio=0.0, max_len_abs=9)
    lens, ctc = make_inputs(w)
    rep, res = lockstep_decode(w, ctc, lens, peek=True)
    print(rep)
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4
    assert res["cells"] == int(res["oracle_cells"])


@pytest.mark.parametrize("shape", ["regs", "odd_vocab", "full_v"])
def test_logits_mode_folds_log_softmax_in(shape):
    """att_is_logits = 1: the library normalises the decoder's raw scores itself; the oracle is fed the
    fp64 log_softmax of the very same fp32 logits."""
    over = dict(n_utt=3, t_lo=40, t_hi=100, vocab=1000, beam=4, cand_k=20, win_m1=20, win_m2=20,
                end_flags=7, eos_run=5)
    if shape == "odd_vocab":
        over.update(vocab=997)                       # not a multiple of four: the slower selection path
    elif shape == "full_v":
        over.update(vocab=120, cand_k=0)
    w = small("cfg1", **over)
    lens, ctc = make_inputs(w)

    def logits(a):                                   # per-row shift and scale-free noise: a valid logit row
        shift = np.nan_to_num(a[..., 5:6]) * 0.37 + 2.5
        return (a.astype(np.float64) + shift).astype(np.float32)

    def normalised(a):
        z = logits(a).astype(np.float64)
        m = np.nanmax(z, axis=-1, keepdims=True)
        lse = m + np.log(np.nansum(np.exp(z - m), axis=-1, keepdims=True))
        return (z - lse).astype(np.float32)

    wg = dict(w); wg["att_is_logits"] = 1
    rep, res = lockstep_decode(wg, ctc, lens, att_fn=normalised, gpu_att_fn=logits)
    print(shape, rep)
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4 and rep["utt_steps"] > 20


@pytest.mark.parametrize("m1,m2", [(5, 20), (5, -1), (12, 12)])
def test_batch_union_window(m1, m2):
    """The paper's batch-wide window (s^l = min s_ij, e^l = max e_ij) with its own margins M1 = 5, M2 in
    {20, inf}: every utterance of the batch is followed, the union couples them."""
    w = small("cfg1", n_utt=4, t_lo=45, t_hi=150, vocab=600, beam=4, cand_k=16, win_m1=m1, win_m2=m2,
              end_flags=3, win_union=1)
    lens, ctc = make_inputs(w)
    rep, res = lockstep_decode(w, ctc, lens)
    print(rep, res["cells"])
    assert rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4
    assert res["cells"] == int(res["oracle_cells"])
    # the union window is never narrower than the per-hypothesis one: at least as many terms
    w2 = dict(w); w2["win_union"] = 0
    rep2, res2 = lockstep_decode(w2, ctc, lens)
    assert res["cells"] / res["steps"] >= res2["cells"] / res2["steps"] * 0.999


def test_run_many_reproduces_single_decodes():
    """The library's executor (several batches in flight, two host threads, recorded rows served by
    ctcbs_att_replay) returns for every batch exactly what a lone decode of that batch returns;
    the lone decodes themselves are validated against the oracle step by step."""
    import torch
    import paper_2101_05600_amd as m
    ws = [small("cfg1", n_utt=3, t_lo=40, t_hi=110, vocab=600, beam=4, cand_k=16, win_m1=15, win_m2=15,
                end_flags=7, eos_run=5, seed=2101 + i) for i in range(3)]
    singles, recs, decs = [], [], []
    inputs = [make_inputs(w) for w in ws]
    T = max(ctc.shape[1] for _, ctc in inputs)             # one frame pitch for all: any handle takes any batch

    def padded(ctc):
        out = np.full((ctc.shape[0], T, ctc.shape[2]), np.nan, np.float32)
        out[:, :ctc.shape[1]] = ctc
        return out
    inputs = [(lens, padded(ctc)) for lens, ctc in inputs]
    try:
        for w, (lens, ctc) in zip(ws, inputs):
            rows = []
            rep, res = lockstep_decode(w, ctc, lens, gpu_att_fn=lambda a, rows=rows: rows.append(a.copy()) or a)
            assert rep["max_score_err"] < 1e-4
            singles.append(res)
            recs.append(rows)
            decs.append(GpuDecoder(dict(w, stream=torch.cuda.Stream().cuda_stream), ctc, lens, poll_every=4))
        keep = [[torch.from_numpy(r).cuda() for r in rows] for rows in recs]   # dead rows hold NaN
        torch.cuda.synchronize()
        m.ctcbs_run_many([d.h for d in decs], replay=[[t.data_ptr() for t in k] for k in keep], n_threads=2)
        for d, res in zip(decs, singles):
            tok, nt, sc, frm, fl = d.finalize()
            assert np.array_equal(tok, res["tokens"]) and np.array_equal(nt, res["ntok"])
            assert np.array_equal(sc, res["score"]) and np.array_equal(fl, res["flags"])
        # a Python provider (one thread): same results once more on fresh state
        for d, (lens, ctc) in zip(decs, inputs):
            m.ctcbs_reset(d.h, torch.from_numpy(ctc).cuda(), lens)
        m.ctcbs_run_many([d.h for d in decs], att_fn=lambda i, step, prev: keep[i][min(step, len(keep[i])) - 1])
        for d, res in zip(decs, singles):
            tok, nt, sc, frm, fl = d.finalize()
            assert np.array_equal(tok, res["tokens"]) and np.array_equal(sc, res["score"])
        # the job queue: five jobs (the three batches, two of them twice) on two of the handles
        jobs = [0, 1, 2, 1, 0]
        data = [(torch.from_numpy(ctc).cuda(), lens) for lens, ctc in inputs]
        got = [None] * len(jobs)

        def job_fn(job, slot, h, phase):
            b = jobs[job]
            if phase == m.JOB_LOAD:
                m.ctcbs_reset(h, data[b][0], data[b][1])
            else:
                got[job] = m.ctcbs_finalize(h, 3, singles[b]["tokens"].shape[1])
        # (the three batches share shapes: any handle takes any of them after a reset)
        m.ctcbs_run_queue([decs[0].h, decs[1].h], len(jobs), job_fn,
                          replay=[[t.data_ptr() for t in keep[b]] for b in jobs], n_threads=2)
        for job, b in enumerate(jobs):
            tok, nt, sc, frm, fl = got[job]
            assert np.array_equal(tok, singles[b]["tokens"]) and np.array_equal(sc, singles[b]["score"])
    finally:
        for d in decs:
            d.close()


def test_offline_job_segments_to_batches_to_queue():
    """The offline recipe end to end on a small scale (Sec. 4.2 and 4.4): a recording is cut into
    segments of bounded length, the segments are sorted by length and dealt into batches of four (the
    last one not full: unused slots), and the batches are decoded through the job queue on two
    handles.  Every batch's lone decode is validated against the oracle step by step; the queue must
    return exactly those results."""
    import torch
    import paper_2101_05600_amd as m
    seg = np.concatenate([m.ctcbs_hard_segments(431, 40, 75), m.ctcbs_hard_segments(158, 40, 75)])
    assert seg.sum() == 431 + 158 and seg.max() <= 75
    order, begin = m.ctcbs_plan_batches(seg, 4)
    n_b = len(begin) - 1
    assert n_b == 3 and begin[-1] == len(seg) == 9           # 4 + 4 + 1
    T = int(seg.max())
    ws, data, singles, recs = [], [], [], []
    for j in range(n_b):
        ids = order[begin[j]:begin[j + 1]]
        lens = np.zeros(4, np.int32)
        lens[:len(ids)] = seg[ids]
        w = small("cfg1", n_utt=4, vocab=300, beam=4, cand_k=12, win_m1=12, win_m2=12, end_flags=7, eos_run=4,
                  seed=77 + j)
        ctc = np.full((4, T, 300), np.nan, np.float32)
        g = gen.workload_ctc(w, np.maximum(lens, 1))
        for u in range(4):
            ctc[u, :lens[u]] = g[u, :lens[u]]
        rows = []
        rep, res = lockstep_decode(w, ctc, lens, check_utts=[u for u in range(4) if lens[u] > 0],
                                   gpu_att_fn=lambda a, rows=rows: rows.append(a.copy()) or a)
        assert rep["max_score_err"] < 1e-4
        ws.append(w); data.append((torch.from_numpy(ctc).cuda(), lens)); singles.append(res)
        recs.append([torch.from_numpy(r).cuda() for r in rows])
    decs = [GpuDecoder(dict(ws[0], stream=torch.cuda.Stream().cuda_stream), data[0][0].cpu().numpy(), data[0][1],
                       poll_every=3) for _ in range(2)]
    try:
        got = [None] * n_b
        cap = max(r["tokens"].shape[1] for r in singles)

        def job_fn(job, slot, h, phase):
            if phase == m.JOB_LOAD:
                m.ctcbs_reset(h, data[job][0], data[job][1])
            else:
                got[job] = m.ctcbs_finalize(h, 4, cap)
        torch.cuda.synchronize()
        m.ctcbs_run_queue([d.h for d in decs], n_b, job_fn,
                          replay=[[t.data_ptr() for t in rec] for rec in recs], n_threads=2)
        for j in range(n_b):
            tok, nt, sc, frm, fl = got[j]
            c = singles[j]["tokens"].shape[1]
            assert np.array_equal(tok[:, :c], singles[j]["tokens"]) and np.array_equal(nt, singles[j]["ntok"])
            assert np.array_equal(sc, singles[j]["score"]) and np.array_equal(fl, singles[j]["flags"])
        assert (got[-1][1][1:] == 0).all()                   # the unused slots of the last batch
    finally:
        for d in decs:
            d.close()


def test_executor_error_paths():
    """A failing callback stops the executor with its error; the handles stay usable."""
    import torch
    import paper_2101_05600_amd as m
    w = small("cfg1", n_utt=2, t_lo=30, t_hi=50, vocab=300, beam=3, cand_k=8, win_m1=10, win_m2=10, end_flags=3)
    lens, ctc = make_inputs(w)
    decs = [GpuDecoder(dict(w, stream=torch.cuda.Stream().cuda_stream), ctc, lens, poll_every=2) for _ in range(2)]
    try:
        d_ctc = torch.from_numpy(np.ascontiguousarray(ctc)).cuda()
        rows = torch.zeros((2, 3, 300), dtype=torch.float32, device="cuda")
        rows[:] = torch.log_softmax(torch.arange(300, dtype=torch.float32, device="cuda") * 0.01, dim=0)

        class Boom(RuntimeError):
            pass

        def bad_job(job, slot, h, phase):
            if job == 1 and phase == m.JOB_LOAD:
                raise Boom("no such batch")
            if phase == m.JOB_LOAD:
                m.ctcbs_reset(h, d_ctc, lens)
        with pytest.raises(Boom):
            m.ctcbs_run_queue([d.h for d in decs], 4, bad_job, att_fn=lambda job, step, prev: rows, n_threads=2)

        def bad_att(index, step, prev):
            if step == 3:
                raise Boom("decoder failed")
            return rows
        for d in decs:
            m.ctcbs_reset(d.h, d_ctc, lens)
        with pytest.raises(m.CtcbsError):
            m.ctcbs_run_many([d.h for d in decs], att_fn=bad_att)
        with pytest.raises(m.CtcbsError):
            m.ctcbs_run_many([d.h for d in decs], replay=[[rows.data_ptr()]] * 2, n_threads=0)
        # after the failures: reset and decode normally, both handles give the same result
        for d in decs:
            m.ctcbs_reset(d.h, d_ctc, lens)
        m.ctcbs_run_many([d.h for d in decs], att_fn=lambda i, step, prev: rows, n_threads=1)
        r0, r1 = decs[0].finalize(), decs[1].finalize()
        assert np.array_equal(r0[0], r1[0]) and np.array_equal(r0[2], r1[2]) and (r0[1] > 0).all()
    finally:
        for d in decs:
            d.close()


def _decode_outputs(w, ctc, lens, keep, att_offset=0):
    """Free-running decode (no oracle): every step's outputs, and the result.  att_offset: the attention
    buffer handed to ctcbs_step starts that many floats after a 16-byte boundary."""
    import torch
    import paper_2101_05600_amd as m
    U, Wb, V = len(lens), w["beam"], w["vocab"]
    cfg = m.make_config(n_utt=U, t_max=ctc.shape[1], keep_candidates=keep,
                        **{k: v for k, v in w.items() if k not in ("n_utt", "keep_candidates")})
    d_ctc = torch.from_numpy(np.ascontiguousarray(ctc)).cuda()
    h = m.ctcbs_create(cfg, d_ctc, lens)
    out = m.StepOut()
    buf = torch.empty(U * Wb * V + 8, dtype=torch.float32, device="cuda")
    d_att = buf[att_offset:att_offset + U * Wb * V].view(U, Wb, V)
    assert d_att.data_ptr() % 16 == (4 * att_offset) % 16
    steps = []
    try:
        basis = gen.prefix_hash([])
        hashes = [[basis] * Wb for _ in range(U)]
        live = np.zeros((U, Wb), bool)
        live[:, 0] = True
        for step in range(1, 10000):
            att = host_att(w, step, hashes, live, U)
            d_att.copy_(torch.from_numpy(att))
            if m.ctcbs_step(h, d_att.data_ptr(), out) == m.DONE:
                break
            g = lambda p, shape, dt: m.view(p, shape, dt).cpu().numpy()
            o = dict(parent=g(out.d_parent, (U, Wb), np.int32), token=g(out.d_token, (U, Wb), np.int32),
                     score=g(out.d_score, (U, Wb), np.float32), live=g(out.d_live, (U, Wb), np.uint8),
                     finished=g(out.d_finished, (U,), np.uint8), tau=g(out.d_tau, (U, Wb), np.int32),
                     eos_added=g(out.d_eos_added, (U, Wb), np.uint8), stopped=g(out.d_stopped, (U, Wb), np.uint8))
            steps.append(o)
            new_hashes = [[basis] * Wb for _ in range(U)]
            for u in range(U):
                for n in range(Wb):
                    if o["live"][u, n]:
                        new_hashes[u][n] = gen.prefix_hash_extend(hashes[u][o["parent"][u, n]], o["token"][u, n])
            hashes, live = new_hashes, o["live"].astype(bool)
            if o["finished"].all():
                break
        peek_rc = m.lib().ctcbs_peek(h, m.PEEK_CAND_ID, None, 0, None)
        res = m.ctcbs_finalize(h, U, 400)
    finally:
        m.ctcbs_destroy(h)
    return steps, res, peek_rc


def test_keep_candidates_off_gives_the_same_steps_and_results():
    """The per-candidate arrays that ctcbs_peek reads are a create-time option; without them the step
    outputs and the results are bit-identical (and peeking at them is refused)."""
    import paper_2101_05600_amd as m
    w = small("cfg1", n_utt=4, t_lo=60, t_hi=170, vocab=1200, beam=6, cand_k=24, win_m1=15, win_m2=20,
              end_flags=7, eos_run=5)
    lens, ctc = make_inputs(w)
    s1, r1, rc1 = _decode_outputs(w, ctc, lens, keep=1)
    s0, r0, rc0 = _decode_outputs(w, ctc, lens, keep=0)
    assert rc1 == m.OK and rc0 == m.ESTATE
    assert len(s1) == len(s0) and len(s1) > 10
    for a, b in zip(s1, s0):
        for k in a:
            assert np.array_equal(a[k], b[k]), k
    for a, b in zip(r1, r0):
        assert (a is None and b is None) or np.array_equal(a, b)


def test_attention_rows_off_a_16_byte_boundary():
    """An attention buffer that does not start on a 16-byte boundary takes the slower candidate
    selection and gives the same decode."""
    w = small("cfg1", n_utt=3, t_lo=50, t_hi=120, vocab=1200, beam=4, cand_k=16, win_m1=15, win_m2=20,
              end_flags=7, eos_run=5)
    lens, ctc = make_inputs(w)
    s_al, r_al, _ = _decode_outputs(w, ctc, lens, keep=0, att_offset=0)
    s_un, r_un, _ = _decode_outputs(w, ctc, lens, keep=0, att_offset=1)
    assert len(s_al) == len(s_un) and len(s_al) > 10
    for a, b in zip(s_al, s_un):
        for k in a:
            assert np.array_equal(a[k], b[k]), k
    for a, b in zip(r_al, r_un):
        assert (a is None and b is None) or np.array_equal(a, b)
