"""Shared pieces of the parity tests: drive libctcbs step by step and feed the lock-step check."""
import ctypes

import numpy as np

import gen
import oracle
from oracle.lockstep import Lockstep

PEEKS = None


def orc_cfg_from(w):
    kw = {k: w[k] for k in (
        "vocab", "beam", "blank_id", "eos_id", "cand_k", "win_m1", "win_m2", "ctc_weight",
        "length_bonus", "max_len_ratio", "max_len_abs", "end_flags", "end_m", "end_d", "end_c",
        "eos_run")}
    kw["win_union"] = w.get("win_union", 0)
    # the C ABI carries these three as fp32: give the oracle the same values
    for k in ("ctc_weight", "length_bonus", "max_len_ratio", "end_d"):
        kw[k] = float(np.float32(kw[k]))
    return oracle.make_cfg(**kw)


def host_att(w, step, hashes, live, n_utt, dead_fill=np.nan):
    """[U, Wb, V] attention rows of this step from the host generator; dead rows poisoned."""
    Wb, V = w["beam"], w["vocab"]
    att = np.full((n_utt, Wb, V), dead_fill, dtype=np.float32)
    idx = np.argwhere(live)
    if len(idx):
        rows = gen.att_rows(w["seed"], idx[:, 0], step, [hashes[u][j] for u, j in idx], V,
                            w["att_scale"])
        att[idx[:, 0], idx[:, 1]] = rows
    return att


class GpuDecoder:
    """Thin driver of the C ABI for tests: owns device buffers, returns numpy copies."""

    def __init__(self, w, ctc, lens, poll_every=0):
        import torch
        import paper_2101_05600_amd as m
        self.m, self.torch, self.w = m, torch, w
        self.U, self.Wb, self.V = len(lens), w["beam"], w["vocab"]
        self.lens = np.asarray(lens, np.int32)
        t_max = ctc.shape[1]
        self.cfg = m.make_config(n_utt=self.U, t_max=t_max, poll_every=poll_every,
                                 **{k: v for k, v in w.items() if k not in ("n_utt",)})
        d_ctc = torch.from_numpy(np.ascontiguousarray(ctc)).cuda()
        self.h = m.ctcbs_create(self.cfg, d_ctc, self.lens)
        del d_ctc
        self.out = m.StepOut()
        self.d_att = torch.empty((self.U, self.Wb, self.V), dtype=torch.float32, device="cuda")
        self.K = int(m.ctcbs_peek(self.h, m.PEEK_N_CAND)[0])

    def step(self, att):
        self.d_att.copy_(self.torch.from_numpy(att))
        rc = self.m.ctcbs_step(self.h, self.d_att, self.out)
        return rc

    def outputs(self):
        m, o, U, Wb = self.m, self.out, self.U, self.Wb
        g = lambda p, shape, dt: m.view(p, shape, dt).cpu().numpy()
        return dict(parent=g(o.d_parent, (U, Wb), np.int32), token=g(o.d_token, (U, Wb), np.int32),
                    score=g(o.d_score, (U, Wb), np.float32), live=g(o.d_live, (U, Wb), np.uint8),
                    finished=g(o.d_finished, (U,), np.uint8), tau=g(o.d_tau, (U, Wb), np.int32),
                    tau_end=g(o.d_tau_end, (U, Wb), np.int32),
                    eos_added=g(o.d_eos_added, (U, Wb), np.uint8),
                    stopped=g(o.d_stopped, (U, Wb), np.uint8))

    def peeks(self):
        m, U, Wb, K = self.m, self.U, self.Wb, self.K
        pk = lambda what: m.ctcbs_peek(self.h, what)
        return dict(cand_id=pk(m.PEEK_CAND_ID).reshape(U, Wb, K),
                    cand_ctc=pk(m.PEEK_CAND_CTC).reshape(U, Wb, K),
                    cand_joint=pk(m.PEEK_CAND_JOINT).reshape(U, Wb, K),
                    win_s=pk(m.PEEK_WIN_S).reshape(U, Wb), win_e=pk(m.PEEK_WIN_E).reshape(U, Wb),
                    ctc_eos=pk(m.PEEK_CTC_EOS).reshape(U, Wb), joint_eos=pk(m.PEEK_JOINT_EOS).reshape(U, Wb))

    def finalize(self, frames=False):
        cap = int(max(oracle.lib().orc_lmax(ctypes.byref(orc_cfg_from(self.w)), int(t)) for t in self.lens if t > 0))
        return self.m.ctcbs_finalize(self.h, self.U, cap, want_frames=frames)

    def close(self):
        if self.h:
            self.m.ctcbs_destroy(self.h)
            self.h = None


class EmuDecoder(GpuDecoder):
    """The same driver over the CPU build of the kernels (tests/cpu_emu): "device" memory is host
    memory, so plain numpy arrays stand where GpuDecoder has CUDA tensors.  The caller must have
    pointed the binding at the CPU library before its first use (see tests/test_cpu_emulation.py)."""

    def __init__(self, w, ctc, lens, poll_every=0):
        import paper_2101_05600_amd as m
        self.m, self.w = m, w
        self.U, self.Wb, self.V = len(lens), w["beam"], w["vocab"]
        self.lens = np.asarray(lens, np.int32)
        self.cfg = m.make_config(n_utt=self.U, t_max=ctc.shape[1], poll_every=poll_every,
                                 **{k: v for k, v in w.items() if k not in ("n_utt",)})
        d_ctc = np.ascontiguousarray(ctc, dtype=np.float32)
        self.h = m.ctcbs_create(self.cfg, d_ctc.ctypes.data, self.lens)
        self.out = m.StepOut()
        self.d_att = np.empty((self.U, self.Wb, self.V), dtype=np.float32)
        self.K = int(m.ctcbs_peek(self.h, m.PEEK_N_CAND)[0])

    def step(self, att):
        self.d_att[...] = att
        return self.m.ctcbs_step(self.h, self.d_att.ctypes.data, self.out)

    def outputs(self):
        o, U, Wb = self.out, self.U, self.Wb

        def g(p, shape, dt):
            n = int(np.prod(shape)) * np.dtype(dt).itemsize
            return np.frombuffer((ctypes.c_char * n).from_address(int(p)), dtype=dt).reshape(shape).copy()
        return dict(parent=g(o.d_parent, (U, Wb), np.int32), token=g(o.d_token, (U, Wb), np.int32),
                    score=g(o.d_score, (U, Wb), np.float32), live=g(o.d_live, (U, Wb), np.uint8),
                    finished=g(o.d_finished, (U,), np.uint8), tau=g(o.d_tau, (U, Wb), np.int32),
                    tau_end=g(o.d_tau_end, (U, Wb), np.int32),
                    eos_added=g(o.d_eos_added, (U, Wb), np.uint8),
                    stopped=g(o.d_stopped, (U, Wb), np.uint8))


def lockstep_decode(w, ctc, lens, peek=True, check_utts=None, max_steps=None, progress=None,
                    att_fn=None, gpu_att_fn=None, eps=1e-4, decoder_cls=None):
    """Decode the batch on the GPU with host-generated attention rows, validating every step of
    the utterances in check_utts (default: all) against the oracle.  Returns (report, results)."""
    U, Wb = len(lens), w["beam"]
    check = list(range(U)) if check_utts is None else list(check_utts)
    ls = Lockstep([ctc[u, :lens[u]] for u in check], orc_cfg_from(w), eps=eps, utt_ids=check)
    dec = (decoder_cls or GpuDecoder)(w, ctc, lens)
    try:
        basis = gen.prefix_hash([])
        hashes = [[basis] * Wb for _ in range(U)]
        live = np.zeros((U, Wb), bool)
        live[:, 0] = True
        step = 0
        while True:
            step += 1
            if max_steps is not None and step > max_steps:
                break
            raw = host_att(w, step, hashes, live, U)
            att = att_fn(raw) if att_fn is not None else raw
            rc = dec.step(gpu_att_fn(raw) if gpu_att_fn is not None else att)
            if rc == dec.m.DONE:
                break
            out = dec.outputs()
            ls.step(att, out, dec.peeks() if peek else None)
            new_hashes = [[basis] * Wb for _ in range(U)]
            for u in range(U):
                for n in range(Wb):
                    if out["live"][u, n]:
                        new_hashes[u][n] = gen.prefix_hash_extend(hashes[u][out["parent"][u, n]],
                                                                  out["token"][u, n])
            hashes = new_hashes
            live = out["live"].astype(bool)
            if progress:
                progress(step, out)
            if out["finished"].all():
                break
        tok, nt, sc, frm, fl = dec.finalize(frames=True)
        if max_steps is None:
            ls.check_results(tok, nt, sc, fl, frames=frm)
        cells, _groups, steps = dec.m.ctcbs_stats(dec.h)
        res = dict(tokens=tok, ntok=nt, score=sc, flags=fl, cells=cells, steps=steps,
                   oracle_cells=sum(o.cells for o in ls.utts))
        return ls.report, res
    finally:
        dec.close()
