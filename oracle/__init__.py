"""CPU oracle (fp64, plain C) of the batched joint CTC/attention beam-search step.

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg.  It shares no code with the GPU library and the
product path never calls it.  See ``ctc_oracle.c`` for what each routine follows.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")
_lib = None

LOG0 = -1.0e30
END_BASELINE, END_TAU_COUNT, END_EOS_RUN = 1, 2, 4


def build():
    subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-o", _SO,
                           os.path.join(_HERE, "ctc_oracle.c"), "-lm"])


class OrcCfg(ctypes.Structure):
    _fields_ = [("vocab", ctypes.c_int32), ("beam", ctypes.c_int32), ("blank_id", ctypes.c_int32),
                ("eos_id", ctypes.c_int32), ("cand_k", ctypes.c_int32), ("win_m1", ctypes.c_int32),
                ("win_m2", ctypes.c_int32), ("max_len_abs", ctypes.c_int32),
                ("end_flags", ctypes.c_int32), ("end_m", ctypes.c_int32), ("end_c", ctypes.c_int32),
                ("eos_run", ctypes.c_int32), ("win_union", ctypes.c_int32), ("pad_", ctypes.c_int32),
                ("ctc_weight", ctypes.c_double),
                ("length_bonus", ctypes.c_double), ("max_len_ratio", ctypes.c_double),
                ("end_d", ctypes.c_double)]


class OrcCand(ctypes.Structure):
    _fields_ = [("parent", ctypes.c_int32), ("token", ctypes.c_int32), ("joint", ctypes.c_double),
                ("ctc", ctypes.c_double), ("att", ctypes.c_double)]


CAND_DTYPE = np.dtype([("parent", "<i4"), ("token", "<i4"), ("joint", "<f8"), ("ctc", "<f8"),
                       ("att", "<f8")])


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build()
        L = ctypes.CDLL(_SO)
        vp, i32, dbl = ctypes.c_void_p, ctypes.c_int32, ctypes.c_double
        L.orc_create.restype = vp
        L.orc_create.argtypes = [vp, i32, i32, ctypes.POINTER(OrcCfg)]
        L.orc_destroy.argtypes = [vp]
        L.orc_lmax.restype = i32
        L.orc_lmax.argtypes = [ctypes.POINTER(OrcCfg), i32]
        L.orc_score.restype = i32
        L.orc_score.argtypes = [vp, vp]
        L.orc_rank.restype = i32
        L.orc_rank.argtypes = [vp, vp]
        L.orc_commit.restype = i32
        L.orc_commit.argtypes = [vp, i32, vp, vp, vp, vp]
        L.orc_override.argtypes = [vp, vp, vp, i32]
        L.orc_step_auto.restype = i32
        L.orc_step_auto.argtypes = [vp, vp]
        L.orc_result.restype = i32
        L.orc_result.argtypes = [vp, vp, i32, ctypes.POINTER(dbl), ctypes.POINTER(i32)]
        for name in ("orc_step_index", "orc_finished", "orc_T", "orc_lmax_of", "orc_k",
                     "orc_n_sorted", "orc_n_ended"):
            getattr(L, name).restype = i32
            getattr(L, name).argtypes = [vp]
        for name in ("orc_cells", "orc_best", "orc_e1_margin"):
            getattr(L, name).restype = dbl
            getattr(L, name).argtypes = [vp]
        for name in ("orc_sorted", "orc_win_s", "orc_win_e", "orc_cand_id", "orc_cand_ctc",
                     "orc_cand_att", "orc_cand_joint", "orc_ctc_eos", "orc_joint_eos",
                     "orc_e2_eligible", "orc_e2_fire", "orc_e2_margin", "orc_child_max_n",
                     "orc_child_max_b", "orc_child_lo"):
            getattr(L, name).restype = vp
            getattr(L, name).argtypes = [vp]
        L.orc_ended_get.argtypes = [vp, i32, vp, vp, vp, vp]
        L.orc_hyp_get.argtypes = [vp, i32] + [vp] * 9
        L.orc_result_frames.restype = i32
        L.orc_result_frames.argtypes = [vp, vp, vp, i32, ctypes.POINTER(dbl), ctypes.POINTER(i32)]
        for name in ("orc_hyp_labels", "orc_hyp_gn", "orc_hyp_gb", "orc_ended_labels", "orc_ended_taus",
                     "orc_hyp_taus"):
            getattr(L, name).restype = vp
            getattr(L, name).argtypes = [vp, i32]
        L.orc_prefix_and_full.restype = i32
        L.orc_prefix_and_full.argtypes = [vp, i32, i32, i32, vp, i32, ctypes.POINTER(dbl),
                                          ctypes.POINTER(dbl)]
        L.orc_batch_step_auto.argtypes = [vp, i32, vp, vp]
        L.orc_union_contrib.restype = i32
        L.orc_union_contrib.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.orc_set_union.argtypes = [vp, i32, i32]
        L.orc_end_detect.restype = i32
        L.orc_end_detect.argtypes = [ctypes.POINTER(OrcCfg), i32, i32, i32, vp, vp, vp,
                                     ctypes.POINTER(dbl)]
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _view(ptr, dtype, n):
    if n == 0:
        return np.empty(0, dtype=dtype)
    buf = (ctypes.c_char * (np.dtype(dtype).itemsize * n)).from_address(ptr)
    return np.frombuffer(buf, dtype=dtype, count=n)


def make_cfg(vocab, beam, blank_id=0, eos_id=None, cand_k=0, win_m1=-1, win_m2=-1, ctc_weight=0.3,
             length_bonus=0.0, max_len_ratio=0.0, max_len_abs=0, end_flags=3, end_m=3, end_d=-10.0,
             end_c=2, eos_run=10, win_union=0, **_ignored):
    c = OrcCfg()
    c.vocab, c.beam, c.blank_id = vocab, beam, blank_id
    c.eos_id = vocab - 1 if eos_id is None else eos_id
    c.cand_k, c.win_m1, c.win_m2 = cand_k, win_m1, win_m2
    c.ctc_weight, c.length_bonus = ctc_weight, length_bonus
    c.max_len_ratio, c.max_len_abs = max_len_ratio, max_len_abs
    c.end_flags, c.end_m, c.end_d, c.end_c, c.eos_run = end_flags, end_m, end_d, end_c, eos_run
    c.win_union = win_union
    return c


def prefix_and_full(x, labels, blank_id=0):
    """(log psi(g), log phi_T(g)) of label sequence g under posteriors x[T, V] (unrestricted)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    lab = np.ascontiguousarray(labels, dtype=np.int32)
    a, b = ctypes.c_double(), ctypes.c_double()
    lib().orc_prefix_and_full(_p(x), x.shape[0], x.shape[1], blank_id, _p(lab), lab.size,
                              ctypes.byref(a), ctypes.byref(b))
    return a.value, b.value


def end_detect(cfg, T, l, lens, taus, scores):
    """Algorithm 3 on a plain list of ended hypotheses -> (detected, margin)."""
    ln = np.ascontiguousarray(lens, dtype=np.int32)
    ta = np.ascontiguousarray(taus, dtype=np.int32)
    sc = np.ascontiguousarray(scores, dtype=np.float64)
    m = ctypes.c_double()
    r = lib().orc_end_detect(ctypes.byref(cfg), T, l, ln.size, _p(ln), _p(ta), _p(sc),
                             ctypes.byref(m))
    return bool(r), m.value


class OracleUtt:
    """One utterance's beam search, driven step by step."""

    def __init__(self, x, cfg: OrcCfg):
        self.x = np.ascontiguousarray(x, dtype=np.float32)   # keep alive: the C side borrows it
        assert self.x.ndim == 2
        self.cfg = cfg
        self.L = lib()
        self.h = self.L.orc_create(_p(self.x), self.x.shape[0], self.x.shape[1], ctypes.byref(cfg))
        if not self.h:
            raise ValueError("orc_create rejected its arguments")
        self.B = cfg.beam
        self.K = self.L.orc_k(self.h)
        self.T = self.x.shape[0]
        self.V = self.x.shape[1]

    def __del__(self):
        if getattr(self, "h", None):
            self.L.orc_destroy(self.h)
            self.h = None

    # ---- stepping -------------------------------------------------------------------
    def score(self, att):
        att = np.ascontiguousarray(att, dtype=np.float32)
        assert att.shape == (self.B, self.V)
        self._att = att
        r = self.L.orc_score(self.h, _p(att))
        if r < 0:
            raise RuntimeError("orc_score failed")

    def rank(self, stopped=None):
        if stopped is None:
            return self.L.orc_rank(self.h, None)
        s = np.ascontiguousarray(stopped, dtype=np.int32)
        return self.L.orc_rank(self.h, _p(s))

    def commit(self, sel_parent=None, sel_token=None, eos_add=None, stopped=None):
        if sel_parent is None:
            r = self.L.orc_commit(self.h, 0, None, None, None, None)
        else:
            sp = np.ascontiguousarray(sel_parent, dtype=np.int32)
            st = np.ascontiguousarray(sel_token, dtype=np.int32)
            ea = np.ascontiguousarray(eos_add, dtype=np.int32)
            so = np.ascontiguousarray(stopped, dtype=np.int32)
            r = self.L.orc_commit(self.h, sp.size, _p(sp), _p(st), _p(ea), _p(so))
        if r < 0:
            raise RuntimeError(f"orc_commit failed ({r})")
        return r

    def override(self, tau=None, tau_end=None, finished=-1):
        t = None if tau is None else np.ascontiguousarray(tau, dtype=np.int32)
        te = None if tau_end is None else np.ascontiguousarray(tau_end, dtype=np.int32)
        self.L.orc_override(self.h, None if t is None else _p(t), None if te is None else _p(te),
                            int(finished))

    def union_contrib(self):
        a, b = ctypes.c_int32(), ctypes.c_int32()
        if not self.L.orc_union_contrib(self.h, ctypes.byref(a), ctypes.byref(b)):
            return None
        return a.value, b.value

    def set_union(self, tau_min, e_max):
        self.L.orc_set_union(self.h, int(tau_min), int(e_max))

    def step_auto(self, att):
        att = np.ascontiguousarray(att, dtype=np.float32)
        r = self.L.orc_step_auto(self.h, _p(att))
        if r < 0:
            raise RuntimeError("orc_step_auto failed")
        return r

    # ---- views ----------------------------------------------------------------------
    @property
    def step(self):
        return self.L.orc_step_index(self.h)

    @property
    def finished(self):
        return bool(self.L.orc_finished(self.h))

    @property
    def lmax(self):
        return self.L.orc_lmax_of(self.h)

    @property
    def cells(self):
        return self.L.orc_cells(self.h)

    @property
    def best(self):
        return self.L.orc_best(self.h)

    @property
    def e1_margin(self):
        return self.L.orc_e1_margin(self.h)

    def sorted_cands(self):
        n = self.L.orc_n_sorted(self.h)
        return _view(self.L.orc_sorted(self.h), CAND_DTYPE, n).copy()

    def _arr(self, name, dtype, n, shape=None):
        a = _view(getattr(self.L, name)(self.h), dtype, n).copy()
        return a if shape is None else a.reshape(shape)

    def windows(self):
        return self._arr("orc_win_s", np.int32, self.B), self._arr("orc_win_e", np.int32, self.B)

    def cand_id(self):
        return self._arr("orc_cand_id", np.int32, self.B * self.K, (self.B, self.K))

    def cand_ctc(self):
        return self._arr("orc_cand_ctc", np.float64, self.B * self.K, (self.B, self.K))

    def cand_att(self):
        return self._arr("orc_cand_att", np.float64, self.B * self.K, (self.B, self.K))

    def cand_joint(self):
        return self._arr("orc_cand_joint", np.float64, self.B * self.K, (self.B, self.K))

    def ctc_eos(self):
        return self._arr("orc_ctc_eos", np.float64, self.B)

    def joint_eos(self):
        return self._arr("orc_joint_eos", np.float64, self.B)

    def e2(self):
        return (self._arr("orc_e2_eligible", np.int32, self.B),
                self._arr("orc_e2_fire", np.int32, self.B),
                self._arr("orc_e2_margin", np.float64, self.B))

    def child_tau_info(self):
        return (self._arr("orc_child_max_n", np.float64, self.B),
                self._arr("orc_child_max_b", np.float64, self.B),
                self._arr("orc_child_lo", np.int32, self.B))

    def hyp(self, j):
        i = [ctypes.c_int32() for _ in range(6)]
        d = [ctypes.c_double() for _ in range(3)]
        self.L.orc_hyp_get(self.h, j, *[ctypes.addressof(v) for v in i],
                           *[ctypes.addressof(v) for v in d])
        live, ln, tau, tau_end, rs, re = [v.value for v in i]
        att, ctc, joint = [v.value for v in d]
        labels = _view(self.L.orc_hyp_labels(self.h, j), np.int32, ln).copy() if ln else \
            np.empty(0, np.int32)
        taus = _view(self.L.orc_hyp_taus(self.h, j), np.int32, ln).copy() if ln else np.empty(0, np.int32)
        return dict(live=live, len=ln, tau=tau, tau_end=tau_end, rs=rs, re=re, att=att, ctc=ctc,
                    joint=joint, labels=labels, taus=taus)

    def hyp_gamma(self, j):
        gn = _view(self.L.orc_hyp_gn(self.h, j), np.float64, self.T + 1).copy()
        gb = _view(self.L.orc_hyp_gb(self.h, j), np.float64, self.T + 1).copy()
        return gn, gb

    def ended(self):
        out = []
        for i in range(self.L.orc_n_ended(self.h)):
            a, b, c = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
            s = ctypes.c_double()
            self.L.orc_ended_get(self.h, i, ctypes.addressof(a), ctypes.addressof(b),
                                 ctypes.addressof(c), ctypes.addressof(s))
            n = a.value - 1
            lab = _view(self.L.orc_ended_labels(self.h, i), np.int32, n).copy() if n > 0 else \
                np.empty(0, np.int32)
            taus = _view(self.L.orc_ended_taus(self.h, i), np.int32, n).copy() if n > 0 else \
                np.empty(0, np.int32)
            out.append(dict(len=a.value, tau=b.value, slot=c.value, score=s.value, labels=lab, taus=taus))
        return out

    def result(self):
        cap = self.lmax + 1
        lab = np.zeros(cap, dtype=np.int32)
        s, fb = ctypes.c_double(), ctypes.c_int32()
        n = self.L.orc_result(self.h, _p(lab), cap, ctypes.byref(s), ctypes.byref(fb))
        if n < 0:
            raise RuntimeError("orc_result: capacity")
        return lab[:n].copy(), s.value, bool(fb.value)

    def result_frames(self):
        """-> (labels, time stamp tau of every label, score, fallback flag)"""
        cap = self.lmax + 1
        lab = np.zeros(cap, dtype=np.int32)
        frm = np.zeros(cap, dtype=np.int32)
        s, fb = ctypes.c_double(), ctypes.c_int32()
        n = self.L.orc_result_frames(self.h, _p(lab), _p(frm), cap, ctypes.byref(s), ctypes.byref(fb))
        if n < 0:
            raise RuntimeError("orc_result_frames: capacity")
        return lab[:n].copy(), frm[:n].copy(), s.value, bool(fb.value)
