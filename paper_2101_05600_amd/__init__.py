"""Python binding of libctcbs (batched joint CTC/attention beam-search step, MI355X).

Argument marshalling only: every step of the decoding path runs in the HIP kernels behind
the C ABI declared in ``include/ctcbs.h``.  The functions carry the C names.  Device
buffers are passed as torch tensors (their ``data_ptr()`` is handed over) or raw integer
addresses.  There is no CPU fallback: if the library is missing, loading raises.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_SO = os.path.join(_HERE, "libctcbs.so")
_lib = None

OK, DONE, EINVAL, ENOMEM, EHIP, ESTATE, ECAP = 0, 1, -1, -2, -3, -4, -5
END_BASELINE, END_TAU_COUNT, END_EOS_RUN = 1, 2, 4
PEEK_CAND_ID, PEEK_CAND_CTC, PEEK_CAND_JOINT, PEEK_WIN_S, PEEK_WIN_E = 1, 2, 3, 4, 5
PEEK_CTC_EOS, PEEK_JOINT_EOS, PEEK_N_CAND = 6, 7, 8

# (kernarg preload: the leading plain arguments of a kernel -- up to 16 dwords -- are handed to its waves in
# registers when they start; the score and the split select kernel keep what their first loads need there)
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-mllvm", "-amdgpu-kernarg-preload-count=16"]

EXPORTS = ["ctcbs_create", "ctcbs_step", "ctcbs_step_static", "ctcbs_poll", "ctcbs_finalize", "ctcbs_stats", "ctcbs_peek",
           "ctcbs_destroy", "ctcbs_strerror", "ctcbs_last_hip_error", "ctcbs_profile",
           "ctcbs_profile_read", "ctcbs_reset", "ctcbs_hard_segments", "ctcbs_merge_pieces",
           "ctcbs_plan_batches", "ctcbs_run_many", "ctcbs_att_replay", "ctcbs_run_queue"]


_PROBE_SO = os.path.join(_HERE, "libctcbs_probe.so")
_probe = None


def build():
    """Compile the HIP library for gfx950 (cross-compiles without a GPU), and the measurement
    kernels of the latency floor (their own small library: not part of the decoding path)."""
    src = os.path.join(_HERE, "csrc", "ctcbs.hip")
    subprocess.check_call(["hipcc", *HIP_FLAGS, "-o", _SO, src])
    subprocess.check_call(["hipcc", *HIP_FLAGS, "-o", _PROBE_SO, os.path.join(_HERE, "csrc", "probe.hip")])


def probe_lib():
    """The measurement kernels of csrc/probe.hip (bench.py --floor)."""
    global _probe
    if _probe is None:
        if not os.path.exists(_PROBE_SO):
            raise RuntimeError(f"{_PROBE_SO} is missing: run __graft_entry__.build() first")
        L = ctypes.CDLL(_PROBE_SO)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.probe_chain.restype = i32
        L.probe_chain.argtypes = [i32, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, vp]
        L.probe_empty.restype = i32
        L.probe_empty.argtypes = [i32, i32, i32, i32, vp]
        L.probe_touch.restype = i32
        L.probe_touch.argtypes = [vp, vp, i32, vp]
        _probe = L
    return _probe


class Config(ctypes.Structure):
    _fields_ = [("n_utt", ctypes.c_int32), ("t_max", ctypes.c_int32), ("vocab", ctypes.c_int32),
                ("beam", ctypes.c_int32), ("blank_id", ctypes.c_int32), ("eos_id", ctypes.c_int32),
                ("cand_k", ctypes.c_int32), ("win_m1", ctypes.c_int32), ("win_m2", ctypes.c_int32),
                ("ctc_weight", ctypes.c_float), ("length_bonus", ctypes.c_float),
                ("max_len_ratio", ctypes.c_float), ("max_len_abs", ctypes.c_int32),
                ("end_flags", ctypes.c_int32), ("end_m", ctypes.c_int32), ("end_d", ctypes.c_float),
                ("end_c", ctypes.c_int32), ("eos_run", ctypes.c_int32), ("poll_every", ctypes.c_int32),
                ("win_union", ctypes.c_int32), ("att_is_logits", ctypes.c_int32),
                ("keep_candidates", ctypes.c_int32), ("stream", ctypes.c_void_p)]


class StepOut(ctypes.Structure):
    _fields_ = [("step", ctypes.c_int32), ("n_finished", ctypes.c_int32),
                ("d_parent", ctypes.c_void_p), ("d_token", ctypes.c_void_p),
                ("d_score", ctypes.c_void_p), ("d_live", ctypes.c_void_p),
                ("d_finished", ctypes.c_void_p), ("d_tau", ctypes.c_void_p),
                ("d_tau_end", ctypes.c_void_p), ("d_eos_added", ctypes.c_void_p),
                ("d_stopped", ctypes.c_void_p)]


def lib():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            raise RuntimeError(f"{_SO} is missing: run __graft_entry__.build() first "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(_SO)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.ctcbs_create.restype = i32
        L.ctcbs_create.argtypes = [ctypes.POINTER(Config), vp, vp, ctypes.POINTER(vp)]
        L.ctcbs_reset.restype = i32
        L.ctcbs_reset.argtypes = [vp, vp, vp]
        L.ctcbs_step.restype = i32
        L.ctcbs_step.argtypes = [vp, vp, ctypes.POINTER(StepOut)]
        L.ctcbs_step_static.restype = i32
        L.ctcbs_step_static.argtypes = [vp, vp, ctypes.POINTER(StepOut)]
        L.ctcbs_poll.restype = i32
        L.ctcbs_poll.argtypes = [vp, ctypes.POINTER(i32)]
        L.ctcbs_finalize.restype = i32
        L.ctcbs_finalize.argtypes = [vp, vp, i32, vp, vp, vp, vp]
        L.ctcbs_stats.restype = i32
        L.ctcbs_stats.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64),
                                  ctypes.POINTER(i32)]
        L.ctcbs_profile.restype = i32
        L.ctcbs_profile.argtypes = [vp, i32]
        L.ctcbs_profile_read.restype = i32
        L.ctcbs_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double),
                                         ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
        L.ctcbs_peek.restype = i32
        L.ctcbs_peek.argtypes = [vp, i32, vp, ctypes.c_size_t, ctypes.POINTER(ctypes.c_size_t)]
        L.ctcbs_destroy.restype = None
        L.ctcbs_destroy.argtypes = [vp]
        L.ctcbs_strerror.restype = ctypes.c_char_p
        L.ctcbs_strerror.argtypes = [i32]
        L.ctcbs_last_hip_error.restype = i32
        i64 = ctypes.c_int64
        L.ctcbs_hard_segments.restype = i32
        L.ctcbs_hard_segments.argtypes = [i64, i32, i32, vp, i32, ctypes.POINTER(i32)]
        L.ctcbs_merge_pieces.restype = i32
        L.ctcbs_merge_pieces.argtypes = [vp, i32, i32, i32, vp, i32, ctypes.POINTER(i32)]
        L.ctcbs_plan_batches.restype = i32
        L.ctcbs_plan_batches.argtypes = [vp, i32, i32, i64, vp, vp, i32, ctypes.POINTER(i32)]
        L.ctcbs_run_many.restype = i32
        L.ctcbs_run_many.argtypes = [vp, i32, vp, vp, i32]
        L.ctcbs_run_queue.restype = i32
        L.ctcbs_run_queue.argtypes = [vp, i32, i32, vp, vp, vp, i32]
        L.ctcbs_att_replay.restype = i32
        L.ctcbs_att_replay.argtypes = [vp, i32, i32, vp, vp]
        _lib = L
    return _lib


class CtcbsError(RuntimeError):
    def __init__(self, code):
        self.code = code
        msg = lib().ctcbs_strerror(code).decode()
        if code == EHIP:
            msg += f" (hip error {lib().ctcbs_last_hip_error()})"
        super().__init__(f"ctcbs: {msg} [{code}]")


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def make_config(n_utt, t_max, vocab, beam, blank_id=0, eos_id=None, cand_k=0, win_m1=-1, win_m2=-1,
                ctc_weight=0.3, length_bonus=0.0, max_len_ratio=0.0, max_len_abs=0, end_flags=3,
                end_m=3, end_d=-10.0, end_c=2, eos_run=10, poll_every=0, stream=None, att_is_logits=0,
                win_union=0, keep_candidates=1, **_ignored):
    c = Config()
    c.n_utt, c.t_max, c.vocab, c.beam, c.blank_id = n_utt, t_max, vocab, beam, blank_id
    c.eos_id = vocab - 1 if eos_id is None else eos_id
    c.cand_k, c.win_m1, c.win_m2 = cand_k, win_m1, win_m2
    c.ctc_weight, c.length_bonus = ctc_weight, length_bonus
    c.max_len_ratio, c.max_len_abs = max_len_ratio, max_len_abs
    c.end_flags, c.end_m, c.end_d, c.end_c, c.eos_run = end_flags, end_m, end_d, end_c, eos_run
    c.poll_every = poll_every
    c.att_is_logits = att_is_logits
    c.win_union = win_union
    c.keep_candidates = keep_candidates
    c.stream = stream
    return c


def ctcbs_create(cfg: Config, d_ctc_logp, h_lens):
    """-> opaque handle (int).  d_ctc_logp: device fp32 [U][t_max][V]; h_lens: host int32 [U]."""
    lens = np.ascontiguousarray(h_lens, dtype=np.int32)
    out = ctypes.c_void_p()
    rc = lib().ctcbs_create(ctypes.byref(cfg), _ptr(d_ctc_logp), lens.ctypes.data_as(ctypes.c_void_p),
                            ctypes.byref(out))
    if rc != OK:
        raise CtcbsError(rc)
    return out.value


def ctcbs_reset(handle, d_ctc_logp, h_lens):
    """Start the next batch on an existing handle (same configuration, lengths <= t_max)."""
    lens = np.ascontiguousarray(h_lens, dtype=np.int32)
    rc = lib().ctcbs_reset(handle, _ptr(d_ctc_logp), lens.ctypes.data_as(ctypes.c_void_p))
    if rc != OK:
        raise CtcbsError(rc)


def ctcbs_step(handle, d_att_logp, out: StepOut = None):
    """-> OK or DONE.  d_att_logp: device fp32 [U][Wb][V]."""
    rc = lib().ctcbs_step(handle, _ptr(d_att_logp), ctypes.byref(out) if out is not None else None)
    if rc < 0:
        raise CtcbsError(rc)
    return rc


def ctcbs_step_static(handle, d_att_logp, out: StepOut = None):
    """ctcbs_step with its per-step scratch in the library's fixed array (allocates nothing)."""
    rc = lib().ctcbs_step_static(handle, _ptr(d_att_logp), ctypes.byref(out) if out is not None else None)
    if rc < 0:
        raise CtcbsError(rc)
    return rc


def ctcbs_poll(handle):
    n = ctypes.c_int32()
    rc = lib().ctcbs_poll(handle, ctypes.byref(n))
    if rc != OK:
        raise CtcbsError(rc)
    return n.value


def ctcbs_finalize(handle, n_utt, cap, want_frames=False):
    """-> (tokens [U][cap] int32, ntok [U], score [U] fp32, frames or None, flags [U])."""
    tok = np.full((n_utt, max(cap, 1)), -1, dtype=np.int32)
    frm = np.full((n_utt, max(cap, 1)), -1, dtype=np.int32) if want_frames else None
    nt = np.zeros(n_utt, dtype=np.int32)
    sc = np.zeros(n_utt, dtype=np.float32)
    fl = np.zeros(n_utt, dtype=np.int32)
    vp = ctypes.c_void_p
    rc = lib().ctcbs_finalize(handle, tok.ctypes.data_as(vp), cap, nt.ctypes.data_as(vp),
                              sc.ctypes.data_as(vp), frm.ctypes.data_as(vp) if want_frames else None,
                              fl.ctypes.data_as(vp))
    if rc != OK:
        raise CtcbsError(rc)
    return tok, nt, sc, frm, fl


def ctcbs_stats(handle):
    """-> (cells, groups, steps)"""
    c, g, s = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_int32()
    rc = lib().ctcbs_stats(handle, ctypes.byref(c), ctypes.byref(g), ctypes.byref(s))
    if rc != OK:
        raise CtcbsError(rc)
    return c.value, g.value, s.value


def ctcbs_profile(handle, enable=True):
    rc = lib().ctcbs_profile(handle, 1 if enable else 0)
    if rc != OK:
        raise CtcbsError(rc)


def ctcbs_profile_read(handle):
    """-> (score_ms, select_ms, n_steps)"""
    a, b, n = ctypes.c_double(), ctypes.c_double(), ctypes.c_int32()
    rc = lib().ctcbs_profile_read(handle, ctypes.byref(a), ctypes.byref(b), ctypes.byref(n))
    if rc != OK:
        raise CtcbsError(rc)
    return a.value, b.value, n.value


_PEEK_DTYPE = {PEEK_CAND_ID: np.int32, PEEK_CAND_CTC: np.float64, PEEK_CAND_JOINT: np.float64,
               PEEK_WIN_S: np.int32, PEEK_WIN_E: np.int32, PEEK_CTC_EOS: np.float64,
               PEEK_JOINT_EOS: np.float64, PEEK_N_CAND: np.int32}


def ctcbs_peek(handle, what):
    need = ctypes.c_size_t()
    rc = lib().ctcbs_peek(handle, what, None, 0, ctypes.byref(need))
    if rc != OK:
        raise CtcbsError(rc)
    dt = np.dtype(_PEEK_DTYPE[what])
    out = np.empty(need.value // dt.itemsize, dtype=dt)
    rc = lib().ctcbs_peek(handle, what, out.ctypes.data_as(ctypes.c_void_p), need.value, None)
    if rc != OK:
        raise CtcbsError(rc)
    return out


def _lengths_call(fn, *args):
    """Two calls: the first sizes the output, the second fills it."""
    n = ctypes.c_int32()
    rc = fn(*args, None, 0, ctypes.byref(n))
    if rc not in (OK, ECAP):
        raise CtcbsError(rc)
    out = np.empty(max(n.value, 1), dtype=np.int32)
    if n.value:
        rc = fn(*args, out.ctypes.data_as(ctypes.c_void_p), n.value, ctypes.byref(n))
        if rc != OK:
            raise CtcbsError(rc)
    return out[:n.value].copy()


def ctcbs_hard_segments(n_frames, min_len, max_len):
    """-> int32 lengths of the hard segmentation of a recording of n_frames frames."""
    return _lengths_call(lib().ctcbs_hard_segments, int(n_frames), int(min_len), int(max_len))


def ctcbs_merge_pieces(piece_len, min_len, max_len):
    """-> int32 segment lengths from voice-activity piece lengths."""
    pl = np.ascontiguousarray(piece_len, dtype=np.int32)
    return _lengths_call(lib().ctcbs_merge_pieces, pl.ctypes.data_as(ctypes.c_void_p), pl.size, int(min_len),
                         int(max_len))


def ctcbs_plan_batches(lens, max_utt, max_padded_frames=0):
    """-> (order, begin): batch b holds segments order[begin[b]:begin[b+1]], longest first."""
    ln = np.ascontiguousarray(lens, dtype=np.int32)
    order = np.empty(max(ln.size, 1), dtype=np.int32)
    nb = ctypes.c_int32()
    vp = ctypes.c_void_p
    rc = lib().ctcbs_plan_batches(ln.ctypes.data_as(vp), ln.size, int(max_utt), int(max_padded_frames),
                                  order.ctypes.data_as(vp), None, 0, ctypes.byref(nb))
    if rc not in (OK, ECAP):
        raise CtcbsError(rc)
    begin = np.empty(nb.value + 1, dtype=np.int32)
    rc = lib().ctcbs_plan_batches(ln.ctypes.data_as(vp), ln.size, int(max_utt), int(max_padded_frames),
                                  order.ctypes.data_as(vp), begin.ctypes.data_as(vp), nb.value, ctypes.byref(nb))
    if rc != OK:
        raise CtcbsError(rc)
    return order[:ln.size].copy(), begin


class Replay(ctypes.Structure):
    """Mirror of ctcbs_replay_t."""
    _fields_ = [("d_att", ctypes.POINTER(ctypes.c_void_p)), ("n_steps", ctypes.c_int32)]


ATT_FN = ctypes.CFUNCTYPE(ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                          ctypes.POINTER(StepOut), ctypes.POINTER(ctypes.c_void_p))


def ctcbs_run_many(handles, att_fn=None, replay=None, n_threads=1):
    """Decode the batches of `handles` at once.  Either `replay`: per handle a list of device
    pointers (ints), one [U][Wb][V] row block per step, served by the library's own
    ctcbs_att_replay; or `att_fn(index, step, prev_out_or_None) -> device pointer` (a Python
    callable; use one thread with it)."""
    L = lib()
    hs = (ctypes.c_void_p * len(handles))(*handles)
    if replay is not None:
        keep = [(ctypes.c_void_p * len(r))(*r) for r in replay]
        tabs = (Replay * len(handles))()
        for i, k in enumerate(keep):
            tabs[i].d_att = ctypes.cast(k, ctypes.POINTER(ctypes.c_void_p))
            tabs[i].n_steps = len(replay[i])
        fn = ctypes.cast(L.ctcbs_att_replay, ctypes.c_void_p)
        rc = L.ctcbs_run_many(hs, len(handles), fn, ctypes.cast(tabs, ctypes.c_void_p), int(n_threads))
    else:
        def tramp(_user, index, step, prev, d_att):
            try:
                d_att[0] = _ptr(att_fn(index, step, prev.contents if prev else None))
                return OK
            except Exception:                       # never let an exception cross the C frames
                return EINVAL
        cb = ATT_FN(tramp)
        rc = L.ctcbs_run_many(hs, len(handles), ctypes.cast(cb, ctypes.c_void_p), None, int(n_threads))
    if rc != OK:
        raise CtcbsError(rc)


JOB_LOAD, JOB_DONE = 0, 1
JOB_FN = ctypes.CFUNCTYPE(ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p,
                          ctypes.c_int32)


def ctcbs_run_queue(handles, n_jobs, job_fn, replay=None, att_fn=None, n_threads=1):
    """Decode n_jobs batches on the given handles (as many in flight).  job_fn(job, slot, handle,
    phase): phase JOB_LOAD -> ctcbs_reset(handle, ...) for that batch, JOB_DONE -> ctcbs_finalize.
    Attention rows: `replay` (per job a list of device pointers, one per step) or a Python
    `att_fn(job, step, prev)` (then use one thread).  Callbacks run on the executor's threads."""
    L = lib()
    hs = (ctypes.c_void_p * len(handles))(*handles)
    errors = []

    def job_tramp(_user, job, slot, h, phase):
        try:
            job_fn(job, slot, h, phase)
            return OK
        except Exception as e:                      # never let an exception cross the C frames
            errors.append(e)
            return EINVAL
    jcb = JOB_FN(job_tramp)
    if replay is not None:
        keep = [(ctypes.c_void_p * len(r))(*r) for r in replay]
        tabs = (Replay * n_jobs)()
        for i, k in enumerate(keep):
            tabs[i].d_att = ctypes.cast(k, ctypes.POINTER(ctypes.c_void_p))
            tabs[i].n_steps = len(replay[i])
        rc = L.ctcbs_run_queue(hs, len(handles), n_jobs, ctypes.cast(jcb, ctypes.c_void_p),
                               ctypes.cast(L.ctcbs_att_replay, ctypes.c_void_p),
                               ctypes.cast(tabs, ctypes.c_void_p), int(n_threads))
    else:
        def tramp(_user, index, step, prev, d_att):
            try:
                d_att[0] = _ptr(att_fn(index, step, prev.contents if prev else None))
                return OK
            except Exception as e:
                errors.append(e)
                return EINVAL
        cb = ATT_FN(tramp)
        rc = L.ctcbs_run_queue(hs, len(handles), n_jobs, ctypes.cast(jcb, ctypes.c_void_p),
                               ctypes.cast(cb, ctypes.c_void_p), None, int(n_threads))
    if errors:
        raise errors[0]
    if rc != OK:
        raise CtcbsError(rc)


def ctcbs_destroy(handle):
    if handle:
        lib().ctcbs_destroy(handle)


def ctcbs_strerror(code):
    return lib().ctcbs_strerror(code).decode()


def view(ptr, shape, dtype):
    """A torch tensor aliasing a library-owned device array (step outputs)."""
    import torch
    n = int(np.prod(shape))
    tdt = {np.int32: torch.int32, np.float32: torch.float32, np.uint8: torch.uint8}[dtype]
    nbytes = n * np.dtype(dtype).itemsize

    class _Holder:
        pass

    hold = _Holder()
    hold.__cuda_array_interface__ = {
        "shape": (nbytes,), "typestr": "|u1", "data": (int(ptr), False), "version": 2}
    return torch.as_tensor(hold, device="cuda").view(tdt).reshape(shape)
