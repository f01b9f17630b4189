"""Seeded synthetic inputs for the batched CTC/attention beam-search step.

Input recipes only (counter-based RNG, normals, log_softmax); none of the
decoding method's arithmetic lives here.  The host generator is plain C built
into ``gen/libgen_host.so``; the optional device twin (``gen/libgen_dev.so``)
produces inputs of the same recipe directly in GPU memory for throughput runs.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_HOST_SO = os.path.join(_HERE, "libgen_host.so")
_DEV_SO = os.path.join(_HERE, "libgen_dev.so")
_host = None
_dev = None

HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-shared",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(device=True):
    """Compile the host generator (gcc) and, if asked, the device twin (hipcc)."""
    subprocess.check_call(["gcc", "-O2", "-fPIC", "-shared", "-fopenmp", "-o", _HOST_SO,
                           os.path.join(_HERE, "gen_host.c"), "-lm"])
    if device:
        subprocess.check_call(["hipcc", *HIP_FLAGS, "-o", _DEV_SO,
                               os.path.join(_HERE, "gen_device.hip")])


def _lib():
    global _host
    if _host is None:
        if not os.path.exists(_HOST_SO):
            build(device=False)
        L = ctypes.CDLL(_HOST_SO)
        u64, u32, i32, dbl = ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int32, ctypes.c_double
        vp = ctypes.c_void_p
        L.gen_fnv1a64.restype = u64
        L.gen_fnv1a64.argtypes = [vp, ctypes.c_size_t, u64]
        L.gen_fnv_basis.restype = u64
        L.gen_prefix_hash.restype = u64
        L.gen_prefix_hash.argtypes = [vp, i32]
        L.gen_prefix_hash_extend.restype = u64
        L.gen_prefix_hash_extend.argtypes = [u64, i32]
        L.gen_stream_key.restype = u64
        L.gen_stream_key.argtypes = [u64, u32, u32, u32, u64]
        L.gen_philox4x32_10.argtypes = [vp, vp, vp]
        L.gen_normals.argtypes = [u64, ctypes.c_size_t, vp]
        L.gen_uniforms.argtypes = [u64, ctypes.c_size_t, vp]
        L.gen_lengths.argtypes = [u64, i32, i32, i32, vp]
        L.gen_ctc_utt.argtypes = [u64, u32, i32, i32, i32, dbl, dbl, dbl, vp]
        L.gen_att_row.argtypes = [u64, u32, u32, u64, i32, dbl, vp]
        L.gen_att_rows.argtypes = [u64, vp, u32, vp, i32, i32, dbl, vp]
        L.gen_ctc_batch.argtypes = [u64, i32, vp, i32, i32, i32, dbl, dbl, dbl, ctypes.c_float, vp]
        _host = L
    return _host


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def fnv1a64(data: bytes, h=None) -> int:
    L = _lib()
    if h is None:
        h = L.gen_fnv_basis()
    buf = ctypes.create_string_buffer(data, len(data))
    return int(L.gen_fnv1a64(ctypes.cast(buf, ctypes.c_void_p), len(data), h))


def prefix_hash(labels) -> int:
    a = np.ascontiguousarray(labels, dtype=np.int32)
    return int(_lib().gen_prefix_hash(_p(a), a.size))


def prefix_hash_extend(h: int, label: int) -> int:
    return int(_lib().gen_prefix_hash_extend(h, int(label)))


def philox4x32_10(ctr, key):
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = np.ascontiguousarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    _lib().gen_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def stream_key(seed, tag, a=0, b=0, c=0) -> int:
    return int(_lib().gen_stream_key(seed, tag, a, b, c))


def normals(key: int, n: int):
    out = np.empty(n, dtype=np.float64)
    _lib().gen_normals(key, n, _p(out))
    return out


def uniforms(key: int, n: int):
    out = np.empty(n, dtype=np.float64)
    _lib().gen_uniforms(key, n, _p(out))
    return out


def lengths(seed: int, n_utt: int, lo: int, hi: int):
    out = np.empty(n_utt, dtype=np.int32)
    _lib().gen_lengths(seed, n_utt, lo, hi, _p(out))
    return out


def ctc_utt(seed, utt, T, V, blank_id=0, blank_boost=4.0, p_boost=0.7, zipf_s=0.0):
    """[T, V] fp32 CTC log-posteriors of one utterance (row t = frame t+1)."""
    out = np.empty((T, V), dtype=np.float32)
    _lib().gen_ctc_utt(seed, utt, T, V, blank_id, blank_boost, p_boost, zipf_s, _p(out))
    return out


def ctc_batch(seed, lens, V, t_max=None, blank_id=0, blank_boost=4.0, p_boost=0.7, zipf_s=0.0,
              pad_value=float("nan")):
    """[U, t_max, V] fp32; rows at and beyond an utterance's length hold pad_value."""
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    if t_max is None:
        t_max = int(lens.max())
    out = np.empty((lens.size, t_max, V), dtype=np.float32)
    _lib().gen_ctc_batch(seed, lens.size, _p(lens), t_max, V, blank_id, blank_boost, p_boost,
                         zipf_s, pad_value, _p(out))
    return out


def att_row(seed, utt, step, phash, V, scale=2.0):
    out = np.empty(V, dtype=np.float32)
    _lib().gen_att_row(seed, utt, step, phash, V, scale, _p(out))
    return out


def att_rows(seed, utts, step, phashes, V, scale=2.0):
    """One attention log-prob row per (utt, prefix hash) pair -> [n, V] fp32."""
    u = np.ascontiguousarray(utts, dtype=np.uint32)
    h = np.ascontiguousarray(phashes, dtype=np.uint64)
    out = np.empty((u.size, V), dtype=np.float32)
    _lib().gen_att_rows(seed, _p(u), step, _p(h), u.size, V, scale, _p(out))
    return out


# ----------------------------------------------------------------------------
# Named workloads (shapes and search parameters of the benchmark configurations)
# ----------------------------------------------------------------------------
END_BASELINE, END_TAU_COUNT, END_EOS_RUN = 1, 2, 4


def workload(name: str, seed: int = 2101):
    """Shapes, input recipe and search parameters of a named configuration."""
    base = dict(seed=seed, blank_id=0, ctc_weight=0.3, blank_boost=4.0, p_boost=0.7,
                att_scale=2.0, end_m=3, end_d=-10.0, end_c=2, eos_run=10)
    if name == "cfg0":
        w = dict(n_utt=1, t_lo=100, t_hi=100, vocab=32, beam=4, cand_k=0, win_m1=-1, win_m2=-1,
                 length_bonus=0.0, max_len_ratio=0.0, max_len_abs=20, zipf_s=0.0,
                 end_flags=END_BASELINE | END_TAU_COUNT)
    elif name == "cfg1":
        w = dict(n_utt=16, t_lo=200, t_hi=500, vocab=5000, beam=10, cand_k=40, win_m1=-1,
                 win_m2=-1, length_bonus=0.5, max_len_ratio=0.3, max_len_abs=0, zipf_s=1.1,
                 end_flags=END_BASELINE | END_TAU_COUNT)
    elif name == "cfg2":
        w = dict(n_utt=64, t_lo=250, t_hi=875, vocab=5000, beam=10, cand_k=40, win_m1=50,
                 win_m2=50, length_bonus=0.5, max_len_ratio=0.3, max_len_abs=0, zipf_s=1.1,
                 end_flags=END_BASELINE | END_TAU_COUNT | END_EOS_RUN)
    elif name == "cfg3":  # one batch of Korean-meeting-like segments (lengths come from segments())
        w = dict(n_utt=128, t_lo=375, t_hi=500, vocab=2300, beam=10, cand_k=40, win_m1=50,
                 win_m2=50, length_bonus=0.5, max_len_ratio=0.3, max_len_abs=0, zipf_s=1.1,
                 end_flags=END_BASELINE | END_TAU_COUNT | END_EOS_RUN)
    elif name == "cfg4a":
        w = dict(n_utt=256, t_lo=1500, t_hi=1500, vocab=5000, beam=20, cand_k=0, win_m1=-1,
                 win_m2=-1, length_bonus=0.5, max_len_ratio=0.3, max_len_abs=0, zipf_s=1.1,
                 end_flags=END_BASELINE | END_TAU_COUNT)
    elif name == "cfg4b":
        w = dict(n_utt=256, t_lo=1500, t_hi=1500, vocab=5000, beam=20, cand_k=60, win_m1=80,
                 win_m2=80, length_bonus=0.5, max_len_ratio=0.3, max_len_abs=0, zipf_s=1.1,
                 end_flags=END_BASELINE | END_TAU_COUNT | END_EOS_RUN)
    else:
        raise KeyError(name)
    base.update(w)
    base["name"] = name
    base["eos_id"] = base["vocab"] - 1
    return base


def workload_lengths(w):
    return lengths(w["seed"], w["n_utt"], w["t_lo"], w["t_hi"])


def workload_ctc(w, lens=None, pad_value=float("nan")):
    if lens is None:
        lens = workload_lengths(w)
    return ctc_batch(w["seed"], lens, w["vocab"], blank_id=w["blank_id"],
                     blank_boost=w["blank_boost"], p_boost=w["p_boost"], zipf_s=w["zipf_s"],
                     pad_value=pad_value)


def segments(seed, n_rec=32, min_minutes=30.0, max_minutes=60.0, fps=100, cut_lo_s=15.0,
             cut_hi_s=20.0, subsample=4):
    """Korean-meeting-like segment lengths (in subsampled frames), sorted ascending.

    Each synthetic recording lasts U[min,max] minutes.  A log-energy track alternates
    speech and pause stretches (renewal process: speech ~ 0.5-6 s, pause ~ 0.1-1.2 s,
    pause energy well below speech energy, both jittered); the recording is cut at the
    lowest-energy frame between cut_lo_s and cut_hi_s after the previous cut.
    """
    out = []
    for r in range(n_rec):
        key = stream_key(seed, 5, r, 0, 0)
        u = uniforms(key, 4)
        n_frames = int((min_minutes + (max_minutes - min_minutes) * u[0]) * 60 * fps)
        # renewal process of (speech, pause) stretches
        n_st = n_frames // 40 + 8
        us = uniforms(stream_key(seed, 5, r, 1, 0), 2 * n_st)
        energy = np.empty(n_frames, dtype=np.float64)
        pos, i = 0, 0
        while pos < n_frames:
            sp = int((0.5 + 5.5 * us[2 * i % us.size]) * fps)
            pa = int((0.1 + 1.1 * us[(2 * i + 1) % us.size]) * fps)
            energy[pos:pos + sp] = 0.0
            energy[pos + sp:pos + sp + pa] = -6.0
            pos += sp + pa
            i += 1
        energy += 0.5 * normals(stream_key(seed, 5, r, 2, 0), n_frames)
        start = 0
        lo, hi = int(cut_lo_s * fps), int(cut_hi_s * fps)
        while n_frames - start > hi:
            seg = energy[start + lo:start + hi]
            cut = start + lo + int(np.argmin(seg))
            out.append(-(-(cut - start) // subsample))
            start = cut
        if n_frames - start > 0:
            out.append(-(-(n_frames - start) // subsample))
    return np.sort(np.asarray(out, dtype=np.int32))


# ----------------------------------------------------------------------------
# Device twin (same recipe, written straight into GPU memory)
# ----------------------------------------------------------------------------
def dev():
    """ctypes handle of the device generator; raises if it has not been built."""
    global _dev
    if _dev is None:
        if not os.path.exists(_DEV_SO):
            raise RuntimeError("gen/libgen_dev.so missing: run __graft_entry__.build() first")
        L = ctypes.CDLL(_DEV_SO)
        u64, u32, i32, dbl, vp = (ctypes.c_uint64, ctypes.c_uint32, ctypes.c_int32,
                                  ctypes.c_double, ctypes.c_void_p)
        L.gen_dev_ctc.restype = i32
        L.gen_dev_ctc.argtypes = [u64, i32, vp, i32, i32, i32, dbl, dbl, dbl, vp, vp]
        L.gen_dev_att_step.restype = i32
        L.gen_dev_att_step.argtypes = [u64, u32, i32, i32, i32, dbl, vp, vp, vp, vp, vp, vp, vp]
        _dev = L
    return _dev
