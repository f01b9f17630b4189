"""Child process of tests/test_cpu_emulation.py: decodes small batches with the CPU build of the
kernels (argv[1] = its shared library), every step compared with the oracle exactly as the GPU
tests do.  Prints "emu ok <name>" per case; any sanitizer report or mismatch ends it with a non-zero
status."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

import numpy as np  # noqa: E402

import paper_2101_05600_amd as m  # noqa: E402

m._SO = sys.argv[1]          # the binding loads this instead of the GPU library (tests only)

import gen  # noqa: E402
from helpers import EmuDecoder, lockstep_decode  # noqa: E402

CASES = {
    # split select kernel, 16-lane score kernel, eos-run rule, an unused slot
    "windowed": (dict(n_utt=3, vocab=40, beam=3, cand_k=6, win_m1=5, win_m2=5, end_flags=7, eos_run=2,
                      max_len_ratio=0.4), [17, 0, 26]),
    # per-utterance select kernel (batch-wide window), 64-lane score kernel (no end margin)
    "batch_window": (dict(n_utt=2, vocab=36, beam=2, cand_k=5, win_m1=4, win_m2=-1, win_union=1, end_flags=3,
                          max_len_ratio=0.4), [21, 14]),
    # every id a candidate: all-candidates score kernel, list builder from registers
    "all_candidates": (dict(n_utt=1, vocab=12, beam=2, cand_k=0, win_m1=-1, win_m2=-1, end_flags=3,
                            max_len_ratio=0.4), [15]),
    # fewer ids than beam slots: most slots never hold a hypothesis, their records are never written
    "all_candidates_few_ids": (dict(n_utt=2, vocab=6, beam=6, cand_k=0, win_m1=-1, win_m2=-1, end_flags=3,
                                    max_len_ratio=0.4), [13, 9]),
    # logits in, odd vocabulary (radix selection), one candidate per hypothesis
    "logits_odd_vocab": (dict(n_utt=1, vocab=33, beam=2, cand_k=1, win_m1=3, win_m2=8, end_flags=2, att_is_logits=1,
                              max_len_ratio=0.4), [19]),
}


def main():
    names = sys.argv[2:] or list(CASES)
    for name in names:
        over, lens = CASES[name]
        w = gen.workload("cfg1")
        w.update(over)
        w["eos_id"] = w["vocab"] - 1
        lens = np.asarray(lens, np.int32)
        ctc = gen.workload_ctc(w, np.maximum(lens, 1))
        used = [u for u in range(len(lens)) if lens[u] > 0]
        kw = {}
        if w.get("att_is_logits"):
            # the library takes unnormalised scores; the oracle takes their log_softmax
            def to_logits(a):
                return (a * 1.7 + 0.3).astype(np.float32)

            def normalised(a):
                z = to_logits(a).astype(np.float64)
                mx = np.nanmax(z, axis=-1, keepdims=True)
                return (z - (mx + np.log(np.nansum(np.exp(z - mx), axis=-1, keepdims=True)))).astype(np.float32)
            kw = dict(att_fn=normalised, gpu_att_fn=to_logits)
        rep, res = lockstep_decode(w, ctc, lens, check_utts=used, decoder_cls=EmuDecoder, **kw)
        tol = 2e-4 if w.get("att_is_logits") else 1e-4
        assert rep["max_score_err"] < tol and rep["max_ctc_err"] < tol, (name, rep)
        assert res["cells"] == int(res["oracle_cells"]), (name, res["cells"], res["oracle_cells"])
        print(f"emu ok {name} steps={rep['utt_steps']} score_err={rep['max_score_err']:.2e}", flush=True)


if __name__ == "__main__":
    main()
