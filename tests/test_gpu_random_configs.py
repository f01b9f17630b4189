"""GPU parity on seeded random small configurations: combinations of beam width, vocabulary,
candidate count, window form (per hypothesis, batch-wide, none; one-sided), end rules, batch shape
(ragged, unused slots) that the hand-written tests do not spell out, each decoded step by step against
the oracle.  All cases run in ONE process, handle after handle, as a long-running service would: device
memory that a new handle gets is whatever earlier handles left there (a kernel that lets a never-written
value steer an access shows up here and nowhere in a fresh process; tests/cpu_emu hunts the same on the
CPU with poisoned memory).  The cases come from the one table in tests/random_cases.py, a subset of which
the CPU suite decodes on the CPU build of the kernels under AddressSanitizer."""
import numpy as np
import pytest

import gen
from helpers import lockstep_decode
from random_cases import RUNS, case_params, describe

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed0,n_cases", RUNS)
def test_random_small_configurations_one_process(seed0, n_cases):
    bad = []
    for case in range(n_cases):
        mode, w, lens = case_params(case, seed0)
        used = [u for u in range(len(lens)) if lens[u] > 0]
        if not used:
            continue
        print(describe(seed0, case, mode, w, lens), flush=True)
        ctc = gen.workload_ctc(w, np.maximum(lens, 1))
        rep, res = lockstep_decode(w, ctc, lens, check_utts=used)
        ok = (rep["max_score_err"] < 1e-4 and rep["max_ctc_err"] < 1e-4
              and res["cells"] == int(res["oracle_cells"]))
        if not ok:
            bad.append((case, mode, rep))
    assert not bad, bad
