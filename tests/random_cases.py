"""The seeded random small configurations of the parity tests: ONE table for the GPU run
(tests/test_gpu_random_configs.py walks every case of RUNS) and for the CPU run of the kernel sources
under AddressSanitizer with garbage-filled device memory (tests/test_cpu_emulation.py walks CPU_SUBSET;
any other case: `python tests/cpu_emu/run_case.py <libctcbs_emu.so> random:<seed>:<case>`).
A case that is to go to the GPU for the first time goes through the CPU build first."""
import random

import gen

RUNS = [(1, 60), (2, 40), (3, 30)]          # (seed of the list, number of cases)

# The subset decoded on the CPU build in the ordinary CPU suite (the emulation runs one OS thread per
# work-item, so only the first steps of each case are followed there -- which is where memory that nothing
# has written yet is met): all-candidates kernel with
# fewer ids than beam slots (1:4), batch-wide window at beam 20 with one candidate per hypothesis (1:5 --
# the configuration in which a one-off randomised GPU run once ended in a memory fault), ragged windowed
# batch with an unused slot (1:6), all-candidates + window at beam 1 with an unused slot (1:7).
CPU_SUBSET = [(1, 4, 3), (1, 5, 5), (1, 6, 8), (1, 7, 3)]     # (seed of the list, case, decoding steps followed)


def small(name="cfg1", **over):
    w = gen.workload(name)
    w.update(over)
    w["eos_id"] = w["vocab"] - 1
    return w


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


def describe(seed0, case, mode, w, lens):
    return (f"case {seed0}/{case}: {mode} U={len(lens)} beam={w['beam']} V={w['vocab']} K={w['cand_k']} "
            f"M=({w['win_m1']},{w['win_m2']}) union={w.get('win_union', 0)} end={w['end_flags']} lens={[int(x) for x in lens]}")
