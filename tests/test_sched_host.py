"""Host-side scheduling helpers of the C library against their plain definitions and against the
properties the paper states for them (no GPU needed: none of these calls touches the device)."""
import numpy as np
import pytest

import paper_2101_05600_amd as m
from oracle import sched as ref


@pytest.fixture(scope="module", autouse=True)
def _built():
    import os
    if not os.path.exists(m._SO):
        m.build()


def test_hard_segments_paper_setting():
    """19-20 s at 100 frames/s (Sec. 4.4) on recordings of 5 s to 36 min (Sec. 4.1): every length in
    [min, max] once the recording is long enough, lengths differ by at most one frame."""
    rng = np.random.default_rng(5)
    for n in [500, 1899, 1900, 2000, 2001, 3800, 3999, 4001, 38000, 216000] + list(rng.integers(1, 220000, 200)):
        got = m.ctcbs_hard_segments(int(n), 1900, 2000)
        assert got.tolist() == ref.hard_segments(int(n), 1900, 2000)
        assert got.sum() == n and got.max() <= 2000 and got.max() - got.min() <= 1
        assert len(got) == -(-int(n) // 2000)                       # fewest pieces
        feasible = any(k * 1900 <= n <= k * 2000 for k in range(1, 200))
        if feasible:
            assert got.min() >= 1900
    assert len(m.ctcbs_hard_segments(0, 19, 20)) == 0
    with pytest.raises(m.CtcbsError):
        m.ctcbs_hard_segments(10, 5, 4)


def test_hard_segments_small_exhaustive():
    for n in range(0, 200):
        for lo, hi in [(1, 1), (3, 4), (7, 7), (9, 20), (19, 20)]:
            assert m.ctcbs_hard_segments(n, lo, hi).tolist() == ref.hard_segments(n, lo, hi)


def test_merge_pieces():
    rng = np.random.default_rng(11)
    # pieces like the paper's voice-activity output: short (a few seconds), some long ones
    for trial in range(100):
        k = int(rng.integers(0, 60))
        pieces = rng.integers(1, 1300, k)
        if k and trial % 3 == 0:
            pieces[rng.integers(0, k)] = rng.integers(2000, 9000)
        got = m.ctcbs_merge_pieces(pieces, 1500, 2000)
        assert got.tolist() == ref.merge_pieces(pieces.tolist(), 1500, 2000)
        assert got.sum() == pieces.sum()
        assert (got <= 2000).all()
        # every segment but the last reaches the minimum unless it is a part of a split one
        # (a split of a segment of length L >= min into ceil(L/max) parts gives parts >= L/2 > min/2)
        assert (got[:-1] >= 750).all()
    assert m.ctcbs_merge_pieces([], 15, 20).size == 0
    assert m.ctcbs_merge_pieces([3, 4], 15, 20).tolist() == [7]
    assert m.ctcbs_merge_pieces([10, 10, 30, 1], 15, 20).tolist() == [20, 15, 15, 1]


def test_plan_batches_properties():
    rng = np.random.default_rng(3)
    for trial in range(60):
        n = int(rng.integers(0, 300))
        lens = rng.integers(1, 500, n)
        max_utt = int(rng.integers(1, 40))
        cap = int(rng.choice([0, 600, 5000, 20000]))
        if cap and n and lens.max() > cap:
            with pytest.raises(m.CtcbsError):
                m.ctcbs_plan_batches(lens, max_utt, cap)
            continue
        order, begin = m.ctcbs_plan_batches(lens, max_utt, cap)
        ro, rb = ref.plan_batches(lens.tolist(), max_utt, cap)
        assert order.tolist() == ro and begin.tolist() == rb
        assert sorted(order.tolist()) == list(range(n))                  # a permutation
        sl = lens[order]
        assert (np.diff(sl) <= 0).all()                                  # longest first
        for b in range(len(begin) - 1):
            seg = sl[begin[b]:begin[b + 1]]
            assert 1 <= len(seg) <= max_utt
            if cap:
                assert len(seg) * seg[0] <= cap                          # padded size
            # greedy: the batch stops only where a limit would be broken (or the list ends)
            if begin[b + 1] < n:
                assert len(seg) == max_utt or (cap and (len(seg) + 1) * seg[0] > cap)


def test_plan_batches_korean_like_workload():
    """cfg3's segment list: batches of 128 sorted by length waste little padding."""
    import gen
    w = gen.workload("cfg3")
    lens = gen.segments(w["seed"])
    order, begin = m.ctcbs_plan_batches(lens, 128)
    assert len(begin) - 1 == -(-len(lens) // 128)
    sl = np.asarray(lens)[order]
    padded = sum((begin[b + 1] - begin[b]) * sl[begin[b]] for b in range(len(begin) - 1))
    assert padded <= 1.05 * sl.sum()
    # unsorted batching of the same list pads far more
    un = np.asarray(lens)[np.random.default_rng(0).permutation(len(lens))]
    padded_un = sum(len(un[i:i + 128]) * un[i:i + 128].max() for i in range(0, len(un), 128))
    assert padded_un > padded
