"""The synthetic-input generator: primitives against published vectors, recipe properties."""
import os

import numpy as np

import gen

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_philox_known_answers():
    n = 0
    for line in open(os.path.join(GOLD, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        w = [int(t, 16) for t in line.split()]
        assert list(gen.philox4x32_10(w[0:4], w[4:6])) == w[6:10]
        n += 1
    assert n == 3


def test_fnv_known_answers():
    for line in open(os.path.join(GOLD, "fnv1a64_kat.txt")):
        if line.startswith("#"):
            continue
        parts = line.rstrip("\n").split(" ")
        assert gen.fnv1a64(parts[0].encode()) == int(parts[1], 16)


def test_prefix_hash_is_incremental_and_le_int32():
    h = gen.prefix_hash([])
    assert h == 0xcbf29ce484222325
    for k in (5, 4999, 70000):
        h = gen.prefix_hash_extend(h, k)
    assert h == gen.prefix_hash([5, 4999, 70000])
    assert gen.prefix_hash([1]) == gen.fnv1a64(bytes([1, 0, 0, 0]))


def test_normals_and_streams():
    z = gen.normals(gen.stream_key(1, 3, 0, 1, 2), 200000)
    assert abs(z.mean()) < 0.01 and abs(z.std() - 1) < 0.01 and abs((z ** 4).mean() - 3) < 0.1
    z2 = gen.normals(gen.stream_key(1, 3, 0, 1, 3), 1000)
    assert abs(np.corrcoef(z[:1000], z2)[0, 1]) < 0.15
    # element e depends only on (key, e): a prefix of a longer draw is the shorter draw
    assert np.array_equal(gen.normals(9, 10), gen.normals(9, 1001)[:10])


def test_ctc_rows_are_log_distributions_and_blank_peaky():
    x = gen.ctc_utt(3, 0, 400, 5000, zipf_s=1.1)
    assert x.dtype == np.float32 and x.shape == (400, 5000)
    assert np.allclose(np.exp(x.astype(np.float64)).sum(1), 1.0, atol=1e-5)
    pb = np.exp(x[:, 0])
    assert 0.5 < (pb > 0.9).mean() < 0.75         # most of the ~70 % boosted frames are blank-dominated
    # Zipf prior: low ids carry most non-blank mass
    assert np.exp(x[:, 1]).mean() > 20 * np.exp(x[:, 2500]).mean()


def test_att_rows_keyed_by_prefix():
    a = gen.att_row(1, 0, 3, gen.prefix_hash([7, 8]), 5000)
    b = gen.att_row(1, 0, 3, gen.prefix_hash([7, 9]), 5000)
    assert abs(np.exp(a.astype(np.float64)).sum() - 1) < 1e-5 and not np.array_equal(a, b)
    rows = gen.att_rows(1, [0, 0], 3, [gen.prefix_hash([7, 8]), gen.prefix_hash([7, 9])], 5000)
    assert np.array_equal(rows[0], a) and np.array_equal(rows[1], b)


def test_workloads_and_lengths():
    w = gen.workload("cfg2")
    lens = gen.workload_lengths(w)
    assert lens.size == 64 and lens.min() >= 250 and lens.max() <= 875
    assert np.array_equal(lens, gen.workload_lengths(w))
    x = gen.ctc_batch(5, [3, 5], 8)
    assert x.shape == (2, 5, 8) and np.isnan(x[0, 3:]).all() and np.isfinite(x[0, :3]).all()
    seg = gen.segments(11, n_rec=2)
    assert seg.max() <= 500 and seg.size > 200 and np.all(np.diff(seg) >= 0)
