"""Seeded generators: determinism, ranges, and the backing-row formula against big integers."""
import numpy as np
import pytest

from paper_2210_08804_amd import inputs

M64 = (1 << 64) - 1


def py_mix(x):
    x &= M64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & M64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & M64
    x ^= x >> 31
    return x


def py_value(key, j, version):
    z = py_mix((key & M64) ^ py_mix((((version << 32) | j) + 0x9E3779B97F4A7C15) & M64))
    return ((z >> 40) - (1 << 23)) / float(1 << 23)


def test_backing_rows_match_bigint_formula():
    keys = np.array([0, 1, -1, 123456789012345, (1 << 63) - 1, -(1 << 63) + 5], dtype=np.int64)
    for version in (0, 1, 77):
        rows = inputs.backing_rows(keys, 16, version)
        assert rows.dtype == np.float32 and rows.shape == (6, 16)
        for i, k in enumerate(keys.tolist()):
            for j in range(16):
                assert float(rows[i, j]) == py_value(k, j, version)
    per_key = inputs.backing_rows(keys, 8, np.array([0, 1, 2, 3, 4, 5]))
    for i, k in enumerate(keys.tolist()):
        assert float(per_key[i, 3]) == py_value(k, 3, i)


def test_backing_rows_range_and_spread():
    rows = inputs.backing_rows(np.arange(4096, dtype=np.int64), 128)
    assert rows.min() >= -1.0 and rows.max() < 1.0
    assert abs(float(rows.mean())) < 0.01
    # rows of different keys / versions differ
    assert len({r.tobytes() for r in rows}) == 4096
    assert (inputs.backing_rows([5], 128, 0) != inputs.backing_rows([5], 128, 1)).any()


def test_key_streams_are_seeded_and_in_range():
    a = inputs.uniform_keys(26624, 1 << 18, 0)
    assert (a == inputs.uniform_keys(26624, 1 << 18, 0)).all()
    assert a.min() >= 0 and a.max() < (1 << 18) and a.dtype == np.int64
    z = inputs.zipf_keys(106496, 10 ** 8, 1.05, 1)
    assert (z == inputs.zipf_keys(106496, 10 ** 8, 1.05, 1)).all()
    assert (z != inputs.zipf_keys(106496, 10 ** 8, 1.05, 2)).any()
    assert z.min() >= 0 and z.max() < 10 ** 8
    # power law with alpha 1.05 over 1e8 ids: the hottest id takes a few percent of all draws and
    # ids below 2^24 take the bulk
    top = float((z == 0).mean())
    assert 0.03 < top < 0.09
    assert 0.90 < float((z < (1 << 24)).mean()) < 0.97


def test_vocab_sizes_log_uniform():
    v = inputs.log_uniform_vocab(26, 1e3, 1e8, 7)
    assert v.shape == (26,) and v.min() >= 1000 and v.max() <= 10 ** 8
    assert (v == inputs.log_uniform_vocab(26, 1e3, 1e8, 7)).all()


@pytest.mark.parametrize("alpha,space", [(1.05, 10 ** 8), (1.2, 10 ** 6), (1.5, 10 ** 5)])
def test_zipf_keys_follow_the_power_law(alpha, space):
    """The key streams stand in for the paper's power-law query distributions (Sec. 2.2; its
    synthetic dataset draws with alpha = 1.2 and sends about 95 % of the lookups to 10 % of the
    table, Sec. 7.1).  Checked against the closed form of the sampled law: the share of lookups
    that fall on the hottest fraction f of the key space is ((f N)^(1-alpha) - 1) / (N^(1-alpha) - 1),
    and the rank-frequency curve has slope -alpha in log-log."""
    n = 400000
    keys = inputs.zipf_keys(n, space, alpha, 11)
    a = 1.0 - alpha
    for f in (0.001, 0.01, 0.1, 0.5):
        share = float((keys < f * space).mean())
        expect = ((f * space) ** a - 1.0) / (float(space) ** a - 1.0)
        assert abs(share - expect) < 0.004, (f, share, expect)
    if alpha == 1.2:
        assert 0.94 < float((keys < 0.1 * space).mean()) < 0.975        # the paper's "95 % on 10 %"
    # slope of log(count) over log(rank) for the ranks that occur often enough to be measured
    counts = np.bincount(keys[keys < 200], minlength=200).astype(np.float64)
    ranks = np.arange(1, 201, dtype=np.float64)
    ok = counts >= 50
    # the sampled law is the continuous density integrated over [r, r+1): compare with that
    expect = (ranks + 1.0) ** a - ranks ** a
    expect = expect / expect[ok].sum() * counts[ok].sum()
    rel = np.abs(counts[ok] - expect[ok]) / np.sqrt(expect[ok])
    assert rel.max() < 6.0, "rank frequencies leave the power law by more than sampling noise"
    slope = np.polyfit(np.log(ranks[ok][2:]), np.log(counts[ok][2:]), 1)[0]
    assert abs(slope + alpha) < 0.15, slope
