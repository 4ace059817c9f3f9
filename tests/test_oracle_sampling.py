"""Pins for the oracle's boundary sampling (Algorithm 1, selection step).

The paper fixes: each boundary node is kept independently with probability p,
redrawn every epoch and independently per partition (Section 3.2); p = 1 is
unsampled training and p = 0 drops every boundary node (Section 4).
The generator itself (Philox-4x32-10) is pinned to its published
known-answer vectors.
"""
import os

import numpy as np
import pytest

from bns_inputs import SAMPLING_SEED, make_workload
from oracle import bns_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _philox_py(ctr, key):
    """Independent big-integer Philox-4x32-10 (used to check the key/counter mapping)."""
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r:
            k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
    return c


def test_philox_known_answers():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        out = orc.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]
        assert _philox_py(v[0:4], v[4:6]) == v[6:10]


def test_draw_uses_every_key_word():
    seed, epoch, part, gid = 0x0123456789ABCDEF, 7, 3, 0x00000005_0000002A
    base = orc.draw(seed, epoch, part, gid)
    expect = _philox_py([gid & 0xFFFFFFFF, gid >> 32, epoch, part], [seed & 0xFFFFFFFF, seed >> 32])[0]
    assert base == expect
    others = [orc.draw(seed ^ 1, epoch, part, gid), orc.draw(seed ^ (1 << 32), epoch, part, gid),
              orc.draw(seed, epoch + 1, part, gid), orc.draw(seed, epoch, part + 1, gid),
              orc.draw(seed, epoch, part, gid ^ 1), orc.draw(seed, epoch, part, gid ^ (1 << 32))]
    assert len(set(others + [base])) == 7


def test_threshold_is_integer_rule():
    assert orc.threshold(1.0) == 2**32
    assert orc.threshold(0.0) == 0
    assert orc.threshold(0.5) == 2**31
    assert orc.threshold(0.1) == int(np.floor(0.1 * 2**32))


def test_p0_keeps_none_p1_keeps_all(tiny):
    gid = tiny.part.halo_gid
    k0, r0 = orc.sample(SAMPLING_SEED, 0, 0, 0.0, gid)
    assert k0.size == 0 and np.all(r0 == -1)
    k1, r1 = orc.sample(SAMPLING_SEED, 0, 0, 1.0, gid)
    assert np.array_equal(k1, np.arange(gid.size)) and np.array_equal(r1, np.arange(gid.size))


def test_kept_list_and_remap_agree(tiny):
    gid = tiny.part.halo_gid
    T = orc.threshold(0.3)
    kept, remap = orc.sample(11, 5, 2, 0.3, gid)
    flags = np.array([orc.draw(11, 5, 2, int(g)) < T for g in gid])
    assert np.array_equal(kept, np.nonzero(flags)[0])
    assert np.all(np.diff(kept) > 0)
    assert np.array_equal(remap[kept], np.arange(kept.size))
    assert np.all(remap[~flags] == -1)


@pytest.mark.parametrize("B,p", [(329, 0.1), (200_000, 0.1), (200_000, 0.01), (3_000_000, 0.1)])
def test_kept_count_is_binomial(B, p):
    gid = np.arange(1000, 1000 + B, dtype=np.int64) * 37
    kept, _ = orc.sample(SAMPLING_SEED, 0, 0, p, gid)
    q = orc.threshold(p) / 2**32
    assert abs(kept.size - B * q) <= 5.0 * np.sqrt(B * q * (1 - q))


def test_per_epoch_counts_and_per_node_frequency(tiny):
    """100 epochs: every count within 5 sigma; 10^4 epochs: chi-square on per-node keep
    frequency, lag-1 correlation across epochs and correlation across partitions ~ 0."""
    gid = tiny.part.halo_gid
    B, p = gid.size, 0.1
    n_ep = 10_000
    keep = np.zeros((n_ep, B), dtype=np.int8)
    other = np.zeros((n_ep, B), dtype=np.int8)
    for t in range(n_ep):
        k, _ = orc.sample(SAMPLING_SEED, t, 0, p, gid)
        keep[t, k] = 1
        k, _ = orc.sample(SAMPLING_SEED, t, 1, p, gid)      # same nodes seen by another partition
        other[t, k] = 1
    counts = keep.sum(axis=1)
    sd = np.sqrt(B * p * (1 - p))
    assert np.all(np.abs(counts[:100] - B * p) <= 5 * sd)
    assert abs(counts.var() / (B * p * (1 - p)) - 1.0) < 0.1            # binomial variance
    freq = keep.sum(axis=0)
    chi2 = np.sum((freq - n_ep * p) ** 2 / (n_ep * p * (1 - p)))        # ~ chi2(B)
    assert abs(chi2 - B) < 5 * np.sqrt(2 * B)
    x = keep.astype(np.float64) - p
    lag1 = np.mean(x[1:] * x[:-1]) / (p * (1 - p))
    cross = np.mean(x * (other.astype(np.float64) - p)) / (p * (1 - p))
    neigh = np.mean(x[:, 1:] * x[:, :-1]) / (p * (1 - p))               # adjacent nodes
    tol = 5.0 / np.sqrt(n_ep * B)
    assert abs(lag1) < tol and abs(cross) < tol and abs(neigh) < tol


def test_samples_differ_between_epochs_and_partitions(tiny):
    gid = tiny.part.halo_gid
    a, _ = orc.sample(SAMPLING_SEED, 0, 0, 0.5, gid)
    b, _ = orc.sample(SAMPLING_SEED, 1, 0, 0.5, gid)
    c, _ = orc.sample(SAMPLING_SEED, 0, 1, 0.5, gid)
    assert not np.array_equal(a, b) and not np.array_equal(a, c)
