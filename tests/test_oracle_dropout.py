"""Pins for the oracle's dropout on hidden activations (Section 4 trains with dropout; the draw is
this build's counter-based reading).  No HIP here."""
import os

import numpy as np
import pytest

from bns_inputs import SAMPLING_SEED, make_workload
from bns_inputs.workloads import sage_weights
from oracle import bns_oracle as orc

M32 = 0xFFFFFFFF


def _philox_py(ctr, key):
    """Philox-4x32-10 in plain Python integers (Salmon et al., SC'11), independent of the oracle's C."""
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r:
            k[0] = (k[0] + 0x9E3779B9) & M32
            k[1] = (k[1] + 0xBB67AE85) & M32
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & M32, (p0 >> 32) ^ c[3] ^ k[1], p0 & M32]
    return c


def test_python_philox_matches_the_published_vectors():
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert _philox_py(v[0:4], v[4:6]) == v[6:10]


@pytest.mark.parametrize("q", [0.1, 0.5])
def test_mask_is_the_stated_draw(q):
    """Element (row, col): first word of Philox(counter (row, col, part*256+layer, epoch),
    key (seed lo, seed hi ^ 'drop')) below floor((1-q) 2^32)."""
    seed, epoch, part, layer, n, d = (5 << 32) | 77, 9, 3, 2, 37, 19
    mask = orc.dropout_mask(seed, epoch, part, layer, n, d, q)
    T = int(np.floor((1.0 - q) * 4294967296.0))
    key = [seed & M32, ((seed >> 32) ^ 0x64726F70) & M32]
    for row in range(n):
        for col in range(d):
            w = _philox_py([row, col, (part << 8) | layer, epoch], key)[0]
            assert mask[row, col] == (1 if w < T else 0), (row, col)


def test_keep_rate_and_independence():
    n, d = 4000, 64
    for q in (0.1, 0.3, 0.5):
        m = orc.dropout_mask(SAMPLING_SEED, 0, 0, 1, n, d, q).astype(np.float64)
        sd = np.sqrt(q * (1 - q) / (n * d))
        assert abs(m.mean() - (1 - q)) < 5 * sd
        # other layer / epoch / partition / seed: fresh, uncorrelated masks
        for other in (orc.dropout_mask(SAMPLING_SEED, 0, 0, 2, n, d, q),
                      orc.dropout_mask(SAMPLING_SEED, 1, 0, 1, n, d, q),
                      orc.dropout_mask(SAMPLING_SEED, 0, 1, 1, n, d, q),
                      orc.dropout_mask(SAMPLING_SEED + 1, 0, 0, 1, n, d, q)):
            o = other.astype(np.float64)
            corr = ((m - m.mean()) * (o - o.mean())).mean() / (q * (1 - q))
            assert abs(corr) < 5 / np.sqrt(n * d)
        # neighbouring elements (the four rows that share one Philox call, adjacent columns)
        for a, b in ((m[0::4], m[1::4]), (m[1::4], m[3::4]), (m[:, :-1], m[:, 1:])):
            corr = ((a - a.mean()) * (b - b.mean())).mean() / (q * (1 - q))
            assert abs(corr) < 5 / np.sqrt(a.size)
    assert orc.dropout_mask(1, 0, 0, 1, 50, 7, 0.0).all()


def test_dropout_stream_is_not_the_boundary_stream(tiny):
    """The mask of row block 0 must not repeat the boundary draw of the node with the same counter."""
    P = tiny.part
    kept, _ = orc.sample(SAMPLING_SEED, 0, 0, 0.5, np.arange(4096, dtype=np.int64))
    bd = np.zeros(4096)
    bd[kept] = 1
    # boundary counter (gid, 0, epoch 0, part 0) vs dropout counter (row//4, col 0, layer 0 part 0, epoch 0)
    m = orc.dropout_mask(SAMPLING_SEED, 0, 0, 0, 4 * 4096, 1, 0.5)[0::4, 0].astype(np.float64)
    corr = ((m - m.mean()) * (bd - bd.mean())).mean() / 0.25
    assert abs(corr) < 5 / np.sqrt(4096)


@pytest.mark.parametrize("kind", [0, 1], ids=["gcn", "sage"])
def test_rate_zero_changes_nothing(tiny, kind):
    w = tiny
    W = w.W if kind == 0 else sage_weights(3, w.dims)
    a = orc.step(w.part, w.loss_kind, w.X, w.halo_h, w.labels, W, SAMPLING_SEED, 0, 0.5, layer_kind=kind)
    b = orc.step(w.part, w.loss_kind, w.X, w.halo_h, w.labels, W, SAMPLING_SEED, 0, 0.5, layer_kind=kind,
                 dropout=0.0)
    assert a["loss"] == b["loss"]
    for x, y in zip(a["dW"], b["dW"]):
        assert np.array_equal(x, y)


def _dense_P(P, kept, p):
    """[P_VV P_VU] S of Appendix A as a dense fp64 matrix."""
    rows = np.repeat(np.arange(P.n_in), np.diff(P.row_ptr0))
    M = np.zeros((P.n_in, P.n_in + P.n_halo))
    M[rows, P.col0] = 1.0
    dis = np.concatenate([P.deg_in, P.deg_halo]).astype(np.float64) ** -0.5
    M = dis[:P.n_in, None] * M * dis[None, :]
    cols = np.concatenate([np.arange(P.n_in), P.n_in + kept])
    S = np.concatenate([np.ones(P.n_in), np.full(kept.size, 1.0 / p)])
    return M[:, cols] * S[None, :]


def test_dense_brute_force_with_dropout(tiny):
    """Three-layer GCN on Tiny with dense matrices, masks applied by hand."""
    w, p, q, epoch = tiny, 0.5, 0.4, 2
    P = w.part
    dims = [64, 16, 12, 8]
    rng = np.random.default_rng(0)
    W = [rng.standard_normal((a, b)) * 0.3 for a, b in zip(dims[:-1], dims[1:])]
    halo_h = [w.halo_h[0], w.halo_h[1], np.abs(rng.standard_normal((P.n_halo, 12))).astype(np.float32)]
    kept, _ = orc.sample(SAMPLING_SEED, epoch, P.part_id, p, P.halo_gid)
    Pm = _dense_P(P, kept, p)
    sc = float(np.float32(1.0 / (1.0 - q)))
    H, A, Mk = [w.X.astype(np.float64)], [None], [None]
    for l in (1, 2, 3):
        A.append(Pm @ np.vstack([H[l - 1], halo_h[l - 1][kept].astype(np.float64)]))
        z = A[l] @ W[l - 1]
        if l < 3:
            Mk.append(orc.dropout_mask(SAMPLING_SEED, epoch, P.part_id, l, P.n_in, dims[l], q))
            H.append(np.maximum(z, 0) * Mk[l] * sc)
        else:
            H.append(z)
    pr = np.exp(H[3] - H[3].max(1, keepdims=True))
    pr /= pr.sum(1, keepdims=True)
    n = np.arange(P.n_in)
    g = pr.copy()
    g[n, w.labels] -= 1
    out = orc.step(P, 0, w.X, halo_h, w.labels, W, SAMPLING_SEED, epoch, p, dropout=q)
    np.testing.assert_allclose(out["loss"], -np.log(pr[n, w.labels]).sum(), rtol=1e-12)
    assert 0.3 < (out["H"][1] > 0).mean() / (np.maximum(out["Z"][1], 0) > 0).mean() < 0.9
    for l in (3, 2, 1):
        np.testing.assert_allclose(out["H"][l], H[l], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(out["dW"][l - 1], A[l].T @ g, rtol=1e-9, atol=1e-11)
        if l > 1:
            dcat = Pm.T @ (g @ W[l - 1].T)
            np.testing.assert_allclose(out["dhalo"][l - 1], dcat[P.n_in:], rtol=1e-9, atol=1e-12)
            z_prev = A[l - 1] @ W[l - 2]
            g = dcat[:P.n_in] * (z_prev > 0) * Mk[l - 1] * sc


@pytest.mark.parametrize("kind", [0, 1], ids=["gcn", "sage"])
def test_finite_differences_with_dropout(tiny, kind):
    """The mask is a function of (seed, epoch) only, so the loss stays differentiable in W."""
    w, p, q = tiny, 0.5, 0.3
    P = w.part
    W = [x.astype(np.float64) for x in (w.W if kind == 0 else sage_weights(3, w.dims))]
    sub = orc.sample_and_build(P, SAMPLING_SEED, 0, p)
    out = orc.step(P, w.loss_kind, w.X, w.halo_h, w.labels, W, SAMPLING_SEED, 0, p, layer_kind=kind, dropout=q)
    fwd = orc.forward if kind == 0 else orc.forward_sage

    def loss_of(Wx):
        _, H = fwd(P, sub, w.X, w.halo_h, Wx, p, dropout=(q, SAMPLING_SEED, 0))
        return orc.loss_and_grad(H[-1], w.labels, w.loss_kind)[0]

    rng = np.random.default_rng(4)
    h = 1e-6
    for l in range(w.n_layers):
        big = np.abs(out["dW"][l]).max()
        for _ in range(120):
            i, j = rng.integers(W[l].shape[0]), rng.integers(W[l].shape[1])
            old = W[l][i, j]
            W[l][i, j] = old + h
            fp = loss_of(W)
            W[l][i, j] = old - h
            fm = loss_of(W)
            W[l][i, j] = old
            assert abs((fp - fm) / (2 * h) - out["dW"][l][i, j]) <= 1e-6 * big


def test_dropped_activation_keeps_its_expectation(tiny):
    """Mean over epochs of the dropped, rescaled hidden layer -> the plain ReLU output (p = 1)."""
    w, q, T = tiny, 0.5, 1500
    P = w.part
    sub = orc.sample_and_build(P, SAMPLING_SEED, 0, 1.0)
    _, H0 = orc.forward(P, sub, w.X, w.halo_h, w.W, 1.0)
    acc = np.zeros_like(H0[1])
    for t in range(T):
        acc += np.maximum(H0[1], 0) * orc.dropout_mask(SAMPLING_SEED, t, P.part_id, 1, *H0[1].shape, q) \
            * orc.dropout_scale(q)
    mean = acc / T
    sd = H0[1] * np.sqrt(q / (1 - q) / T)
    pos = H0[1] > 0
    assert (np.abs(mean - H0[1])[pos] / sd[pos]).max() < 5.5
    assert np.all(mean[~pos] == 0)
