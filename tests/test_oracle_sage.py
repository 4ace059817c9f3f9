"""Pins for the oracle's GraphSAGE-mean layer (Section 2: mean aggregator, W . CONCAT(z_v, h_v))
under boundary sampling (Section 3.2: kept boundary features divided by p).  No HIP here."""
import numpy as np
import pytest

from bns_inputs import SAMPLING_SEED, make_workload, partition_of_global_graph
from bns_inputs.workloads import tiny_global, sage_weights
from oracle import bns_oracle as orc


def _dense_mean_matrix(P, kept, p):
    """D^-1 [A_VV A_VU] S without self-loops, dense fp64, from the full local CSR."""
    M = np.zeros((P.n_in, P.n_in + P.n_halo))
    rows = np.repeat(np.arange(P.n_in), np.diff(P.row_ptr0))
    M[rows, P.col0] = 1.0
    M[np.arange(P.n_in), np.arange(P.n_in)] = 0.0
    deg = (P.deg_in - 1).astype(np.float64)
    inv = np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0)
    cols = np.concatenate([np.arange(P.n_in), P.n_in + kept])
    S = np.concatenate([np.ones(P.n_in), np.full(kept.size, 1.0 / p if kept.size else 1.0)])
    return inv[:, None] * M[:, cols] * S[None, :]


@pytest.mark.parametrize("p,epoch", [(0.1, 0), (0.5, 1), (1.0, 0), (0.0, 0)])
def test_dense_brute_force_tiny(tiny, p, epoch):
    w = tiny
    P = w.part
    W = sage_weights(3, w.dims)
    kept, _ = orc.sample(SAMPLING_SEED, epoch, P.part_id, p, P.halo_gid)
    Mn = _dense_mean_matrix(P, kept, p)
    L = w.n_layers
    H, Zs = [w.X.astype(np.float64)], [None]
    for l in range(1, L + 1):
        Hcat = np.vstack([H[l - 1], w.halo_h[l - 1][kept].astype(np.float64)])
        Zs.append(Mn @ Hcat)
        pre = np.hstack([Zs[l], H[l - 1]]) @ W[l - 1].astype(np.float64)
        H.append(np.maximum(pre, 0) if l < L else pre)
    pr = np.exp(H[L] - H[L].max(1, keepdims=True))
    pr /= pr.sum(1, keepdims=True)
    n = np.arange(P.n_in)
    loss = -np.log(pr[n, w.labels]).sum()
    g = pr.copy()
    g[n, w.labels] -= 1
    out = orc.step(P, w.loss_kind, w.X, w.halo_h, w.labels, W, SAMPLING_SEED, epoch, p, layer_kind=1)
    np.testing.assert_allclose(out["loss"], loss, rtol=1e-13)
    for l in range(L, 0, -1):
        np.testing.assert_allclose(out["A"][l], Zs[l], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(out["H"][l], H[l], rtol=1e-12, atol=1e-13)
        d_in = w.dims[l - 1]
        np.testing.assert_allclose(out["dW"][l - 1], np.hstack([Zs[l], H[l - 1]]).T @ g, rtol=1e-10, atol=1e-12)
        if l > 1:
            dcat = g @ W[l - 1].astype(np.float64).T
            dHcat = Mn.T @ dcat[:, :d_in]
            np.testing.assert_allclose(out["dhalo"][l - 1], dHcat[P.n_in:], rtol=1e-10, atol=1e-13)
            g = (dHcat[:P.n_in] + dcat[:, d_in:]) * (H[l - 1] > 0)


def test_mean_of_constant_features_is_the_constant():
    """With every neighbour present (p = 1) the mean of a constant is the constant."""
    w = make_workload(3, scale=64)
    P = w.part
    sub = orc.sample_and_build(P, SAMPLING_SEED, 0, 1.0)
    X = np.full((P.n_in, 3), -1.75)
    halo = np.full((P.n_halo, 3), -1.75, dtype=np.float32)
    Z = orc.aggregate_mean(P, sub["row_ptr"], sub["col_idx"], sub["kept_ids"], 1.0, X, halo)
    has_nbr = P.deg_in > 1
    np.testing.assert_allclose(Z[has_nbr], -1.75, rtol=1e-13)
    assert np.all(Z[~has_nbr] == 0.0)


def test_finite_differences(tiny):
    w, p = tiny, 0.5
    P = w.part
    W = [x.astype(np.float64) for x in sage_weights(3, w.dims)]
    sub = orc.sample_and_build(P, SAMPLING_SEED, 0, p)
    out = orc.step(P, w.loss_kind, w.X, w.halo_h, w.labels, W, SAMPLING_SEED, 0, p, layer_kind=1)

    def loss_of(Wx, hh):
        A, H = orc.forward_sage(P, sub, w.X, hh, Wx, p)
        return orc.loss_and_grad(H[-1], w.labels, w.loss_kind)[0]

    rng = np.random.default_rng(2)
    h = 1e-6
    for l in range(w.n_layers):
        big = np.abs(out["dW"][l]).max()
        for _ in range(150):
            i, j = rng.integers(W[l].shape[0]), rng.integers(W[l].shape[1])
            old = W[l][i, j]
            W[l][i, j] = old + h
            fp = loss_of(W, w.halo_h)
            W[l][i, j] = old - h
            fm = loss_of(W, w.halo_h)
            W[l][i, j] = old
            assert abs((fp - fm) / (2 * h) - out["dW"][l][i, j]) <= 1e-6 * big
    kept = sub["kept_ids"]
    hs = 2.0 ** -8
    big = np.abs(out["dhalo"][1]).max()
    for _ in range(30):
        r, j = rng.integers(kept.size), rng.integers(w.dims[1])
        hh = [x.copy() for x in w.halo_h]
        hh[1][kept[r], j] += hs
        fp = loss_of(W, hh)
        hh[1][kept[r], j] -= 2 * hs
        fm = loss_of(W, hh)
        assert abs((fp - fm) / (2 * hs) - out["dhalo"][1][r, j]) <= 2e-3 * big


def test_four_partition_emulation_equals_full_graph_sage():
    """p = 1 with real exchange reproduces dense full-graph GraphSAGE-mean training."""
    ptr, col, X_all, y_all = tiny_global()
    n, m = X_all.shape[0], 4
    blk = n // m
    dims = [64, 16, 8]
    W = [x.astype(np.float64) for x in sage_weights(9, dims)]
    Xd = X_all.astype(np.float64)
    # dense reference
    Adj = np.zeros((n, n))
    Adj[np.repeat(np.arange(n), np.diff(ptr)), col] = 1.0
    deg = Adj.sum(1)
    Mn = np.where(deg > 0, 1.0 / np.maximum(deg, 1), 0.0)[:, None] * Adj
    Z1 = Mn @ Xd
    P1 = np.hstack([Z1, Xd]) @ W[0]
    H1 = np.maximum(P1, 0)
    Z2 = Mn @ H1
    P2 = np.hstack([Z2, H1]) @ W[1]
    pr = np.exp(P2 - P2.max(1, keepdims=True))
    pr /= pr.sum(1, keepdims=True)
    loss_ref = -np.log(pr[np.arange(n), y_all]).sum()
    g2 = pr.copy()
    g2[np.arange(n), y_all] -= 1
    dW2_ref = np.hstack([Z2, H1]).T @ g2
    dcat = g2 @ W[1].T
    g1 = (Mn.T @ dcat[:, :16] + dcat[:, 16:]) * (P1 > 0)
    dW1_ref = np.hstack([Z1, Xd]).T @ g1
    # partition-parallel emulation
    parts = [partition_of_global_graph(i, ptr, col, i * blk, (i + 1) * blk) for i in range(m)]
    subs = [orc.sample_and_build(P, SAMPLING_SEED, 0, 1.0) for P in parts]
    Hg = [Xd, np.zeros((n, 16)), np.zeros((n, 8))]
    Zs = [[None] * 3 for _ in range(m)]
    for l in (1, 2):
        for i, P in enumerate(parts):
            sl = slice(i * blk, (i + 1) * blk)
            z = orc.aggregate_mean(P, subs[i]["row_ptr"], subs[i]["col_idx"], subs[i]["kept_ids"], 1.0,
                                   Hg[l - 1][sl], Hg[l - 1][P.halo_gid].astype(np.float32))
            Zs[i][l] = z
            pre = np.hstack([z, Hg[l - 1][sl]]) @ W[l - 1]
            Hg[l][sl] = np.maximum(pre, 0) if l == 1 else pre
    np.testing.assert_allclose(Hg[2], P2, rtol=0, atol=1e-6 * np.abs(P2).max())
    loss, dW2, dH1 = 0.0, np.zeros_like(W[1]), np.zeros((n, 16))
    for i, P in enumerate(parts):
        sl = slice(i * blk, (i + 1) * blk)
        f, g = orc.loss_and_grad(Hg[2][sl], y_all[sl], 0)
        loss += f
        dW2 += np.hstack([Zs[i][2], Hg[1][sl]]).T @ g
        dc = g @ W[1].T
        dh, dhalo = orc.aggregate_mean_bwd(P, subs[i]["t_row_ptr"], subs[i]["t_col_idx"], subs[i]["kept_ids"],
                                           1.0, np.ascontiguousarray(dc[:, :16]))
        dH1[sl] += dh + dc[:, 16:]
        np.add.at(dH1, P.halo_gid, dhalo)
    dW1 = np.zeros_like(W[0])
    for i in range(m):
        sl = slice(i * blk, (i + 1) * blk)
        dW1 += np.hstack([Zs[i][1], Xd[sl]]).T @ (dH1[sl] * (Hg[1][sl] > 0))
    np.testing.assert_allclose(loss, loss_ref, rtol=1e-6)
    np.testing.assert_allclose(dW2, dW2_ref, rtol=0, atol=2e-6 * np.abs(dW2_ref).max())
    np.testing.assert_allclose(dW1, dW1_ref, rtol=0, atol=2e-6 * np.abs(dW1_ref).max())


def test_mean_estimate_is_unbiased(tiny):
    w, p, T = tiny, 0.3, 2000
    P = w.part
    full = orc.sample_and_build(P, SAMPLING_SEED, 0, 1.0)
    Z = orc.aggregate_mean(P, full["row_ptr"], full["col_idx"], full["kept_ids"], 1.0, w.X, w.halo_h[0])
    acc, acc2 = np.zeros_like(Z), np.zeros_like(Z)
    for t in range(T):
        sub = orc.sample_and_build(P, SAMPLING_SEED, t, p)
        Zt = orc.aggregate_mean(P, sub["row_ptr"], sub["col_idx"], sub["kept_ids"], 1.0 / p, w.X, w.halo_h[0])
        acc += Zt
        acc2 += Zt * Zt
    mean = acc / T
    var = np.maximum(acc2 / T - mean ** 2, 0)
    touched = var > 1e-20
    assert (np.abs(mean - Z)[touched] / np.sqrt(var[touched] / T)).max() < 5.5
    np.testing.assert_allclose(mean[~touched], Z[~touched], rtol=1e-12, atol=1e-13)
