"""Pins for the oracle's forward, loss and backward (Eq. 1-2, Appendix A, Algorithm 1).

Nothing here calls the HIP library.  The oracle is checked against dense
brute force, closed forms, fp64 finite differences, a four-partition emulation
of partition-parallel training against the dense full-graph GCN (p = 1 is
full-graph training, Section 4), and the estimator's mean and variance
(Section 3.2 "unbiased", Appendix A).
"""
import numpy as np
import pytest

from bns_inputs import SAMPLING_SEED, make_workload, partition_of_global_graph
from bns_inputs.workloads import tiny_global, glorot_weights
from oracle import bns_oracle as orc


# ----------------------------------------------------------------------------- dense brute force
def _dense_P_sampled(P, kept, p):
    """[P_VV P_VU] S as a dense fp64 matrix, built from the *full* local CSR."""
    M = np.zeros((P.n_in, P.n_in + P.n_halo))
    rows = np.repeat(np.arange(P.n_in), np.diff(P.row_ptr0))
    M[rows, P.col0] = 1.0
    dis = np.concatenate([P.deg_in, P.deg_halo]).astype(np.float64) ** -0.5
    Pfull = dis[:P.n_in, None] * M * dis[None, :]
    cols = np.concatenate([np.arange(P.n_in), P.n_in + kept])
    S = np.concatenate([np.ones(P.n_in), np.full(kept.size, 1.0 / p if kept.size else 1.0)])
    return Pfull[:, cols] * S[None, :]


def _dense_step(w, p, epoch):
    P = w.part
    kept, _ = orc.sample(SAMPLING_SEED, epoch, P.part_id, p, P.halo_gid)
    Ps = _dense_P_sampled(P, kept, p)
    L = w.n_layers
    Wd = [x.astype(np.float64) for x in w.W]
    H, A = [w.X.astype(np.float64)], [None]
    for l in range(1, L + 1):
        Hcat = np.vstack([H[l - 1], w.halo_h[l - 1][kept].astype(np.float64)])
        A.append(Ps @ Hcat)
        Z = A[l] @ Wd[l - 1]
        H.append(np.maximum(Z, 0) if l < L else Z)
    # softmax cross-entropy, written directly
    z = H[L]
    pr = np.exp(z - z.max(1, keepdims=True))
    pr /= pr.sum(1, keepdims=True)
    n = np.arange(P.n_in)
    loss = -np.log(pr[n, w.labels]).sum()
    dZ = pr.copy()
    dZ[n, w.labels] -= 1
    dW, dhalo = [None] * L, [None] * L
    for l in range(L, 0, -1):
        dW[l - 1] = A[l].T @ dZ
        if l > 1:
            dHcat = Ps.T @ (dZ @ Wd[l - 1].T)
            dhalo[l - 1] = dHcat[P.n_in:]
            dZ = dHcat[:P.n_in] * (H[l - 1] > 0)
    return dict(A=A, H=H, loss=loss, dW=dW, dhalo=dhalo, kept=kept)


@pytest.mark.parametrize("p,epoch", [(0.1, 0), (0.5, 1), (1.0, 0), (0.0, 0)])
def test_dense_brute_force_tiny(tiny, p, epoch):
    w = tiny
    ref = _dense_step(w, p, epoch)
    out = orc.step(w.part, w.loss_kind, w.X, w.halo_h, w.labels, w.W, SAMPLING_SEED, epoch, p)
    for l in range(1, w.n_layers + 1):
        np.testing.assert_allclose(out["A"][l], ref["A"][l], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(out["H"][l], ref["H"][l], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(out["dW"][l - 1], ref["dW"][l - 1], rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(out["loss"], ref["loss"], rtol=1e-13)
    for l in range(1, w.n_layers):
        np.testing.assert_allclose(out["dhalo"][l], ref["dhalo"][l], rtol=1e-10, atol=1e-13)
    assert out["dhalo"][0] is None


def test_dense_brute_force_three_layers_bce():
    """A deeper model with the multi-label loss on a scaled multilabel workload cut to a size
    where dense matrices are affordable."""
    w = make_workload(4, scale=256)
    P = w.part
    p, epoch = 0.5, 2
    kept, _ = orc.sample(SAMPLING_SEED, epoch, 0, p, P.halo_gid)
    Ps = _dense_P_sampled(P, kept, p)
    Wd = [x.astype(np.float64) for x in w.W]
    L = w.n_layers
    H, A = [w.X.astype(np.float64)], [None]
    for l in range(1, L + 1):
        A.append(Ps @ np.vstack([H[l - 1], w.halo_h[l - 1][kept].astype(np.float64)]))
        Z = A[l] @ Wd[l - 1]
        H.append(np.maximum(Z, 0) if l < L else Z)
    y = w.labels.astype(np.float64)
    sig = 1 / (1 + np.exp(-H[L]))
    loss = -(y * np.log(sig) + (1 - y) * np.log(1 - sig)).sum()
    dZ = sig - y
    out = orc.step(P, w.loss_kind, w.X, w.halo_h, w.labels, w.W, SAMPLING_SEED, epoch, p)
    np.testing.assert_allclose(out["loss"], loss, rtol=1e-12)
    for l in range(L, 0, -1):
        np.testing.assert_allclose(out["dW"][l - 1], A[l].T @ dZ, rtol=1e-9, atol=1e-11)
        if l > 1:
            dHcat = Ps.T @ (dZ @ Wd[l - 1].T)
            np.testing.assert_allclose(out["dhalo"][l - 1], dHcat[P.n_in:], rtol=1e-9, atol=1e-12)
            dZ = dHcat[:P.n_in] * (H[l - 1] > 0)


# ----------------------------------------------------------------------------- closed forms
def test_regular_graph_constant_features_pass_through():
    """On a regular graph with self-loops every row of P sums to one, so constant features
    come out of the aggregate unchanged (p = 1, halves of a circulant graph)."""
    n = 40
    nbr = np.array([[(i + s) % n for s in (-2, -1, 1, 2)] for i in range(n)])
    ptr = np.arange(0, 4 * n + 1, 4)
    col = np.sort(nbr, axis=1).ravel()
    P = partition_of_global_graph(0, ptr, col, 0, n // 2)
    assert P.n_halo == 4 and np.all(P.deg_in == 5) and np.all(P.deg_halo == 5)
    sub = orc.sample_and_build(P, 1, 0, 1.0)
    X = np.full((n // 2, 3), 2.5)
    halo = np.full((P.n_halo, 3), 2.5, dtype=np.float32)
    A = orc.aggregate(P, sub["row_ptr"], sub["col_idx"], sub["kept_ids"], 1.0, X, halo)
    np.testing.assert_allclose(A, 2.5, rtol=1e-14)


def test_loss_closed_forms():
    n, Cc = 37, 8
    labels = np.arange(n) % Cc
    loss, g = orc.loss_and_grad(np.full((n, Cc), 3.25), labels, 0)
    np.testing.assert_allclose(loss, n * np.log(Cc), rtol=1e-14)
    np.testing.assert_allclose(g.sum(axis=1), 0, atol=1e-15)
    y = (np.arange(n * Cc).reshape(n, Cc) % 3 == 0).astype(np.uint8)
    loss, g = orc.loss_and_grad(np.zeros((n, Cc)), y, 1)
    np.testing.assert_allclose(loss, n * Cc * np.log(2), rtol=1e-14)
    np.testing.assert_allclose(g, 0.5 - y, atol=1e-15)
    # large logits stay finite
    loss, g = orc.loss_and_grad(np.array([[800.0, -800.0]]), np.array([1]), 0)
    np.testing.assert_allclose(loss, 1600.0, rtol=1e-14)
    loss, _ = orc.loss_and_grad(np.array([[800.0, -800.0]]), np.array([[0, 1]], dtype=np.uint8), 1)
    np.testing.assert_allclose(loss, 1600.0, rtol=1e-14)


# ----------------------------------------------------------------------------- finite differences
def _loss_of(w, W, halo_h, sub, p):
    A, H = orc.forward(w.part, sub, w.X, halo_h, W, p)
    return orc.loss_and_grad(H[-1], w.labels, w.loss_kind)[0]


def test_finite_differences_every_weight(tiny):
    w, p = tiny, 0.5
    sub = orc.sample_and_build(w.part, SAMPLING_SEED, 0, p)
    out = orc.step(w.part, w.loss_kind, w.X, w.halo_h, w.labels, w.W, SAMPLING_SEED, 0, p)
    h = 1e-6
    for l in range(w.n_layers):
        W = [x.astype(np.float64) for x in w.W]
        g = np.zeros_like(W[l])
        for i in range(W[l].shape[0]):
            for j in range(W[l].shape[1]):
                old = W[l][i, j]
                W[l][i, j] = old + h
                fp = _loss_of(w, W, w.halo_h, sub, p)
                W[l][i, j] = old - h
                fm = _loss_of(w, W, w.halo_h, sub, p)
                W[l][i, j] = old
                g[i, j] = (fp - fm) / (2 * h)
        scale = np.abs(out["dW"][l]).max()
        assert np.abs(g - out["dW"][l]).max() <= 1e-6 * scale


def test_finite_differences_boundary_features(tiny):
    """dhalo[l] is the gradient with respect to the unscaled features of the kept boundary
    nodes at the input of layer l+1."""
    w, p = tiny, 0.5
    sub = orc.sample_and_build(w.part, SAMPLING_SEED, 0, p)
    out = orc.step(w.part, w.loss_kind, w.X, w.halo_h, w.labels, w.W, SAMPLING_SEED, 0, p)
    kept = sub["kept_ids"]
    h = 2.0 ** -8                                   # exactly representable in the fp32 input
    rng = np.random.default_rng(5)
    g_ref = out["dhalo"][1]
    big = np.abs(g_ref).max()
    for _ in range(40):
        r, j = rng.integers(kept.size), rng.integers(w.dims[1])
        hh = [x.copy() for x in w.halo_h]
        hh[1][kept[r], j] += h
        fp = _loss_of(w, w.W, hh, sub, p)
        hh[1][kept[r], j] -= 2 * h
        fm = _loss_of(w, w.W, hh, sub, p)
        assert abs((fp - fm) / (2 * h) - g_ref[r, j]) <= 2e-3 * big
    # a boundary node that was not kept has no influence at all
    dropped = np.setdiff1d(np.arange(w.part.n_halo), kept)[0]
    hh = [x.copy() for x in w.halo_h]
    hh[0][dropped] += 1.0
    hh[1][dropped] += 1.0
    assert _loss_of(w, w.W, hh, sub, p) == _loss_of(w, w.W, w.halo_h, sub, p)


# ----------------------------------------------------------------------------- 4-partition emulation
def _dense_full_graph(ptr, col, X, y, W):
    n = X.shape[0]
    Adj = np.eye(n)
    Adj[np.repeat(np.arange(n), np.diff(ptr)), col] = 1.0
    dis = Adj.sum(1) ** -0.5
    Pm = dis[:, None] * Adj * dis[None, :]
    PX = Pm @ X
    Z1 = PX @ W[0]
    H1 = np.maximum(Z1, 0)
    PH = Pm @ H1
    Z2 = PH @ W[1]
    pr = np.exp(Z2 - Z2.max(1, keepdims=True))
    pr /= pr.sum(1, keepdims=True)
    loss = -np.log(pr[np.arange(n), y]).sum()
    dZ2 = pr.copy()
    dZ2[np.arange(n), y] -= 1
    dW2 = PH.T @ dZ2
    dZ1 = (Pm.T @ (dZ2 @ W[1].T)) * (Z1 > 0)
    dW1 = PX.T @ dZ1
    return Z2, loss, [dW1, dW2]


def test_four_partition_emulation_equals_full_graph():
    """p = 1 with real boundary exchange (features forward, feature gradients backward, sum of
    weight gradients) reproduces dense full-graph GCN training on all 2000 nodes."""
    ptr, col, X_all, y_all = tiny_global()
    n, m = X_all.shape[0], 4
    blk = n // m
    dims = [64, 16, 8]
    W = [x.astype(np.float64) for x in glorot_weights(7, dims)]
    Xd = X_all.astype(np.float64)
    parts = [partition_of_global_graph(i, ptr, col, i * blk, (i + 1) * blk) for i in range(m)]
    subs = [orc.sample_and_build(P, SAMPLING_SEED, 0, 1.0) for P in parts]
    Hg = [Xd, None, None]
    As = [[None] * 3 for _ in range(m)]
    for l in (1, 2):
        nxt = np.zeros((n, dims[l]))
        for i, P in enumerate(parts):
            halo = Hg[l - 1][P.halo_gid].astype(np.float32)        # "receive H_U"
            a = orc.aggregate(P, subs[i]["row_ptr"], subs[i]["col_idx"], subs[i]["kept_ids"], 1.0,
                              Hg[l - 1][i * blk:(i + 1) * blk], halo)
            As[i][l] = a
            z = a @ W[l - 1]
            nxt[i * blk:(i + 1) * blk] = np.maximum(z, 0) if l == 1 else z
        Hg[l] = nxt
    Z2, loss_ref, dW_ref = _dense_full_graph(ptr, col, Xd, y_all, W)
    np.testing.assert_allclose(Hg[2], Z2, rtol=0, atol=1e-6 * np.abs(Z2).max())
    loss = 0.0
    dW = [np.zeros_like(W[0]), np.zeros_like(W[1])]
    dH1 = np.zeros((n, dims[1]))
    for i, P in enumerate(parts):
        sl = slice(i * blk, (i + 1) * blk)
        f, dZ = orc.loss_and_grad(Hg[2][sl], y_all[sl], 0)
        loss += f
        dW[1] += As[i][2].T @ dZ
        dh, dhalo = orc.aggregate_bwd(P, subs[i]["t_row_ptr"], subs[i]["t_col_idx"],
                                      subs[i]["kept_ids"], 1.0, dZ @ W[1].T)
        dH1[sl] += dh
        np.add.at(dH1, P.halo_gid, dhalo)                            # "send feature gradients"
    for i in range(m):
        sl = slice(i * blk, (i + 1) * blk)
        dW[0] += As[i][1].T @ (dH1[sl] * (Hg[1][sl] > 0))
    np.testing.assert_allclose(loss, loss_ref, rtol=1e-6)
    for a, b in zip(dW, dW_ref):
        np.testing.assert_allclose(a, b, rtol=0, atol=2e-6 * np.abs(b).max())


# ----------------------------------------------------------------------------- estimator statistics
def test_unbiased_and_variance_closed_form(tiny):
    """E[Z~] = Z (unbiased), and for the linear part of a layer the exact variance under
    independent Bernoulli keeps is ((1-p)/p) * sum_v sum_{u in B} ||P_vu H_u W||^2, which is
    below the paper's bound (1/p) gamma^2 ||P_VB||_F^2 (Appendix A)."""
    w, p, T = tiny, 0.3, 3000
    P = w.part
    W0 = w.W[0].astype(np.float64)
    full = orc.sample_and_build(P, SAMPLING_SEED, 0, 1.0)
    Z = orc.aggregate(P, full["row_ptr"], full["col_idx"], full["kept_ids"], 1.0,
                      w.X, w.halo_h[0]) @ W0
    acc = np.zeros_like(Z)
    acc2 = np.zeros_like(Z)
    frob = np.zeros(T)
    for t in range(T):
        sub = orc.sample_and_build(P, SAMPLING_SEED, t, p)
        Zt = orc.aggregate(P, sub["row_ptr"], sub["col_idx"], sub["kept_ids"], 1.0 / p,
                           w.X, w.halo_h[0]) @ W0
        acc += Zt
        acc2 += Zt * Zt
        frob[t] = ((Zt - Z) ** 2).sum()
    mean = acc / T
    var = np.maximum(acc2 / T - mean ** 2, 0)
    touched = var > 1e-20
    zscore = np.abs(mean - Z)[touched] / np.sqrt(var[touched] / T)
    assert zscore.max() < 5.5
    np.testing.assert_allclose(mean[~touched], Z[~touched], rtol=1e-12, atol=1e-13)
    # exact variance and the bound, from the dense boundary block of P
    M = np.zeros((P.n_in, P.n_in + P.n_halo))
    M[np.repeat(np.arange(P.n_in), np.diff(P.row_ptr0)), P.col0] = 1.0
    dis = np.concatenate([P.deg_in, P.deg_halo]).astype(np.float64) ** -0.5
    P_VB = (dis[:P.n_in, None] * M * dis[None, :])[:, P.n_in:]
    HW = w.halo_h[0].astype(np.float64) @ W0
    exact = (1 - p) / p * np.sum(P_VB ** 2 * (HW ** 2).sum(1)[None, :])
    bound = (1 / p) * (np.sqrt((HW ** 2).sum(1)).max() ** 2) * (P_VB ** 2).sum()
    assert abs(frob.mean() - exact) < 5 * frob.std() / np.sqrt(T)
    assert abs(frob.mean() / exact - 1) < 0.1
    assert exact <= bound


def test_renumbering_the_inner_nodes_changes_nothing():
    """Local ids are the partitioner's free choice: with the inner nodes renumbered by descending
    degree the same boundary nodes are kept (the draw depends on global ids only), the loss is the
    same and so are the weight gradients (sums over nodes)."""
    a = make_workload(3, scale=32)
    b = make_workload(3, scale=32, local_order="degree")
    assert np.all(np.diff(b.part.deg_in) <= 0) and not np.all(np.diff(a.part.deg_in) <= 0)
    ra = orc.step(a.part, a.loss_kind, a.X, a.halo_h, a.labels, a.W, SAMPLING_SEED, 0, 0.5)
    rb = orc.step(b.part, b.loss_kind, b.X, b.halo_h, b.labels, b.W, SAMPLING_SEED, 0, 0.5)
    assert np.array_equal(ra["sub"]["kept_ids"], rb["sub"]["kept_ids"])
    np.testing.assert_allclose(rb["loss"], ra["loss"], rtol=1e-12)
    for x, y in zip(ra["dW"], rb["dW"]):
        np.testing.assert_allclose(y, x, rtol=1e-9, atol=1e-11)
    for x, y in zip(ra["dhalo"][1:], rb["dhalo"][1:]):
        np.testing.assert_allclose(y, x, rtol=1e-9, atol=1e-11)
