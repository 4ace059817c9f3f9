"""Pins for the oracle's error-bound companions (sums of absolute terms S and term counts K).

The GPU parity tests hold an fp32 result x to
    |x - ref| <= 1e-4 * max(|ref|, 1e-6) + c * 2^-24 * sqrt(K) * S ,
so S and K must be what they claim to be: S the sum of the absolute values of the terms that make
up the element (through the aggregate and the product of one layer, Eq. 1 and Eq. 2 in the sampled
form of Appendix A), K their number.  Checked here against dense brute force with |.| applied to
every factor, against the triangle inequality (S >= |result|, equality for non-negative inputs), and
by showing that a rounded-to-fp32 evaluation in the worst order stays inside the bound while a
dropped term does not.  Nothing here calls the HIP library."""
import numpy as np
import pytest

from bns_inputs import SAMPLING_SEED, make_workload
from bns_inputs.workloads import sage_weights
from oracle import bns_oracle as orc
from parity_util import C_ERR, U, tolerance
from test_oracle_gcn import _dense_P_sampled
from test_oracle_sage import _dense_mean_matrix


@pytest.mark.parametrize("kind", [0, 1], ids=["gcn", "sage"])
@pytest.mark.parametrize("p,epoch", [(0.1, 0), (0.5, 1), (1.0, 0), (0.0, 0)])
def test_bounds_equal_dense_brute_force_of_absolute_values(tiny, kind, p, epoch):
    w = tiny
    P, L = w.part, w.n_layers
    W = w.W if kind == 0 else sage_weights(3, w.dims)
    ref = orc.step(P, w.loss_kind, w.X, w.halo_h, w.labels, W, SAMPLING_SEED, epoch, p, layer_kind=kind)
    bnd = orc.step_bounds(P, ref, w.X, w.halo_h, W, p, layer_kind=kind)
    kept = ref["sub"]["kept_ids"]
    M = np.abs(_dense_P_sampled(P, kept, p) if kind == 0 else _dense_mean_matrix(P, kept, p))
    nnz_row = np.count_nonzero(_dense_P_sampled(P, kept, p), axis=1)[:, None]    # incl. the self-loop
    nnz_col = np.count_nonzero(_dense_P_sampled(P, kept, p), axis=0)[:, None]
    for l in range(1, L + 1):
        d_in, d_out = w.dims[l - 1], w.dims[l]
        H_in = np.abs(ref["H"][l - 1])
        Hcat = np.vstack([H_in, np.abs(w.halo_h[l - 1][kept].astype(np.float64))])
        Wa = np.abs(W[l - 1].astype(np.float64))
        S_A, K_A = bnd["A"][l]
        S_H, K_H = bnd["H"][l]
        np.testing.assert_allclose(S_A, M @ Hcat, rtol=1e-12, atol=1e-300)
        left = M @ Hcat if kind == 0 else np.hstack([M @ Hcat, H_in])
        np.testing.assert_allclose(S_H, left @ Wa, rtol=1e-12, atol=1e-300)
        assert np.array_equal(K_A, np.maximum(nnz_row, 1))
        assert np.array_equal(K_H, nnz_row + (1 + kind) * d_in)
        # triangle inequality; equality where every term has one sign
        assert np.all(S_A >= np.abs(ref["A"][l]) * (1 - 1e-12))
        assert np.all(S_H >= np.abs(ref["H"][l]) * (1 - 1e-12))
        if l > 1 and kind == 0:      # aggregate of post-ReLU (non-negative) rows with positive weights
            np.testing.assert_allclose(S_A, ref["A"][l], rtol=1e-12, atol=1e-300)
        dZ = np.abs(ref["dZ_last"] if l == L else ref["dH"][l] * (ref["H"][l] > 0))
        S_dW, K_dW = bnd["dW"][l - 1]
        lhs = np.abs(ref["A"][l]) if kind == 0 else np.hstack([np.abs(ref["A"][l]), H_in])
        np.testing.assert_allclose(S_dW, lhs.T @ dZ, rtol=1e-12, atol=1e-300)
        assert K_dW == P.n_in
        assert np.all(S_dW >= np.abs(ref["dW"][l - 1]) * (1 - 1e-12))
        if l > 1:
            dcat = dZ @ Wa.T
            dHcat = M.T @ dcat[:, :d_in]
            S_dH, K_dH = bnd["dH"][l - 1]
            S_dh, K_dh = bnd["dhalo"][l - 1]
            want = dHcat[:P.n_in] + (dcat[:, d_in:] if kind == 1 else 0.0)
            np.testing.assert_allclose(S_dH, want, rtol=1e-12, atol=1e-300)
            np.testing.assert_allclose(S_dh, dHcat[P.n_in:], rtol=1e-12, atol=1e-300)
            assert np.array_equal(K_dH, nnz_col[:P.n_in] + d_out + 1)
            assert np.array_equal(K_dh, nnz_col[P.n_in:] + d_out)
            assert np.all(S_dH >= np.abs(ref["dH"][l - 1]) * (1 - 1e-12))
            assert np.all(S_dh >= np.abs(ref["dhalo"][l - 1]) * (1 - 1e-12))
        else:
            assert bnd["dH"][0] is None and bnd["dhalo"][0] is None


def _fp32_sequential_layer(P, sub, H_in, halo_h, W, p):
    """One GCN layer evaluated the way a careless fp32 implementation would: every weight, product
    and running sum rounded to fp32, neighbours and features in storage order."""
    f = np.float32
    n_in, kept = P.n_in, sub["kept_ids"]
    dis_in = (f(1) / np.sqrt(P.deg_in.astype(f))).astype(f)
    dis_h = (f(1) / np.sqrt(P.deg_halo.astype(f))).astype(f)
    s = f(1.0 / p) if kept.size else f(1)
    A = np.zeros((n_in, H_in.shape[1]), dtype=f)
    for v in range(n_in):
        acc = np.zeros(H_in.shape[1], dtype=f)
        for e in range(sub["row_ptr"][v], sub["row_ptr"][v + 1]):
            u = sub["col_idx"][e]
            if u < n_in:
                acc = (acc + f(dis_in[v] * dis_in[u]) * H_in[u].astype(f)).astype(f)
            else:
                b = kept[u - n_in]
                acc = (acc + f(f(dis_in[v] * dis_h[b]) * s) * halo_h[b]).astype(f)
        A[v] = acc
    Z = np.zeros((n_in, W.shape[1]), dtype=f)
    for k in range(W.shape[0]):
        Z = (Z + A[:, k:k + 1] * W[k:k + 1, :].astype(f)).astype(f)
    return A, Z


def test_sequential_fp32_stays_inside_the_bound_and_a_dropped_term_does_not(tiny):
    w = tiny
    P = w.part
    p, epoch = 0.5, 1
    sub = orc.sample_and_build(P, SAMPLING_SEED, epoch, p)
    X32 = w.X.astype(np.float32)
    a, z, _ = orc.layer_forward(P, sub, X32, w.halo_h[0], w.W[0], p, relu=False)
    b = orc.layer_forward_bounds(P, sub, X32, w.halo_h[0], w.W[0], p)
    A32, Z32 = _fp32_sequential_layer(P, sub, X32, w.halo_h[0], w.W[0], p)
    ra = np.abs(A32 - a) / (C_ERR * U * np.sqrt(b["K_A"]) * b["S_A"] + 1e-300)
    rz = np.abs(Z32 - z) / (C_ERR * U * np.sqrt(b["K_Z"]) * b["S_Z"] + 1e-300)
    # the rounding term alone (no relative term) already covers this evaluation order (the largest
    # ratios belong to one-entry rows, where the rounded weight d~_v^-1/2 d~_v^-1/2 is the whole error)
    assert ra.max() < 1.0 and rz.max() < 0.5, (ra.max(), rz.max())
    # ... and is not so wide that a mistake hides in it: drop one neighbour of one row
    v = int(np.argmax(np.diff(sub["row_ptr"])))
    sub2 = dict(sub)
    col2 = sub["col_idx"].copy()
    e = sub["row_ptr"][v] + 1
    rp2 = sub["row_ptr"].copy()
    rp2[v + 1:] -= 1
    sub2["row_ptr"], sub2["col_idx"] = rp2, np.delete(col2, e)
    a_bad, z_bad, _ = orc.layer_forward(P, sub2, X32, w.halo_h[0], w.W[0], p, relu=False)
    assert np.any(np.abs(a_bad[v] - a[v]) > tolerance(a[v], b["S_A"][v], b["K_A"][v]))
    assert np.any(np.abs(z_bad[v] - z[v]) > tolerance(z[v], b["S_Z"][v], b["K_Z"][v]))
    # a wrong 1/p (p of another epoch's setting) on the boundary terms is caught too
    a_p, _, _ = orc.layer_forward(P, sub, X32, w.halo_h[0], w.W[0], p * 1.01, relu=False)
    has_bd = np.diff(sub["row_ptr"]) > 0
    assert np.any(np.abs(a_p - a) > tolerance(a, b["S_A"], b["K_A"]))
    assert has_bd.any()


def test_layer_forward_is_the_step_forward(tiny):
    """layer_forward on the step's own inputs reproduces the step's layer (same arithmetic)."""
    w = tiny
    for kind, W in ((0, w.W), (1, sage_weights(3, w.dims))):
        ref = orc.step(w.part, w.loss_kind, w.X, w.halo_h, w.labels, W, SAMPLING_SEED, 2, 0.5, layer_kind=kind)
        for l in range(1, w.n_layers + 1):
            a, z, h = orc.layer_forward(w.part, ref["sub"], ref["H"][l - 1], w.halo_h[l - 1], W[l - 1], 0.5,
                                        layer_kind=kind, relu=l < w.n_layers)
            assert np.array_equal(a, ref["A"][l]) and np.array_equal(z, ref["Z"][l])
            assert np.array_equal(h, ref["H"][l])


def test_layer_backward_is_the_step_backward(tiny):
    """layer_backward on the step's own inputs reproduces the step's backward stage."""
    w = tiny
    L = w.n_layers
    for kind, W in ((0, w.W), (1, sage_weights(3, w.dims))):
        ref = orc.step(w.part, w.loss_kind, w.X, w.halo_h, w.labels, W, SAMPLING_SEED, 2, 0.5, layer_kind=kind)
        for l in range(L, 0, -1):
            dZ = ref["dZ_last"] if l == L else ref["dH"][l] * (ref["H"][l] > 0)
            dW, dH, dhalo = orc.layer_backward(w.part, ref["sub"], ref["A"][l], ref["H"][l - 1], W[l - 1], dZ, 0.5,
                                               layer_kind=kind, first_layer=(l == 1))
            assert np.array_equal(dW, ref["dW"][l - 1])
            if l > 1:
                assert np.array_equal(dH, ref["dH"][l - 1]) and np.array_equal(dhalo, ref["dhalo"][l - 1])
            else:
                assert dH is None and dhalo is None
