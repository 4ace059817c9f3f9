"""CPU oracle for one partition's BNS-GCN training step  --  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module; the product path never does.  It is independent of the HIP
library (no shared code) and works in fp64.

What it computes, and where the paper defines it:

* ``sample``       Algorithm 1, selection step: keep each boundary node
                   independently with probability p (redrawn every epoch).
* ``induced_csr``  Algorithm 1, subgraph step: node-induced subgraph on the
                   inner nodes plus the kept boundary nodes.
* ``forward``      Eq. 1 (aggregate) then Eq. 2 (update) per layer, in the
                   sampled matrix form of Appendix A:
                   Z = [P_VV P_VU] S [H_V ; H_U] W with the full-graph
                   propagation matrix P = D~^-1/2 (A+I) D~^-1/2 and
                   S = diag(1 for inner, 1/p for kept boundary); ReLU between
                   layers, none after the last.
* ``loss_and_grad``Algorithm 1, loss step: sum over inner nodes.
* ``backward``     Algorithm 1, backward step: gradients of that sum with
                   respect to every weight matrix, plus the gradients of the
                   kept boundary features (what would be sent back to their
                   owners, Section 3.2).
* ``step``         one iteration of Algorithm 1 for one partition, without the
                   exchange steps (one partition only) and with optional SGD.

The heavy integer and sparse loops are plain C (``bns_oracle.c``); dense
products use numpy's fp64 matmul as a library primitive.

Pins (tests/test_oracle_*.py): Philox known-answer vectors; binomial keep
statistics; p = 1 / p = 0 special cases; dense brute-force forward and
backward; fp64 finite differences; multi-partition emulation against the
dense full-graph GCN; unbiasedness and the closed-form variance of Appendix A.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# BNS_ORACLE_LIB: another build of the same source (the sanitizer build of oracle/build.py)
_LIB_PATH = os.environ.get("BNS_ORACLE_LIB") or os.path.join(_HERE, "libbns_oracle.so")
_lib = None

_i32p = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_i64p = np.ctypeslib.ndpointer(dtype=np.int64, flags="C_CONTIGUOUS")
_f64p = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")
_f32p = np.ctypeslib.ndpointer(dtype=np.float32, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(dtype=np.uint32, flags="C_CONTIGUOUS")


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build(force=False)
        L = C.CDLL(_LIB_PATH)
        L.bnso_num_threads.restype = C.c_int
        L.bnso_philox4x32_10.argtypes = [_u32p, _u32p, _u32p]
        L.bnso_draw.restype = C.c_uint32
        L.bnso_draw.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint64]
        L.bnso_threshold.restype = C.c_uint64
        L.bnso_threshold.argtypes = [C.c_double]
        L.bnso_sample.restype = C.c_int64
        L.bnso_sample.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_double, _i64p, C.c_int64,
                                  _i32p, _i32p]
        L.bnso_induced_csr.restype = C.c_int64
        L.bnso_induced_csr.argtypes = [C.c_int64, _i32p, _i32p, _i32p, _i32p, _i32p]
        L.bnso_transpose.argtypes = [C.c_int64, C.c_int64, _i32p, _i32p, _i32p, _i32p]
        L.bnso_aggregate.argtypes = [C.c_int64, C.c_int64, _i32p, _i32p, _i32p, _i32p, _i32p,
                                     C.c_double, _f64p, _f32p, _f64p]
        L.bnso_aggregate_bwd.argtypes = [C.c_int64, C.c_int64, C.c_int64, _i32p, _i32p, _i32p, _i32p,
                                         _i32p, C.c_double, _f64p, _f64p, _f64p]
        L.bnso_aggregate_mean.argtypes = [C.c_int64, C.c_int64, _i32p, _i32p, _i32p, _i32p, C.c_double,
                                          _f64p, _f32p, _f64p]
        L.bnso_aggregate_mean_bwd.argtypes = [C.c_int64, C.c_int64, C.c_int64, _i32p, _i32p, _i32p,
                                              C.c_double, _f64p, _f64p, _f64p]
        L.bnso_dropout_mask.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int64, C.c_int64,
                                        C.c_double, np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().bnso_num_threads())


def philox4x32_10(ctr, key):
    out = np.zeros(4, dtype=np.uint32)
    lib().bnso_philox4x32_10(np.asarray(ctr, dtype=np.uint32), np.asarray(key, dtype=np.uint32), out)
    return out


def draw(seed: int, epoch: int, part_id: int, gid: int) -> int:
    return int(lib().bnso_draw(seed, epoch, part_id, gid))


def threshold(p: float) -> int:
    return int(lib().bnso_threshold(float(p)))


def sample(seed, epoch, part_id, p, halo_gid):
    """-> (kept_ids int32[n_u] ascending, remap int32[B] rank-or-minus-one)."""
    halo_gid = np.ascontiguousarray(halo_gid, dtype=np.int64)
    B = halo_gid.shape[0]
    kept = np.empty(max(B, 1), dtype=np.int32)
    remap = np.empty(max(B, 1), dtype=np.int32)
    n = lib().bnso_sample(seed, epoch, part_id, float(p), halo_gid, B, kept, remap)
    return kept[:n].copy(), remap[:B]


def induced_csr(n_in, row_ptr0, col0, remap):
    """-> (row_ptr int32[n_in+1], col_idx int32[nnz]) of the sampled subgraph."""
    row_ptr = np.empty(n_in + 1, dtype=np.int32)
    col_idx = np.empty(max(col0.shape[0], 1), dtype=np.int32)
    remap_c = np.ascontiguousarray(remap if remap.shape[0] else np.zeros(1, np.int32))
    nnz = lib().bnso_induced_csr(n_in, row_ptr0, col0, remap_c, row_ptr, col_idx)
    return row_ptr, col_idx[:nnz].copy()


def transpose(n_rows, n_cols, row_ptr, col_idx):
    t_ptr = np.empty(n_cols + 1, dtype=np.int32)
    t_col = np.empty(max(col_idx.shape[0], 1), dtype=np.int32)
    ci = np.ascontiguousarray(col_idx if col_idx.shape[0] else np.zeros(1, np.int32))
    lib().bnso_transpose(n_rows, n_cols, row_ptr, ci, t_ptr, t_col)
    return t_ptr, t_col[:col_idx.shape[0]].copy()


def _pad1(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a if a.size else np.zeros(1, dtype=dtype)


def aggregate(part, row_ptr, col_idx, kept_ids, s_halo, H_in, halo_h):
    """Eq. 1 in the sampled form of Appendix A -> A f64[n_in, d]."""
    n_in, d = H_in.shape
    A = np.empty((n_in, d), dtype=np.float64)
    lib().bnso_aggregate(n_in, d, row_ptr, _pad1(col_idx, np.int32), part.deg_in,
                         _pad1(part.deg_halo, np.int32), _pad1(kept_ids, np.int32), float(s_halo),
                         np.ascontiguousarray(H_in, dtype=np.float64),
                         _pad1(halo_h, np.float32), A)
    return A


def aggregate_bwd(part, t_row_ptr, t_col_idx, kept_ids, s_halo, dA):
    """dHcat = S^T P^T dA -> (dH_in f64[n_in, d], dhalo f64[n_u, d])."""
    n_in, d = dA.shape
    n_u = kept_ids.shape[0]
    dH = np.empty((n_in, d), dtype=np.float64)
    dhalo = np.empty((max(n_u, 1), d), dtype=np.float64)
    lib().bnso_aggregate_bwd(n_in, n_u, d, t_row_ptr, _pad1(t_col_idx, np.int32), part.deg_in,
                             _pad1(part.deg_halo, np.int32), _pad1(kept_ids, np.int32),
                             float(s_halo), np.ascontiguousarray(dA, dtype=np.float64), dH, dhalo)
    return dH, dhalo[:n_u]


def halo_scale(p: float, n_kept: int) -> float:
    """S_uu for kept boundary nodes (Appendix A).  Never formed when nothing is kept (p = 0)."""
    return 1.0 / p if n_kept > 0 else 1.0


def dropout_mask(seed, epoch, part_id, layer, n_rows, n_cols, q):
    """uint8[n_rows, n_cols]: 1 where the element of hidden layer ``layer`` survives dropout."""
    keep = np.zeros((n_rows, n_cols), dtype=np.uint8)
    lib().bnso_dropout_mask(seed, epoch, part_id, layer, n_rows, n_cols, float(q), keep)
    return keep


def dropout_scale(q: float) -> float:
    """1/(1-q) in fp32, the factor that keeps the expectation of a dropped activation."""
    return float(np.float32(1.0 / (1.0 - q))) if q > 0.0 else 1.0


def _hidden(z, part, l, dropout):
    """ReLU, then (training with dropout = (q, seed, epoch)) drop and rescale."""
    h = np.maximum(z, 0.0)
    if dropout is not None and dropout[0] > 0.0:
        q, seed, epoch = dropout
        h = h * dropout_mask(seed, epoch, part.part_id, l, h.shape[0], h.shape[1], q) * dropout_scale(q)
    return h


def forward(part, sub, X, halo_h, W, p, Z_out=None, dropout=None):
    """All layers.  ``sub`` = dict(row_ptr, col_idx, kept_ids).  -> (A list, H list) with
    H[0] = X, H[l] = ReLU(A[l] W[l]) for l < L and H[L] = A[L] W[L] (logits).  If ``Z_out`` is a
    list, the pre-activations A[l] W[l] are appended to it (index l-1).  ``dropout`` =
    (q, seed, epoch): the hidden activations are dropped element-wise and rescaled by 1/(1-q)."""
    L = len(W)
    s = halo_scale(p, sub["kept_ids"].shape[0])
    H = [np.asarray(X, dtype=np.float64)]
    A = [None]
    for l in range(1, L + 1):
        a = aggregate(part, sub["row_ptr"], sub["col_idx"], sub["kept_ids"], s, H[l - 1], halo_h[l - 1])
        z = a @ np.asarray(W[l - 1], dtype=np.float64)
        A.append(a)
        H.append(_hidden(z, part, l, dropout) if l < L else z)
        if Z_out is not None:
            Z_out.append(z)
    return A, H


def loss_and_grad(logits, labels, loss_kind):
    """Sum over inner nodes of the per-node loss (Algorithm 1) and its gradient.

    kind 0: softmax cross-entropy, labels int[n];  kind 1: sigmoid binary
    cross-entropy summed over labels, labels {0,1}[n, C].
    """
    z = np.asarray(logits, dtype=np.float64)
    labels = np.asarray(labels)
    if loss_kind == 0:
        train = labels >= 0                      # a negative label: node outside the training set
        m = z.max(axis=1, keepdims=True)
        e = np.exp(z - m)
        se = e.sum(axis=1, keepdims=True)
        lse = (m + np.log(se))[:, 0]
        idx = np.arange(z.shape[0])
        safe = np.where(train, labels, 0)
        loss = float(np.sum((lse - z[idx, safe])[train]))
        g = e / se
        g[idx, safe] -= 1.0
        g[~train] = 0.0
        return loss, g
    train = labels != 255                        # 255: entry outside the training set
    y = np.where(train, labels, 0).astype(np.float64)
    terms = np.maximum(z, 0.0) - z * y + np.log1p(np.exp(-np.abs(z)))
    loss = float(np.sum(terms[train]))
    e = np.exp(-np.abs(z))
    g = np.where(z >= 0, 1.0 / (1.0 + e), e / (1.0 + e)) - y
    g[~train] = 0.0
    return loss, g


def adam_step(W, g, m, v, lr, beta1, beta2, eps, t):
    """One Adam step (Kingma & Ba 2015, the optimiser of Section 4) -> (W, m, v), fp64."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    return W - lr * m_hat / (np.sqrt(v_hat) + eps), m, v


def backward(part, sub, A, H, W, dZ_last, p, drop_scale=1.0):
    """-> (dW list[L], dhalo list[L] (entry 0 is None), dH list: dH[l] = grad wrt H[l], l=1..L-1).
    With dropout, H[l] > 0 exactly where the unit is active and kept, and its slope is drop_scale."""
    L = len(W)
    s = halo_scale(p, sub["kept_ids"].shape[0])
    dW = [None] * L
    dhalo = [None] * L
    dH = [None] * (L + 1)
    dZ = dZ_last
    for l in range(L, 0, -1):
        if l < L:
            dZ = dH[l] * (H[l] > 0.0) * drop_scale
        dW[l - 1] = A[l].T @ dZ
        if l > 1:
            dA = dZ @ np.asarray(W[l - 1], dtype=np.float64).T
            dH[l - 1], dhalo[l - 1] = aggregate_bwd(part, sub["t_row_ptr"], sub["t_col_idx"],
                                                    sub["kept_ids"], s, dA)
    return dW, dhalo, dH


# ---------------------------------------------------------------------------------------------
# GraphSAGE with a mean aggregator (Section 2), the model of the paper's experiments:
#   z_v = mean over the neighbours of v,  h'_v = sigma(W . CONCAT(z_v, h_v)),
# with W of shape [2 d_in, d_out] = [W_n ; W_s] (neighbour half first).  Under boundary sampling
# the kept boundary features are divided by p and the mean keeps the full-graph neighbour count
# (Section 3.2), so that the estimate of z_v is unbiased.
def aggregate_mean(part, row_ptr, col_idx, kept_ids, s_halo, H_in, halo_h):
    n_in, d = H_in.shape
    Z = np.empty((n_in, d), dtype=np.float64)
    lib().bnso_aggregate_mean(n_in, d, row_ptr, _pad1(col_idx, np.int32), part.deg_in,
                              _pad1(kept_ids, np.int32), float(s_halo),
                              np.ascontiguousarray(H_in, dtype=np.float64), _pad1(halo_h, np.float32), Z)
    return Z


def aggregate_mean_bwd(part, t_row_ptr, t_col_idx, kept_ids, s_halo, dZ):
    n_in, d = dZ.shape
    n_u = kept_ids.shape[0]
    dH = np.empty((n_in, d), dtype=np.float64)
    dhalo = np.empty((max(n_u, 1), d), dtype=np.float64)
    lib().bnso_aggregate_mean_bwd(n_in, n_u, d, t_row_ptr, _pad1(t_col_idx, np.int32), part.deg_in,
                                  float(s_halo), np.ascontiguousarray(dZ, dtype=np.float64), dH, dhalo)
    return dH, dhalo[:n_u]


def forward_sage(part, sub, X, halo_h, W, p, Z_out=None, dropout=None):
    """-> (A list, H list): A[l] = mean aggregate z of layer l, H[l] = ReLU([A[l] | H[l-1]] W[l])
    for l < L, no ReLU on the last layer."""
    L = len(W)
    s = halo_scale(p, sub["kept_ids"].shape[0])
    H = [np.asarray(X, dtype=np.float64)]
    A = [None]
    for l in range(1, L + 1):
        a = aggregate_mean(part, sub["row_ptr"], sub["col_idx"], sub["kept_ids"], s, H[l - 1], halo_h[l - 1])
        z = np.hstack([a, H[l - 1]]) @ np.asarray(W[l - 1], dtype=np.float64)
        A.append(a)
        H.append(_hidden(z, part, l, dropout) if l < L else z)
        if Z_out is not None:
            Z_out.append(z)
    return A, H


def backward_sage(part, sub, A, H, W, dZ_last, p, drop_scale=1.0):
    L = len(W)
    s = halo_scale(p, sub["kept_ids"].shape[0])
    dW = [None] * L
    dhalo = [None] * L
    dH = [None] * (L + 1)
    dZ = dZ_last
    for l in range(L, 0, -1):
        if l < L:
            dZ = dH[l] * (H[l] > 0.0) * drop_scale
        d_in = H[l - 1].shape[1]
        dW[l - 1] = np.hstack([A[l], H[l - 1]]).T @ dZ
        if l > 1:
            dcat = dZ @ np.asarray(W[l - 1], dtype=np.float64).T      # [n_in, 2 d_in]
            dh_nbr, dhalo[l - 1] = aggregate_mean_bwd(part, sub["t_row_ptr"], sub["t_col_idx"],
                                                      sub["kept_ids"], s, np.ascontiguousarray(dcat[:, :d_in]))
            dH[l - 1] = dh_nbr + dcat[:, d_in:]
    return dW, dhalo, dH


# ---------------------------------------------------------------------------------------------
# Error-bound companions.  An fp32 implementation of a sum of K products cannot be closer to the
# exact value than a few units of rounding times the sum of the ABSOLUTE values of its terms, however
# small the (possibly cancelling) result is.  The functions below return, for one layer given its
# inputs, that sum of absolute terms S for every output element and the number of terms K, so that a
# test can hold an fp32 result x to |x - ref| <= rtol * max(|ref|, floor) + c * 2^-24 * sqrt(K) * S.
# Every weight of the propagation matrix (Appendix A: P_vu > 0, S_uu = 1 or 1/p > 0; the mean
# aggregator's 1/deg > 0) is positive, so the sum of absolute terms of an aggregate is the same
# aggregate applied to the absolute values of its input.
def layer_forward_bounds(part, sub, H_in, halo_h, W, p, layer_kind=0):
    """-> dict(S_A, K_A, S_Z, K_Z) for A = aggregate(H_in, halo_h) and Z = A W (layer_kind 1:
    Z = [A | H_in] W).  S_*: f64 arrays shaped like A and Z; K_*: f64[n_in, 1] terms per element."""
    s = halo_scale(p, sub["kept_ids"].shape[0])
    agg = aggregate if layer_kind == 0 else aggregate_mean
    H_abs = np.abs(np.asarray(H_in, dtype=np.float64))
    S_A = agg(part, sub["row_ptr"], sub["col_idx"], sub["kept_ids"], s, H_abs, np.abs(halo_h))
    W_abs = np.abs(np.asarray(W, dtype=np.float64))
    K_A = np.diff(sub["row_ptr"]).astype(np.float64)[:, None]
    if layer_kind == 0:
        S_Z = S_A @ W_abs
        K_Z = K_A + H_abs.shape[1]
    else:
        S_Z = np.hstack([S_A, H_abs]) @ W_abs
        K_Z = K_A + 2 * H_abs.shape[1]
    return dict(S_A=S_A, K_A=np.maximum(K_A, 1.0), S_Z=S_Z, K_Z=K_Z)


def layer_backward_bounds(part, sub, A, H_in, W, dZ, p, layer_kind=0, first_layer=False):
    """-> dict(S_dW, K_dW, S_dH, K_dH, S_dhalo, K_dhalo) for dW = A^T dZ (layer_kind 1:
    [A | H_in]^T dZ) and [dH ; dhalo] = S^T P^T (dZ W^T) (layer_kind 1: plus the self half of
    dZ W^T).  first_layer: only the weight gradient exists."""
    s = halo_scale(p, sub["kept_ids"].shape[0])
    dZ_abs = np.abs(np.asarray(dZ, dtype=np.float64))
    A_abs = np.abs(np.asarray(A, dtype=np.float64))
    H_abs = np.abs(np.asarray(H_in, dtype=np.float64))
    n_in, d_in = A_abs.shape
    left = A_abs if layer_kind == 0 else np.hstack([A_abs, H_abs])
    out = dict(S_dW=left.T @ dZ_abs, K_dW=float(max(n_in, 1)))
    if first_layer:
        return out
    S_dA = dZ_abs @ np.abs(np.asarray(W, dtype=np.float64)).T
    d_out = dZ_abs.shape[1]
    t_len = np.diff(sub["t_row_ptr"]).astype(np.float64)[:, None]
    if layer_kind == 0:
        S_dH, S_dhalo = aggregate_bwd(part, sub["t_row_ptr"], sub["t_col_idx"], sub["kept_ids"], s, S_dA)
    else:
        S_dH, S_dhalo = aggregate_mean_bwd(part, sub["t_row_ptr"], sub["t_col_idx"], sub["kept_ids"], s,
                                           np.ascontiguousarray(S_dA[:, :d_in]))
        S_dH = S_dH + S_dA[:, d_in:]
    out.update(S_dH=S_dH, K_dH=t_len[:n_in] + d_out + 1, S_dhalo=S_dhalo, K_dhalo=t_len[n_in:] + d_out)
    return out


def step_bounds(part, ref, X, halo_h, W, p, layer_kind=0, dropout=0.0):
    """The bounds of every layer of ``ref`` = step(...), each taken on the oracle's own inputs of that
    layer.  -> dict of lists indexed like the results: A, H (index l), dW, dhalo (index l-1 as in
    step), dH (index l), each entry a pair (S, K)."""
    L = len(W)
    sub, ds = ref["sub"], dropout_scale(dropout)
    out = dict(A=[None] * (L + 1), H=[None] * (L + 1), dW=[None] * L, dhalo=[None] * L, dH=[None] * (L + 1))
    for l in range(1, L + 1):
        f = layer_forward_bounds(part, sub, ref["H"][l - 1], halo_h[l - 1], W[l - 1], p, layer_kind)
        out["A"][l] = (f["S_A"], f["K_A"])
        out["H"][l] = (f["S_Z"] * (ds if l < L else 1.0), f["K_Z"])
        dZ = ref["dZ_last"] if l == L else ref["dH"][l] * (ref["H"][l] > 0.0) * ds
        b = layer_backward_bounds(part, sub, ref["A"][l], ref["H"][l - 1], W[l - 1], dZ, p, layer_kind,
                                  first_layer=(l == 1))
        out["dW"][l - 1] = (b["S_dW"], b["K_dW"])
        if l > 1:
            out["dH"][l - 1] = (b["S_dH"], b["K_dH"])
            out["dhalo"][l - 1] = (b["S_dhalo"], b["K_dhalo"])
    return out


def layer_forward(part, sub, H_in, halo_h, W, p, layer_kind=0, relu=True, mask=None, drop_scale=1.0):
    """One layer of ``forward`` / ``forward_sage`` on a given input -> (A, Z, H): the aggregate, the
    pre-activation and the output (ReLU iff relu; then ``mask`` (0/1, optional) times drop_scale)."""
    s = halo_scale(p, sub["kept_ids"].shape[0])
    H_in = np.asarray(H_in, dtype=np.float64)
    Wd = np.asarray(W, dtype=np.float64)
    if layer_kind == 0:
        a = aggregate(part, sub["row_ptr"], sub["col_idx"], sub["kept_ids"], s, H_in, halo_h)
        z = a @ Wd
    else:
        a = aggregate_mean(part, sub["row_ptr"], sub["col_idx"], sub["kept_ids"], s, H_in, halo_h)
        z = np.hstack([a, H_in]) @ Wd
    h = np.maximum(z, 0.0) if relu else z
    if mask is not None:
        h = h * mask * drop_scale
    return a, z, h


def layer_backward(part, sub, A, H_in, W, dZ, p, layer_kind=0, first_layer=False):
    """One layer of ``backward`` / ``backward_sage`` on given inputs (dZ = gradient w.r.t. this layer's
    pre-activation) -> (dW, dH_in, dhalo): dH_in is the gradient w.r.t. the layer's input before any
    ReLU mask of the layer below; dH_in and dhalo are None for the first layer."""
    s = halo_scale(p, sub["kept_ids"].shape[0])
    dZ = np.asarray(dZ, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    Wd = np.asarray(W, dtype=np.float64)
    if layer_kind == 0:
        dW = A.T @ dZ
        if first_layer:
            return dW, None, None
        dH, dhalo = aggregate_bwd(part, sub["t_row_ptr"], sub["t_col_idx"], sub["kept_ids"], s, dZ @ Wd.T)
        return dW, dH, dhalo
    H_in = np.asarray(H_in, dtype=np.float64)
    d_in = H_in.shape[1]
    dW = np.hstack([A, H_in]).T @ dZ
    if first_layer:
        return dW, None, None
    dcat = dZ @ Wd.T
    dh_nbr, dhalo = aggregate_mean_bwd(part, sub["t_row_ptr"], sub["t_col_idx"], sub["kept_ids"], s,
                                       np.ascontiguousarray(dcat[:, :d_in]))
    return dW, dh_nbr + dcat[:, d_in:], dhalo


def sample_and_build(part, seed, epoch, p):
    kept_ids, remap = sample(seed, epoch, part.part_id, p, part.halo_gid)
    row_ptr, col_idx = induced_csr(part.n_in, part.row_ptr0, part.col0, remap)
    t_row_ptr, t_col_idx = transpose(part.n_in, part.n_in + kept_ids.shape[0], row_ptr, col_idx)
    return dict(kept_ids=kept_ids, remap=remap, row_ptr=row_ptr, col_idx=col_idx,
                t_row_ptr=t_row_ptr, t_col_idx=t_col_idx)


def step(part, loss_kind, X, halo_h, labels, W, seed, epoch, p, lr=0.0, layer_kind=0, dropout=0.0):
    """One iteration of Algorithm 1 on one partition (no exchange, optional SGD).
    layer_kind 0: GCN layer of Appendix A; 1: GraphSAGE-mean layer of Section 2.
    dropout: rate q on the hidden activations (0 = none)."""
    sub = sample_and_build(part, seed, epoch, p)
    Z = []
    fwd, bwd = (forward, backward) if layer_kind == 0 else (forward_sage, backward_sage)
    drop = (dropout, seed, epoch) if dropout > 0.0 else None
    A, H = fwd(part, sub, X, halo_h, W, p, Z_out=Z, dropout=drop)
    loss, dZ = loss_and_grad(H[-1], labels, loss_kind)
    dW, dhalo, dH = bwd(part, sub, A, H, W, dZ, p, drop_scale=dropout_scale(dropout))
    out = dict(sub=sub, A=A, H=H, Z=[None] + Z, loss=loss, dZ_last=dZ, dW=dW, dhalo=dhalo, dH=dH)
    if lr > 0.0:
        out["W_new"] = [np.asarray(w, dtype=np.float64) - lr * g for w, g in zip(W, dW)]
    return out
