"""Pins for the oracle's node-induced subgraph (Algorithm 1, subgraph step) and transpose."""
import numpy as np
import pytest

from bns_inputs import SAMPLING_SEED, make_workload
from oracle import bns_oracle as orc


def _dense_pattern(n_rows, n_cols, ptr, col):
    M = np.zeros((n_rows, n_cols), dtype=np.int8)
    rows = np.repeat(np.arange(n_rows), np.diff(ptr))
    M[rows, col] = 1
    return M


def _csr_of_dense(M):
    rows, cols = np.nonzero(M)
    ptr = np.zeros(M.shape[0] + 1, dtype=np.int32)
    np.cumsum(np.bincount(rows, minlength=M.shape[0]), out=ptr[1:])
    return ptr, cols.astype(np.int32)


@pytest.mark.parametrize("p,epoch", [(0.1, 0), (0.5, 3), (0.9, 1)])
def test_brute_force_dense_on_tiny(tiny, p, epoch):
    """Dense 0/1 adjacency, delete the dropped boundary columns, re-extract the CSR."""
    P = tiny.part
    sub = orc.sample_and_build(P, SAMPLING_SEED, epoch, p)
    M = _dense_pattern(P.n_in, P.n_in + P.n_halo, P.row_ptr0, P.col0)
    keep_cols = np.concatenate([np.arange(P.n_in), P.n_in + sub["kept_ids"]])
    ptr, col = _csr_of_dense(M[:, keep_cols])
    assert np.array_equal(sub["row_ptr"], ptr)
    assert np.array_equal(sub["col_idx"], col)
    tptr, tcol = _csr_of_dense(M[:, keep_cols].T)
    assert np.array_equal(sub["t_row_ptr"], tptr)
    assert np.array_equal(sub["t_col_idx"], tcol)


@pytest.mark.parametrize("cfg,scale", [(1, 1), (2, 16), (3, 64), (4, 16), (5, 64)])
def test_invariants(cfg, scale):
    w = make_workload(cfg, scale=scale)
    P = w.part
    inc = np.diff(P.halo_ptr)
    for p in sorted(set(w.p_list + [0.0, 1.0, 0.37])):
        sub = orc.sample_and_build(P, SAMPLING_SEED, 2, p)
        kept, ptr, col = sub["kept_ids"], sub["row_ptr"], sub["col_idx"]
        n_u = kept.size
        # edge count: inner block + every local edge of every kept boundary node
        assert ptr[-1] == col.size == P.e_in + inc[kept].sum()
        rows = np.repeat(np.arange(P.n_in), np.diff(ptr))
        # strictly ascending columns inside a row
        same_row = rows[1:] == rows[:-1]
        assert np.all(col[1:][same_row] > col[:-1][same_row])
        assert col.min() >= 0 and col.max() < P.n_in + max(n_u, 1)
        # every row keeps its self-loop
        assert np.array_equal(np.unique(rows[col == rows]), np.arange(P.n_in))
        # transpose twice = identity
        tt_ptr, tt_col = orc.transpose(P.n_in + n_u, P.n_in, sub["t_row_ptr"], sub["t_col_idx"])
        assert np.array_equal(tt_ptr, ptr) and np.array_equal(tt_col, col)
        if p == 1.0:
            assert np.array_equal(ptr, P.row_ptr0) and np.array_equal(col, P.col0)
            # transposed pattern = static inner transpose followed by the boundary-major lists
            assert np.array_equal(sub["t_row_ptr"][:P.n_in + 1], P.t_in_ptr)
            assert np.array_equal(sub["t_col_idx"][:P.e_in], P.t_in_col)
            assert np.array_equal(sub["t_row_ptr"][P.n_in:] - P.e_in, P.halo_ptr)
            assert np.array_equal(sub["t_col_idx"][P.e_in:], P.halo_col)
        if p == 0.0:
            assert n_u == 0 and col.size == P.e_in and col.max() < P.n_in
            assert np.array_equal(col, P.col0[P.col0 < P.n_in])


def test_partition_inputs_are_consistent():
    """Inner degree (with self-loop) equals the full local row length (every neighbour of an
    inner node is local or boundary); boundary degree is at least its local incidence + 1."""
    for cfg, scale in [(1, 1), (3, 64)]:
        P = make_workload(cfg, scale=scale).part
        assert np.array_equal(P.deg_in, np.diff(P.row_ptr0))
        assert np.all(P.deg_halo >= np.diff(P.halo_ptr) + 1)
        assert np.all(np.diff(P.halo_gid) > 0)
        assert np.all(np.diff(P.halo_ptr) >= 1)
