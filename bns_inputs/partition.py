"""Static per-partition index structures (the inputs G_i, B_i of Algorithm 1).

A partition owns ``n_in`` inner nodes (local ids 0..n_in-1) and sees ``n_halo``
boundary nodes: remote nodes with at least one edge into the inner set
(Section 3.1).  Only inner rows exist; a boundary node b appears as column
``n_in + b``.  Everything here is integer index bookkeeping.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass
class Partition:
    part_id: int
    n_in: int
    n_halo: int
    row_ptr0: np.ndarray   # int32[n_in+1]  full local CSR (inner rows)
    col0: np.ndarray       # int32[nnz0]    strictly ascending per row, self-loop present
    t_in_ptr: np.ndarray   # int32[n_in+1]  transpose of the inner-inner block
    t_in_col: np.ndarray   # int32[E_in]
    halo_ptr: np.ndarray   # int32[n_halo+1] boundary-major lists: b -> inner neighbours
    halo_col: np.ndarray   # int32[E_bd]
    halo_gid: np.ndarray   # int64[n_halo]  global node id of each boundary node, ascending
    deg_in: np.ndarray     # int32[n_in]    full-graph degree + 1 (self-loop) of inner nodes
    deg_halo: np.ndarray   # int32[n_halo]  full-graph degree + 1 of boundary nodes

    @property
    def nnz0(self) -> int:
        return int(self.col0.shape[0])

    @property
    def e_in(self) -> int:
        return int(self.t_in_col.shape[0])

    @property
    def e_bd(self) -> int:
        return int(self.halo_col.shape[0])


def _csr_from_sorted_keys(keys: np.ndarray, n_rows: int, n_cols: int):
    rows = keys // n_cols
    cols = keys - rows * n_cols
    counts = np.bincount(rows, minlength=n_rows)
    ptr = np.zeros(n_rows + 1, dtype=np.int64)
    np.cumsum(counts, out=ptr[1:])
    return ptr, cols


def partition_from_entries(part_id: int, n_in: int,
                           src_inner: np.ndarray, dst_inner: np.ndarray,
                           src_bd: np.ndarray, dst_gid: np.ndarray,
                           halo_full_degree=None) -> Partition:
    """Assemble a Partition from raw entry lists.

    ``(src_inner[k], dst_inner[k])`` are inner->inner entries in local ids
    (both directions must be listed by the caller for an undirected graph);
    self-loops are added here.  ``(src_bd[k], dst_gid[k])`` are inner->remote
    entries with the remote endpoint given by global id.  Duplicates are
    removed.  ``halo_full_degree(gids, local_incidence) -> int array`` returns
    the boundary nodes' full-graph degree (without self-loop); by default the
    local incidence is used.
    """
    src_inner = np.asarray(src_inner, dtype=np.int64)
    dst_inner = np.asarray(dst_inner, dtype=np.int64)
    src_bd = np.asarray(src_bd, dtype=np.int64)
    dst_gid = np.asarray(dst_gid, dtype=np.int64)

    halo_gid, b_of_entry = np.unique(dst_gid, return_inverse=True)
    n_halo = int(halo_gid.shape[0])
    n_cols = n_in + n_halo

    loops = np.arange(n_in, dtype=np.int64)
    keys = np.concatenate([
        src_inner * n_cols + dst_inner,
        loops * n_cols + loops,
        src_bd * n_cols + (n_in + b_of_entry.astype(np.int64)),
    ])
    keys = np.unique(keys)
    if keys.shape[0] >= 2**31:
        raise ValueError("partition has >= 2^31 entries")
    row_ptr0, col0 = _csr_from_sorted_keys(keys, n_in, n_cols)
    rows = keys // n_cols

    inner = col0 < n_in
    # transpose of the inner-inner block: sort by (col, row)
    tk = np.sort(col0[inner] * n_in + rows[inner])
    t_in_ptr, t_in_col = _csr_from_sorted_keys(tk, n_in, n_in)
    # boundary-major lists: sort by (b, row)
    if n_halo > 0:
        hk = np.sort((col0[~inner] - n_in) * n_in + rows[~inner])
        halo_ptr, halo_col = _csr_from_sorted_keys(hk, n_halo, n_in)
    else:
        halo_ptr = np.zeros(1, dtype=np.int64)
        halo_col = np.zeros(0, dtype=np.int64)

    deg_in = np.diff(row_ptr0)                      # inner + boundary neighbours + self-loop
    incidence = np.diff(halo_ptr)
    if halo_full_degree is None:
        deg_h = incidence.copy()
    else:
        deg_h = np.maximum(np.asarray(halo_full_degree(halo_gid, incidence), dtype=np.int64),
                           incidence)
    deg_halo = deg_h + 1

    i32 = np.int32
    return Partition(
        part_id=int(part_id), n_in=int(n_in), n_halo=n_halo,
        row_ptr0=row_ptr0.astype(i32), col0=col0.astype(i32),
        t_in_ptr=t_in_ptr.astype(i32), t_in_col=t_in_col.astype(i32),
        halo_ptr=halo_ptr.astype(i32), halo_col=halo_col.astype(i32),
        halo_gid=halo_gid.astype(np.int64),
        deg_in=deg_in.astype(i32), deg_halo=deg_halo.astype(i32),
    )


def partition_of_global_graph(part_id: int, g_ptr: np.ndarray, g_col: np.ndarray,
                              lo: int, hi: int) -> Partition:
    """Cut the partition owning global nodes [lo, hi) out of a whole graph.

    ``g_ptr/g_col`` is the global CSR of an undirected graph *without*
    self-loops.  Boundary nodes get their true full-graph degree.
    """
    g_ptr = np.asarray(g_ptr, dtype=np.int64)
    g_col = np.asarray(g_col, dtype=np.int64)
    n_in = hi - lo
    seg = slice(int(g_ptr[lo]), int(g_ptr[hi]))
    src = np.repeat(np.arange(lo, hi, dtype=np.int64), np.diff(g_ptr[lo:hi + 1])) - lo
    dst = g_col[seg]
    is_in = (dst >= lo) & (dst < hi)
    gdeg = np.diff(g_ptr)

    def full_degree(gids, incidence):
        return gdeg[gids]

    return partition_from_entries(part_id, n_in,
                                  src[is_in], dst[is_in] - lo,
                                  src[~is_in], dst[~is_in],
                                  halo_full_degree=full_degree)


def relabel_inner(part: Partition, order: np.ndarray) -> Partition:
    """The same partition with its inner nodes renumbered: new local id i is old local id
    ``order[i]`` (a permutation of 0..n_in-1).  Local ids are the partitioner's free choice; the
    boundary nodes keep their order (ascending global id).  Index bookkeeping only."""
    order = np.asarray(order, dtype=np.int64)
    rank = np.empty(part.n_in, dtype=np.int64)
    rank[order] = np.arange(part.n_in, dtype=np.int64)
    rows = np.repeat(np.arange(part.n_in, dtype=np.int64), np.diff(part.row_ptr0))
    cols = part.col0.astype(np.int64)
    inner = cols < part.n_in
    deg_h = part.deg_halo.astype(np.int64) - 1
    gid = part.halo_gid

    def full_degree(gids, incidence):
        return deg_h[np.searchsorted(gid, gids)]

    out = partition_from_entries(part.part_id, part.n_in, rank[rows[inner]], rank[cols[inner]],
                                 rank[rows[~inner]], gid[cols[~inner] - part.n_in],
                                 halo_full_degree=full_degree)
    assert np.array_equal(out.halo_gid, part.halo_gid) and np.array_equal(out.deg_in, part.deg_in[order])
    return out
