"""Seeded random graphs that stand in for the paper's datasets (Table 2).

* ``sbm_graph``: a small stochastic block model, every block materialised, so
  that a whole multi-partition run can be emulated on the CPU.
* ``chung_lu_partition0``: one partition's share of a power-law (Chung-Lu)
  graph with planted communities.  Only the community that partition 0 owns is
  built; remote endpoints are drawn from the closed-form weight distribution of
  the other nodes, so a graph of 10^8 nodes is never materialised.
"""
from __future__ import annotations

import numpy as np

from .partition import Partition, partition_from_entries


def sbm_graph(seed: int, n_nodes: int, n_blocks: int, p_intra: float, p_inter: float):
    """Undirected SBM without self-loops -> global CSR (ptr, col), equal blocks."""
    rng = np.random.Generator(np.random.PCG64(seed))
    block = np.arange(n_nodes) // (n_nodes // n_blocks)
    same = block[:, None] == block[None, :]
    prob = np.where(same, p_intra, p_inter)
    upper = np.triu(rng.random((n_nodes, n_nodes)) < prob, k=1)
    adj = upper | upper.T
    rows, cols = np.nonzero(adj)
    ptr = np.zeros(n_nodes + 1, dtype=np.int64)
    np.cumsum(np.bincount(rows, minlength=n_nodes), out=ptr[1:])
    return ptr, cols.astype(np.int64)


def _scaled_pareto_weights(u: np.ndarray, a: float, mean_target: float, cap: float):
    """min(c * u^-a, cap) with c solved so that the sample mean hits mean_target."""
    base = u ** (-a)
    lo, hi = 0.0, mean_target
    for _ in range(60):                      # bisection on c (mean is monotone in c)
        c = 0.5 * (lo + hi)
        if np.minimum(c * base, cap).mean() < mean_target:
            lo = c
        else:
            hi = c
    c = 0.5 * (lo + hi)
    return np.minimum(c * base, cap), c


def chung_lu_partition0(seed: int, n_total: int, n_comm: int, avg_deg: float,
                        exponent: float, intra_frac: float) -> Partition:
    """Partition 0 (= planted community 0) of a Chung-Lu graph.

    Node weights follow a Pareto law with tail exponent ``exponent`` scaled to
    mean ``avg_deg`` and cut at sqrt(total weight) (the usual Chung-Lu
    structural cutoff).  An inner node spends ``intra_frac`` of its weight on
    edges inside the community and the rest on edges to remote nodes.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    n_in = n_total // n_comm
    n_remote = n_total - n_in
    a = 1.0 / (exponent - 1.0)
    cap = float(np.sqrt(n_total * avg_deg))

    w, c = _scaled_pareto_weights(1.0 - rng.random(n_in), a, avg_deg, cap)
    cdf = np.cumsum(w)
    total = float(cdf[-1])

    # inner-inner edges: both endpoints proportional to weight
    m_in = int(round(intra_frac * total / 2.0))
    ea = np.searchsorted(cdf, rng.random(m_in) * total, side="right")
    eb = np.searchsorted(cdf, rng.random(m_in) * total, side="right")
    np.minimum(ea, n_in - 1, out=ea)
    np.minimum(eb, n_in - 1, out=eb)
    keep = ea != eb
    ea, eb = ea[keep], eb[keep]
    src_inner = np.concatenate([ea, eb])
    dst_inner = np.concatenate([eb, ea])

    # inner-remote edges: inner endpoint proportional to weight; the remote
    # endpoint is a weight *rank* r in [0, n_remote) whose weight is the Pareto
    # quantile min(c*((r+.5)/R)^-a, cap).  Ranks below r_cap sit at the cap.
    m_bd = int(round((1.0 - intra_frac) * total))
    src_bd = np.searchsorted(cdf, rng.random(m_bd) * total, side="right")
    np.minimum(src_bd, n_in - 1, out=src_bd)
    R = float(n_remote)
    r_cap = min(R, R * (cap / c) ** (-1.0 / a)) if cap > c else R
    mass_cap = r_cap * cap
    f_cap = (r_cap / R) ** (1.0 - a)
    mass_tail = c * R / (1.0 - a) * (1.0 - f_cap)
    u1 = rng.random(m_bd)
    u2 = rng.random(m_bd)
    in_cap = u1 * (mass_cap + mass_tail) < mass_cap
    rank = np.where(in_cap, u2 * r_cap,
                    R * (f_cap + u2 * (1.0 - f_cap)) ** (1.0 / (1.0 - a)))
    rank = np.minimum(rank.astype(np.int64), n_remote - 1)
    dst_gid = n_in + rank

    def full_degree(gids, incidence):
        r = (gids - n_in).astype(np.float64)
        return np.rint(np.minimum(c * ((r + 0.5) / R) ** (-a), cap)).astype(np.int64)

    return partition_from_entries(0, n_in, src_inner, dst_inner, src_bd, dst_gid,
                                  halo_full_degree=full_degree)
