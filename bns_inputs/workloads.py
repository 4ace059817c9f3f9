"""The five synthetic workloads (shapes follow Table 2 and the models of Section 4).

Seeds: graph = 220310983 + cfg, features +100, labels +200, weights +300,
boundary hidden features +400 + layer.  ``scale`` > 1 shrinks the node count
(and caps the average degree) for quick parity cases with the same feature
widths, so that tile tails and ragged rows still occur.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

from .graphs import chung_lu_partition0, sbm_graph
from .partition import Partition, partition_of_global_graph, relabel_inner

SAMPLING_SEED = 2203
_BASE_SEED = 220310983

LOSS_CE = 0    # softmax cross-entropy, labels int32[n_in]
LOSS_BCE = 1   # sigmoid binary cross-entropy, labels uint8[n_in, C]

CONFIGS = {
    1: dict(name="tiny-sbm", kind="sbm", n_total=2000, n_comm=4, p_intra=0.005, p_inter=0.0005,
            dims=[64, 16, 8], loss=LOSS_CE, label_zipf=None, p_list=[0.1]),
    2: dict(name="dense-degree-share", kind="cl", n_total=233_000, n_comm=8, avg_deg=490.0,
            exponent=2.1, intra=0.85, dims=[602, 256, 256, 256, 41], loss=LOSS_CE,
            label_zipf=None, p_list=[1.0, 0.1, 0.01]),
    3: dict(name="medium-degree-share", kind="cl", n_total=2_450_000, n_comm=8, avg_deg=50.0,
            exponent=2.3, intra=0.90, dims=[100, 128, 128, 47], loss=LOSS_CE,
            label_zipf=1.1, p_list=[0.1]),
    4: dict(name="multilabel-share", kind="cl", n_total=717_000, n_comm=8, avg_deg=20.0,
            exponent=2.5, intra=0.80, dims=[300, 512, 512, 512, 100], loss=LOSS_BCE,
            label_zipf=None, p_list=[0.1]),
    5: dict(name="very-large-one-share", kind="cl", n_total=111_000_000, n_comm=192, avg_deg=29.0,
            exponent=2.2, intra=0.75, dims=[128, 128, 128, 172], loss=LOSS_CE,
            label_zipf=1.05, p_list=[0.1]),
}


@dataclass
class Workload:
    cfg: int
    name: str
    part: Partition
    dims: List[int]                 # d_0 .. d_L
    loss_kind: int
    X: np.ndarray                   # f32[n_in, d_0]
    halo_h: List[np.ndarray]        # L arrays f32[n_halo, d_l], l = 0..L-1
    labels: np.ndarray              # int32[n_in] or uint8[n_in, C]
    W: List[np.ndarray]             # L arrays f32[d_{l-1}, d_l]
    p_list: List[float] = field(default_factory=list)
    seed: int = SAMPLING_SEED

    @property
    def n_layers(self) -> int:
        return len(self.dims) - 1


def glorot_weights(seed: int, dims: List[int]) -> List[np.ndarray]:
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for fan_in, fan_out in zip(dims[:-1], dims[1:]):
        lim = np.sqrt(6.0 / (fan_in + fan_out))
        out.append(rng.uniform(-lim, lim, size=(fan_in, fan_out)).astype(np.float32))
    return out


def _normal_f32(rng, shape):
    return rng.standard_normal(size=shape, dtype=np.float32)


def make_labels(seed: int, n: int, n_classes: int, loss_kind: int, zipf):
    rng = np.random.Generator(np.random.PCG64(seed))
    if loss_kind == LOSS_BCE:
        return (rng.random((n, n_classes)) < 0.05).astype(np.uint8)
    if zipf is None:
        return rng.integers(0, n_classes, size=n).astype(np.int32)
    pr = 1.0 / np.arange(1, n_classes + 1, dtype=np.float64) ** zipf
    pr /= pr.sum()
    return rng.choice(n_classes, size=n, p=pr).astype(np.int32)


def tiny_global(cfg_seed: int = _BASE_SEED + 1):
    """The whole Tiny graph: (ptr, col, X_all f32[2000,64], y_all int32[2000])."""
    c = CONFIGS[1]
    ptr, col = sbm_graph(cfg_seed, c["n_total"], c["n_comm"], c["p_intra"], c["p_inter"])
    rng = np.random.Generator(np.random.PCG64(cfg_seed + 100))
    X_all = _normal_f32(rng, (c["n_total"], c["dims"][0]))
    y_all = make_labels(cfg_seed + 200, c["n_total"], c["dims"][-1], LOSS_CE, None)
    return ptr, col, X_all, y_all


def make_workload(cfg: int, scale: int = 1, part_id: int = 0, local_order: str = "native") -> Workload:
    """local_order: how the partition numbers its inner nodes.  "native": the generator's order (no
    structure: neighbours are spread over the whole id range); "degree": descending full-graph
    degree (ties by native id), an order a partitioner can emit for free and the measurement of what
    node order does to the aggregate's cache behaviour."""
    c = CONFIGS[cfg]
    seed = _BASE_SEED + cfg
    dims = list(c["dims"])
    L = len(dims) - 1
    if c["kind"] == "sbm":
        ptr, col, X_all, y_all = tiny_global(seed)
        n_blk = c["n_total"] // c["n_comm"]
        lo, hi = part_id * n_blk, (part_id + 1) * n_blk
        part = partition_of_global_graph(part_id, ptr, col, lo, hi)
        X = np.ascontiguousarray(X_all[lo:hi])
        labels = np.ascontiguousarray(y_all[lo:hi])
        halo0 = np.ascontiguousarray(X_all[part.halo_gid])
    else:
        if part_id != 0:
            raise ValueError("only partition 0 of the Chung-Lu workloads is materialised")
        n_total = c["n_total"] // scale
        n_in = n_total // c["n_comm"]
        avg_deg = min(c["avg_deg"], max(4.0, n_in / 16.0))
        part = chung_lu_partition0(seed, n_total, c["n_comm"], avg_deg, c["exponent"], c["intra"])
        rng = np.random.Generator(np.random.PCG64(seed + 100))
        X = _normal_f32(rng, (part.n_in, dims[0]))
        halo0 = _normal_f32(rng, (part.n_halo, dims[0]))
        labels = make_labels(seed + 200, part.n_in, dims[-1], c["loss"], c["label_zipf"])
    if local_order == "degree":
        order = np.argsort(-part.deg_in.astype(np.int64), kind="stable")
        part = relabel_inner(part, order)
        X = np.ascontiguousarray(X[order])
        labels = np.ascontiguousarray(labels[order])
    elif local_order != "native":
        raise ValueError("local_order must be 'native' or 'degree'")
    halo_h = [halo0]
    for l in range(1, L):
        rng = np.random.Generator(np.random.PCG64(seed + 400 + l))
        h = _normal_f32(rng, (part.n_halo, dims[l]))
        np.maximum(h, 0.0, out=h)           # post-activation-like
        halo_h.append(h)
    W = glorot_weights(seed + 300, dims)
    return Workload(cfg=cfg, name=c["name"] + ("" if scale == 1 else f"/scale{scale}")
                    + ("" if local_order == "native" else f"/{local_order}-order"),
                    part=part, dims=dims, loss_kind=c["loss"], X=X, halo_h=halo_h,
                    labels=labels, W=W, p_list=list(c["p_list"]))


def sage_weights(seed: int, dims: List[int]) -> List[np.ndarray]:
    """Weights of a GraphSAGE-mean model: per layer f32[2*d_in, d_out], the half that multiplies
    the neighbour mean on top of the half that multiplies the node's own feature."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for fan_in, fan_out in zip(dims[:-1], dims[1:]):
        lim = np.sqrt(6.0 / (2 * fan_in + fan_out))
        out.append(rng.uniform(-lim, lim, size=(2 * fan_in, fan_out)).astype(np.float32))
    return out
