"""Small hand-shaped workloads for the degenerate cases of the partition step."""
import numpy as np

from bns_inputs import Workload
from bns_inputs.partition import partition_from_entries
from bns_inputs.workloads import glorot_weights


def _finish(name, part, dims, loss_kind, seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    L = len(dims) - 1
    X = rng.standard_normal((part.n_in, dims[0]), dtype=np.float32)
    halo_h = [rng.standard_normal((part.n_halo, dims[l]), dtype=np.float32) for l in range(L)]
    for h in halo_h[1:]:
        np.maximum(h, 0.0, out=h)
    if loss_kind == 0:
        labels = rng.integers(0, dims[-1], size=part.n_in).astype(np.int32)
    else:
        labels = (rng.random((part.n_in, dims[-1])) < 0.3).astype(np.uint8)
    return Workload(cfg=name, name=name, part=part, dims=list(dims), loss_kind=loss_kind, X=X,
                    halo_h=halo_h, labels=labels, W=glorot_weights(seed + 1, list(dims)), p_list=[0.5])


def no_boundary():
    """A partition with an empty boundary set (|B| = 0): a circulant graph owned entirely."""
    n = 300
    src = np.repeat(np.arange(n), 4)
    dst = (src + np.tile([-2, -1, 1, 2], n)) % n
    part = partition_from_entries(3, n, src, dst, np.zeros(0, np.int64), np.zeros(0, np.int64))
    return _finish("edge-no-boundary", part, [12, 8, 4], 0, 11)


def no_boundary_wide():
    """Empty boundary set again, large and wide enough that the first (hidden) layer, 256 -> 64, is run
    update first: its ReLU then sits in the aggregate's store and no boundary product exists."""
    n = 20000
    src = np.repeat(np.arange(n), 4)
    dst = (src + np.tile([-2, -1, 1, 2], n)) % n
    part = partition_from_entries(3, n, src, dst, np.zeros(0, np.int64), np.zeros(0, np.int64))
    return _finish("edge-no-boundary-wide", part, [256, 64, 4], 0, 17)


def narrow_first():
    """Output widths that are not multiples of 4 on a graph big enough for an update-first hidden
    layer: 512 -> 101 is run as P (H W) with the rows of H W padded to 104 floats (the aggregate
    gathers 16 bytes per lane and stores dense 101-wide rows, ReLU included), 101 -> 7 aggregates
    first at the odd width 101 and takes the padded gather (8 floats) in its backward pass.  A few
    hundred boundary nodes, each shared by several inner nodes, and one inner hub of 600 entries."""
    n = 20000
    src = np.repeat(np.arange(n), 4)
    dst = (src + np.tile([-2, -1, 1, 2], n)) % n
    hub = np.arange(1, 600)
    src = np.concatenate([src, np.zeros(599, np.int64), hub])
    dst = np.concatenate([dst, hub, np.zeros(599, np.int64)])
    src_bd = np.arange(0, n, 3)
    dst_gid = 7_000_000_000 + (src_bd * 37) % 500
    part = partition_from_entries(2, n, src, dst, src_bd, dst_gid, halo_full_degree=lambda g, inc: inc + 2)
    return _finish("edge-narrow-first", part, [512, 101, 7], 0, 19)


def star():
    """One inner hub adjacent to every inner node (a row of 3000 entries: many segments) and one
    boundary hub adjacent to every inner node (a transposed row far longer than a segment), plus
    boundary leaves; odd feature widths (scalar-load path)."""
    n = 3000
    others = np.arange(1, n)
    src_in = np.concatenate([np.zeros(n - 1, np.int64), others])
    dst_in = np.concatenate([others, np.zeros(n - 1, np.int64)])
    src_bd = np.concatenate([np.arange(n), np.arange(0, n, 7)])
    dst_gid = np.concatenate([np.full(n, 10_000_000_000), 20_000_000_000 + np.arange(0, n, 7)])
    part = partition_from_entries(1, n, src_in, dst_in, src_bd, dst_gid,
                                  halo_full_degree=lambda g, inc: inc * 3)
    return _finish("edge-star", part, [7, 5, 3], 0, 12)


def star_wide():
    """The star graph again with widths between 65 and 128 that are multiples of 4: the layers that
    aggregate and update in one kernel.  The hub row (3000 entries) is finished by the segmented
    pass and read back; 3000 rows leave a ragged last tile of 56; 72 and 100 need depth padding."""
    w = star()
    dims = [72, 100, 128, 5]
    return _finish("edge-star-wide", w.part, dims, 0, 16)


def single_node():
    """|V| = 1 with two boundary neighbours; widths 1 and 2; multi-label loss."""
    part = partition_from_entries(0, 1, np.zeros(0, np.int64), np.zeros(0, np.int64),
                                  np.zeros(2, np.int64), np.array([5, 9], np.int64))
    return _finish("edge-single-node", part, [1, 2, 2], 1, 13)


def wide_odd():
    """Widths that are multiples of 2 but not of 4 (two-float loads) and above one wavefront pass
    (602 = 5 passes of 64 lanes), with a ragged number of rows."""
    rng = np.random.Generator(np.random.PCG64(14))
    n = 517
    src = rng.integers(0, n, size=4000)
    dst = rng.integers(0, n, size=4000)
    keep = src != dst
    src, dst = src[keep], dst[keep]
    src_bd = rng.integers(0, n, size=900)
    dst_gid = 1000 + rng.integers(0, 400, size=900)
    part = partition_from_entries(2, n, np.concatenate([src, dst]), np.concatenate([dst, src]), src_bd, dst_gid,
                                  halo_full_degree=lambda g, inc: inc + 5)
    return _finish("edge-wide-odd", part, [602, 130, 66, 9], 0, 15)


def widest():
    """The widest rows the aggregate kernels take in each of their three load widths: 2048 (16-byte
    loads), 1022 (8-byte), 511 (4-byte), i.e. eight passes of 64 lanes each."""
    w = wide_odd()
    return _finish("edge-widest", w.part, [2048, 1022, 511, 3], 0, 18)


def dense_rows():
    """Rows of about 65 entries (a circulant of 60 neighbours plus boundary nodes of 20 neighbours each)
    and a 96 -> 172 first layer: long enough rows that the mean-aggregator layer aggregates and
    updates in one kernel, an output of two column tiles (128 + 44), depth padding from 96 to 128,
    and a 1500-row partition that leaves a ragged last tile of 28 rows."""
    rng = np.random.Generator(np.random.PCG64(19))
    n, nb = 1500, 300
    offs = np.concatenate([np.arange(1, 31), -np.arange(1, 31)])
    src = np.repeat(np.arange(n), offs.size)
    dst = (src + np.tile(offs, n)) % n
    src_bd = rng.integers(0, n, size=nb * 20)
    dst_gid = 5000 + np.repeat(np.arange(nb), 20)
    part = partition_from_entries(4, n, src, dst, src_bd, dst_gid, halo_full_degree=lambda g, inc: inc + 7)
    return _finish("edge-dense-rows", part, [96, 172, 128, 6], 0, 19)


def degree_ordered():
    """Workload 3 at 1/32 of its size with the inner nodes numbered by descending degree (the hub rows
    first): local ids are the partitioner's choice, and every kernel must be indifferent to it."""
    from bns_inputs import make_workload
    return make_workload(3, scale=32, local_order="degree")


EDGE = {"e-degree": degree_ordered, "e-dense": dense_rows, "e-nobd": no_boundary, "e-max": widest, "e-nobdw": no_boundary_wide, "e-narrow": narrow_first, "e-star": star, "e-starw": star_wide, "e-single": single_node, "e-wide": wide_odd}
