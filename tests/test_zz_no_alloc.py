"""bns_sample_boundary_noalloc (the entry point for callers that cannot allocate device memory)
against bns_sample_boundary: bit-identical kept list, remap and count, on two calls in a row of
which the second has the smaller input, so that whatever the first call left in the library's
fixed scratch array is there when the second one runs."""
import numpy as np
import pytest

from bns_inputs import SAMPLING_SEED, make_workload

pytestmark = pytest.mark.gpu


def _both(pkg, torch, w, p, epoch, dev):
    P = w.part
    i32 = dict(dtype=torch.int32, device=dev)
    ctx = pkg.Context(P, w.dims, w.loss_kind, device=dev)
    want = dict(kept=torch.full((P.n_halo + 1,), -7, **i32), remap=torch.full((P.n_halo + 1,), -7, **i32),
                n=torch.full((1,), -7, **i32))
    ctx.sample_boundary(SAMPLING_SEED, epoch, p, want["kept"], want["remap"], want["n"])
    torch.cuda.synchronize()
    got = dict(kept=torch.full((P.n_halo + 1,), -7, **i32), remap=torch.full((P.n_halo + 1,), -7, **i32),
               n=torch.full((1,), -7, **i32))
    gid = torch.from_numpy(P.halo_gid).to(dev)
    pkg.sample_boundary_noalloc(gid, P.n_halo, P.part_id, SAMPLING_SEED, epoch, p, got["kept"], got["remap"],
                                got["n"])
    torch.cuda.synchronize()
    n = int(want["n"][0])
    assert int(got["n"][0]) == n
    assert torch.equal(got["kept"][:n], want["kept"][:n])
    assert torch.equal(got["remap"][:P.n_halo], want["remap"][:P.n_halo])
    assert int(got["kept"][-1]) == -7 and int(got["remap"][-1]) == -7, "guard entries must stay untouched"
    ctx.close()
    return n


def test_noalloc_sampling_equals_the_context_call_twice_in_a_row():
    import torch
    import paper_2203_10983_amd as pkg
    dev = torch.device("cuda:0")
    big = make_workload(3, scale=8)      # ~100k boundary nodes: about 50 tiles and a ragged tail
    small = make_workload(1)             # a few hundred boundary nodes: one partial tile
    assert small.part.n_halo < big.part.n_halo
    n1 = _both(pkg, torch, big, 0.5, 3, dev)
    n2 = _both(pkg, torch, small, 0.25, 4, dev)
    assert 0 < n2 < n1
    # p = 1 and p = 0 right after, on the small input
    assert _both(pkg, torch, small, 1.0, 5, dev) == small.part.n_halo
    assert _both(pkg, torch, small, 0.0, 6, dev) == 0


def test_noalloc_rejects_what_it_cannot_hold():
    import torch
    import paper_2203_10983_amd as pkg
    dev = torch.device("cuda:0")
    one = torch.zeros(8, dtype=torch.int32, device=dev)
    gid = torch.zeros(8, dtype=torch.int64, device=dev)
    with pytest.raises(pkg.BnsError) as ei:
        pkg.sample_boundary_noalloc(gid, pkg.NOALLOC_MAX_HALO + 1, 0, 1, 0, 0.5, one, one, one)
    assert ei.value.status == 2 and "BNS_NOALLOC_MAX_HALO" in str(ei.value)
    with pytest.raises(pkg.BnsError) as ei:
        pkg.sample_boundary_noalloc(gid, 8, 0, 1, 0, 1.5, one, one, one)
    assert ei.value.status == 1
    with pytest.raises(pkg.BnsError):
        pkg.sample_boundary_noalloc(gid, 8, 0, 1, 0, 0.5, None, one, one)
    # n_halo = 0 is legal: nothing kept
    n = torch.full((1,), -7, dtype=torch.int32, device=dev)
    pkg.sample_boundary_noalloc(None, 0, 0, 1, 0, 0.5, None, None, n)
    torch.cuda.synchronize()
    assert int(n[0]) == 0
    assert np.all(one.cpu().numpy() == 0)
