"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares,
and rejects bad arguments on the host before touching a GPU (no compute calls here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bns_gcn.h")


@pytest.fixture(scope="module")
def pkg():
    import paper_2203_10983_amd as pkg
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2203_10983_amd import build
        build.build()
    return pkg


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bns_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(pkg):
    lib = pkg.load_library()
    declared = _declared_functions()
    assert len(declared) >= 10
    for name in declared:
        assert hasattr(lib, name), f"{name} is declared in bns_gcn.h but not exported"
    assert sorted(pkg.EXPORTED) == declared


def _descs(pkg, n_in=4, n_halo=0, nnz0=4, e_in=4, e_bd=0, dims=(8, 4), loss=0):
    from paper_2203_10983_amd.binding import ModelDesc, PartitionDesc
    pd = PartitionDesc(0, n_in, n_halo, nnz0, e_in, e_bd, *([0x1000] * 9))
    arr = (C.c_int32 * len(dims))(*dims)
    md = ModelDesc(len(dims) - 1, arr, loss)
    return pd, md, arr


def test_workspace_bytes_is_host_arithmetic(pkg):
    lib = pkg.load_library()
    pd, md, _ = _descs(pkg)
    small = lib.bns_workspace_bytes(C.byref(pd), C.byref(md))
    assert small > 0 and small % 256 == 0
    pd2, md2, _k = _descs(pkg, n_in=1000, n_halo=500, nnz0=9000, e_in=8000, e_bd=1000, dims=(64, 32, 8))
    assert lib.bns_workspace_bytes(C.byref(pd2), C.byref(md2)) > small
    # inconsistent entry counts, bad sizes, bad loss kind -> 0
    for bad in (dict(nnz0=5), dict(n_in=0), dict(n_halo=-1), dict(loss=2), dict(dims=(8, 0)),
                dict(dims=(2052, 8)), dict(dims=(1026, 8)), dict(dims=(8, 513))):   # widths past the kernels' reach
        pdb, mdb, _k = _descs(pkg, **bad)
        assert lib.bns_workspace_bytes(C.byref(pdb), C.byref(mdb)) == 0
    assert lib.bns_workspace_bytes(None, C.byref(md)) == 0
    for ok in ((2048, 8), (1022, 8), (8, 511)):
        pdo, mdo, _k = _descs(pkg, dims=ok)
        assert lib.bns_workspace_bytes(C.byref(pdo), C.byref(mdo)) > 0


def test_int32_overflow_is_reported(pkg):
    lib = pkg.load_library()
    pd, md, _ = _descs(pkg, n_in=10, nnz0=2**31 + 10, e_in=2**31 + 10)
    assert lib.bns_workspace_bytes(C.byref(pd), C.byref(md)) == 0
    ctx = C.c_void_p()
    assert lib.bns_create(C.byref(ctx), C.byref(pd), C.byref(md), C.c_void_p(0x10000), 1 << 20, None) == 2
    assert not ctx.value


def test_create_rejects_bad_arguments_on_the_host(pkg):
    lib = pkg.load_library()
    pd, md, _ = _descs(pkg)
    ctx = C.c_void_p()
    need = lib.bns_workspace_bytes(C.byref(pd), C.byref(md))
    assert lib.bns_create(None, C.byref(pd), C.byref(md), C.c_void_p(0x10000), need, None) == 1   # EINVAL
    assert lib.bns_create(C.byref(ctx), None, C.byref(md), C.c_void_p(0x10000), need, None) == 1
    assert lib.bns_create(C.byref(ctx), C.byref(pd), C.byref(md), None, need, None) == 3          # EWORKSPACE
    assert lib.bns_create(C.byref(ctx), C.byref(pd), C.byref(md), C.c_void_p(0x10001), need, None) == 3
    assert lib.bns_create(C.byref(ctx), C.byref(pd), C.byref(md), C.c_void_p(0x10000), need - 1, None) == 3
    assert not ctx.value
    pd.row_ptr0 = None
    assert lib.bns_create(C.byref(ctx), C.byref(pd), C.byref(md), C.c_void_p(0x10000), need, None) == 1


def test_null_context_is_rejected_everywhere(pkg):
    lib = pkg.load_library()
    assert lib.bns_sample_boundary(None, 1, 0, 0.5, None, None, None, None) == 1
    assert lib.bns_build_sampled_csr(None, None, None, None, None, None, None, None, None, None) == 1
    assert lib.bns_gcn_layer_fwd(None, 1, 0.5, None, None, None, None, None, 1, None) == 1
    assert lib.bns_gcn_layer_bwd(None, 1, 0.5, None, None, None, None, None, None, None, None, None) == 1
    assert lib.bns_train_step(None, 1, 0, 0.5, None, None, None, None, None, None, None, 0.0, None) == 1
    assert lib.bns_graph_capture(None, 1, 0, 0.5, None, None, None, None, None, None, None, 0.0, None) == 1
    assert lib.bns_graph_replay(None, 1, None) == 1
    assert lib.bns_set_dropout(None, 0.5) == 1
    assert lib.bns_layer_plan(None, 1) == -1
    assert lib.bns_cache_input_aggregate(None, None, None) == 1
    assert lib.bns_profile_enable(None, 0, 0) == 1
    assert lib.bns_last_error(None) == b"null context"
    lib.bns_destroy(None)


def test_noalloc_entry_point_checks_its_arguments_on_the_host(pkg):
    lib = pkg.load_library()
    f = lib.bns_sample_boundary_noalloc
    ptr = C.c_void_p(0x10000)
    assert f(ptr, pkg.NOALLOC_MAX_HALO + 1, 0, 1, 0, 0.5, ptr, ptr, ptr, None) == 2      # EOVERFLOW
    assert b"BNS_NOALLOC_MAX_HALO" in lib.bns_last_error(None)
    assert f(ptr, 8, 0, 1, 0, 1.5, ptr, ptr, ptr, None) == 1                             # p outside [0, 1]
    assert f(ptr, 8, 0, 1, 0, float("nan"), ptr, ptr, ptr, None) == 1
    assert f(ptr, -1, 0, 1, 0, 0.5, ptr, ptr, ptr, None) == 1
    assert f(None, 8, 0, 1, 0, 0.5, ptr, ptr, ptr, None) == 1                            # null pointers
    assert f(ptr, 8, 0, 1, 0, 0.5, ptr, ptr, None, None) == 1
    assert lib.bns_last_error(None) == b"null pointer"
    header = open(HEADER).read()
    assert int(re.search(r"#define BNS_NOALLOC_MAX_HALO (\d+)", header).group(1)) == pkg.NOALLOC_MAX_HALO


def test_binding_fails_loudly_without_gpu(pkg):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    from bns_inputs import make_workload
    w = make_workload(1)
    with pytest.raises(RuntimeError):
        pkg.Context(w.part, w.dims, w.loss_kind)
