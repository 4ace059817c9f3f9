"""Error behaviour of the C ABI on a live context: every bad argument is turned into a status code
and a message by host-side checks, before anything is launched (so no test here can fault the GPU),
and the context keeps working afterwards."""
import ctypes as C

import numpy as np
import pytest

from bns_inputs import SAMPLING_SEED, make_workload
from oracle import bns_oracle as orc

pytestmark = pytest.mark.gpu

EINVAL, EWORKSPACE = 1, 3


@pytest.fixture(scope="module")
def live():
    import torch
    import paper_2203_10983_amd as pkg
    w = make_workload(1)
    dev = torch.device("cuda:0")
    ctx = pkg.Context(w.part, w.dims, w.loss_kind, device=dev)
    t = dict(X=torch.from_numpy(w.X).to(dev), halo_h=[torch.from_numpy(h).to(dev) for h in w.halo_h],
             labels=torch.from_numpy(w.labels).to(dev), W=[torch.from_numpy(x).to(dev) for x in w.W])
    t["dW"] = [torch.empty_like(x) for x in t["W"]]
    t["loss"] = torch.zeros(1, dtype=torch.float32, device=dev)
    yield pkg, torch, w, ctx, t
    ctx.close()


def _status(pkg, fn):
    with pytest.raises(pkg.BnsError) as e:
        fn()
    return e.value.status, str(e.value)


def test_bad_arguments_are_status_codes(live):
    pkg, torch, w, ctx, t = live
    P = w.part
    i32 = dict(dtype=torch.int32, device="cuda:0")
    kept, remap, n_kept = torch.empty(P.n_halo + 1, **i32), torch.empty(P.n_halo + 1, **i32), torch.zeros(1, **i32)
    for bad_p in (-0.1, 1.5, float("nan")):
        st, msg = _status(pkg, lambda: ctx.sample_boundary(SAMPLING_SEED, 0, bad_p, kept, remap, n_kept))
        assert st == EINVAL and "p must lie" in msg
        st, _ = _status(pkg, lambda: ctx.train_step(SAMPLING_SEED, 0, bad_p, t["X"], t["halo_h"], t["labels"], t["W"],
                                                    t["dW"], None, t["loss"]))
        assert st == EINVAL
    st, msg = _status(pkg, lambda: ctx.sample_boundary(SAMPLING_SEED, 0, 0.5, kept, remap, None))
    assert st == EINVAL and "null" in msg
    st, _ = _status(pkg, lambda: ctx.train_step(SAMPLING_SEED, 0, 0.5, None, t["halo_h"], t["labels"], t["W"],
                                                t["dW"], None, t["loss"]))
    assert st == EINVAL
    for q in (-0.01, 1.0, float("nan")):
        st, msg = _status(pkg, lambda: ctx.set_dropout(q))
        assert st == EINVAL and "dropout" in msg
    A = torch.empty(P.n_in, w.dims[0], dtype=torch.float32, device="cuda:0")
    H = torch.empty(P.n_in, w.dims[1], dtype=torch.float32, device="cuda:0")
    for layer in (0, w.n_layers + 1):
        st, msg = _status(pkg, lambda: ctx.gcn_layer_fwd(layer, 0.5, t["X"], t["halo_h"][0], t["W"][0], A, H, 1))
        assert st == EINVAL and "layer" in msg
    assert ctx.layer_plan(0) == -1 and ctx.layer_plan(w.n_layers + 1) == -1


def test_calls_out_of_order_are_refused():
    """Layer calls before any sampled CSR exists, replay before capture, capture on the null stream."""
    import torch
    import paper_2203_10983_amd as pkg
    w = make_workload(1)
    P = w.part
    dev = torch.device("cuda:0")
    ctx = pkg.Context(P, w.dims, w.loss_kind, device=dev)
    f32 = dict(dtype=torch.float32, device=dev)
    X = torch.from_numpy(w.X).to(dev)
    halo_h = [torch.from_numpy(h).to(dev) for h in w.halo_h]
    W = [torch.from_numpy(x).to(dev) for x in w.W]
    A, H = torch.empty(P.n_in, w.dims[0], **f32), torch.empty(P.n_in, w.dims[1], **f32)
    st, msg = _status(pkg, lambda: ctx.gcn_layer_fwd(1, 0.5, X, halo_h[0], W[0], A, H, 1))
    assert st == EINVAL and "bns_build_sampled_csr" in msg
    dW = torch.empty_like(W[0])
    st, msg = _status(pkg, lambda: ctx.gcn_layer_bwd(1, 0.5, H, None, A, X, W[0], dW, None, None))
    assert st == EINVAL and "bns_build_sampled_csr" in msg
    st, msg = _status(pkg, lambda: ctx.graph_replay(1))
    assert st == EINVAL and "capture" in msg
    labels = torch.from_numpy(w.labels).to(dev)
    dWs = [torch.empty_like(x) for x in W]
    loss = torch.zeros(1, **f32)
    st, msg = _status(pkg, lambda: ctx.graph_capture(SAMPLING_SEED, 0, 0.5, X, halo_h, labels, W, dWs, None, loss))
    assert st == EINVAL and "stream" in msg            # torch's current stream is the null stream here
    ctx.close()


def test_build_refuses_arrays_that_are_not_the_latest_sample(live):
    """bns_build_sampled_csr reads the keep bits the latest bns_sample_boundary left in the workspace,
    so it accepts only that call's three arrays: a replaced (re-allocated) array is refused on the
    host instead of being read."""
    pkg, torch, w, ctx, t = live
    P = w.part
    i32 = dict(dtype=torch.int32, device="cuda:0")
    new = lambda n: torch.empty(n, **i32)  # noqa: E731
    kept, remap, n_kept = new(P.n_halo + 1), new(P.n_halo + 1), torch.zeros(1, **i32)
    out = [new(P.n_in + 1), new(P.nnz0), new(P.n_in + P.n_halo + 1), new(P.nnz0), torch.zeros(1, **i32)]
    ctx.sample_boundary(SAMPLING_SEED, 0, 0.5, kept, remap, n_kept)
    ctx.build_sampled_csr(remap, kept, n_kept, *out)
    torch.cuda.synchronize()
    nnz = int(out[4][0])
    assert nnz > P.e_in
    for bad in ((remap.clone(), kept, n_kept), (remap, kept.clone(), n_kept), (remap, kept, n_kept.clone()),
                (None, kept, n_kept)):
        st, msg = _status(pkg, lambda: ctx.build_sampled_csr(*bad, *out))
        assert st == EINVAL and "latest bns_sample_boundary" in msg
    # a new sample into new arrays replaces the old ones
    kept2, remap2, n2 = new(P.n_halo + 1), new(P.n_halo + 1), torch.zeros(1, **i32)
    ctx.sample_boundary(SAMPLING_SEED, 1, 0.5, kept2, remap2, n2)
    st, _ = _status(pkg, lambda: ctx.build_sampled_csr(remap, kept, n_kept, *out))
    assert st == EINVAL
    ctx.build_sampled_csr(remap2, kept2, n2, *out)
    torch.cuda.synchronize()
    sub = orc.sample_and_build(P, SAMPLING_SEED, 1, 0.5)
    assert int(out[4][0]) == sub["col_idx"].size
    assert np.array_equal(out[1][:sub["col_idx"].size].cpu().numpy(), sub["col_idx"])


def test_failed_capture_leaves_the_phase_timers_on(live):
    """bns_graph_capture switches the event brackets off while it records; a capture that cannot
    begin (the stream is already capturing) must not leave them off."""
    pkg, torch, w, ctx, t = live
    args = (SAMPLING_SEED, 0, 0.1, t["X"], t["halo_h"], t["labels"], t["W"], t["dW"], None, t["loss"])
    ctx.profile_enable(0xFFFFFFFF, 256)
    side = torch.cuda.Stream(device="cuda:0")
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        g.capture_begin(capture_error_mode="relaxed")
        try:
            st, msg = _status(pkg, lambda: ctx.graph_capture(*args))
        finally:
            try:
                g.capture_end()
            except RuntimeError:
                pass        # the refused nested capture may have invalidated the outer one: it ends either way
    assert st == 4 and "hipStreamBeginCapture" in msg      # BNS_EHIP
    torch.cuda.synchronize()
    ctx.train_step(*args)
    torch.cuda.synchronize()
    ph = ctx.profile_read()
    assert ph["sample"][1] >= 1 and ph["spmm_fwd"][1] >= 1, "phase timers must still record after a failed capture"
    ctx.profile_enable(0, 0)
    # and a proper capture still works afterwards
    with torch.cuda.stream(side):
        ctx.graph_capture(*args)
        ctx.graph_replay(1)
    side.synchronize()


def test_short_or_misaligned_workspace_is_refused(live):
    pkg, torch, w, ctx, t = live
    lib = pkg.load_library()
    out = C.c_void_p()
    ws = torch.empty(ctx.ws_bytes, dtype=torch.uint8, device="cuda:0")
    assert lib.bns_create(C.byref(out), C.byref(ctx._pd), C.byref(ctx._md), C.c_void_p(ws.data_ptr()),
                          ctx.ws_bytes - 1, None) == EWORKSPACE
    assert lib.bns_create(C.byref(out), C.byref(ctx._pd), C.byref(ctx._md), C.c_void_p(ws.data_ptr() + 4),
                          ctx.ws_bytes, None) == EWORKSPACE
    assert not out.value


def test_context_still_works_after_errors(live):
    pkg, torch, w, ctx, t = live
    ctx.set_dropout(0.0)
    ctx.train_step(SAMPLING_SEED, 0, 0.1, t["X"], t["halo_h"], t["labels"], t["W"], t["dW"], None, t["loss"])
    torch.cuda.synchronize()
    ref = orc.step(w.part, w.loss_kind, w.X, w.halo_h, w.labels, w.W, SAMPLING_SEED, 0, 0.1)
    assert abs(float(t["loss"][0]) - ref["loss"]) <= 1e-4 * abs(ref["loss"])
    for a, b in zip(t["dW"], ref["dW"]):
        assert np.abs(a.cpu().numpy() - b).max() <= 1e-4 * max(np.abs(b).max(), 1e-6)
