"""Thin ctypes binding of libbns_gcn.so (argument marshalling only).

Every function here forwards to the C entry point of the same name declared in
``include/bns_gcn.h``; all arithmetic runs in the HIP kernels.  PyTorch is used
for device memory and streams only.  There is no CPU fallback: loading fails
loudly when the library has not been built.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# BNS_GCN_LIB: another build of the same library (for A/B measurements of kernel variants)
LIB_PATH = os.environ.get("BNS_GCN_LIB") or os.path.join(_HERE, "libbns_gcn.so")

NOALLOC_MAX_HALO = 1 << 22

EXPORTED = ["bns_workspace_bytes", "bns_create", "bns_destroy", "bns_last_error",
            "bns_sample_boundary", "bns_sample_boundary_noalloc", "bns_build_sampled_csr", "bns_gcn_layer_fwd",
            "bns_gcn_layer_bwd", "bns_train_step", "bns_graph_capture", "bns_graph_replay", "bns_set_dropout", "bns_layer_plan", "bns_adam_update", "bns_cache_input_aggregate", "bns_ws_view",
            "bns_profile_enable", "bns_profile_read", "bns_probe_gather", "bns_probe_mfma"]

PHASES = ["sample", "build", "gather", "spmm_fwd", "gemm_fwd", "loss", "gemm_dw", "gemm_da",
          "spmm_bwd", "sgd", "spmm_long"]

VIEW_KEPT_IDS, VIEW_REMAP, VIEW_N_KEPT, VIEW_ROW_PTR, VIEW_COL_IDX = 0, 1, 2, 3, 4
VIEW_T_ROW_PTR, VIEW_T_COL_IDX, VIEW_NNZ, VIEW_A, VIEW_H, VIEW_DZ = 5, 6, 7, 8, 9, 10
LAYER_TWO_KERNELS, LAYER_ONE_KERNEL, LAYER_UPDATE_FIRST = 0, 1, 2

_STATUS = {0: "BNS_OK", 1: "BNS_EINVAL", 2: "BNS_EOVERFLOW", 3: "BNS_EWORKSPACE", 4: "BNS_EHIP"}


class PartitionDesc(C.Structure):
    _fields_ = [("part_id", C.c_int32), ("n_in", C.c_int32), ("n_halo", C.c_int32),
                ("nnz0", C.c_int64), ("e_in", C.c_int64), ("e_bd", C.c_int64),
                ("row_ptr0", C.c_void_p), ("col0", C.c_void_p),
                ("t_in_ptr", C.c_void_p), ("t_in_col", C.c_void_p),
                ("halo_ptr", C.c_void_p), ("halo_col", C.c_void_p),
                ("halo_gid", C.c_void_p), ("deg_in", C.c_void_p), ("deg_halo", C.c_void_p)]


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("dims", C.POINTER(C.c_int32)), ("loss_kind", C.c_int32),
                ("layer_kind", C.c_int32)]


class BnsError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"{_STATUS.get(status, status)}: {message}")
        self.status = status


_lib = None


def load_library():
    """Load libbns_gcn.so and declare the signatures of include/bns_gcn.h."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; "
                          "g.build()'` (there is no CPU fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i32, u32, u64, f64 = C.c_void_p, C.c_int32, C.c_uint32, C.c_uint64, C.c_double
    L.bns_workspace_bytes.restype = C.c_size_t
    L.bns_workspace_bytes.argtypes = [C.POINTER(PartitionDesc), C.POINTER(ModelDesc)]
    L.bns_create.restype = i32
    L.bns_create.argtypes = [C.POINTER(vp), C.POINTER(PartitionDesc), C.POINTER(ModelDesc), vp,
                             C.c_size_t, vp]
    L.bns_destroy.restype = None
    L.bns_destroy.argtypes = [vp]
    L.bns_last_error.restype = C.c_char_p
    L.bns_last_error.argtypes = [vp]
    L.bns_sample_boundary.restype = i32
    L.bns_sample_boundary.argtypes = [vp, u64, u32, f64, vp, vp, vp, vp]
    L.bns_sample_boundary_noalloc.restype = i32
    L.bns_sample_boundary_noalloc.argtypes = [vp, i32, i32, u64, u32, f64, vp, vp, vp, vp]
    L.bns_build_sampled_csr.restype = i32
    L.bns_build_sampled_csr.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.bns_gcn_layer_fwd.restype = i32
    L.bns_gcn_layer_fwd.argtypes = [vp, i32, f64, vp, vp, vp, vp, vp, i32, vp]
    L.bns_gcn_layer_bwd.restype = i32
    L.bns_gcn_layer_bwd.argtypes = [vp, i32, f64, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.bns_train_step.restype = i32
    L.bns_train_step.argtypes = [vp, u64, u32, f64, vp, C.POINTER(vp), vp, C.POINTER(vp),
                                 C.POINTER(vp), C.POINTER(vp), vp, C.c_float, vp]
    L.bns_graph_capture.restype = i32
    L.bns_graph_capture.argtypes = L.bns_train_step.argtypes
    L.bns_graph_replay.restype = i32
    L.bns_graph_replay.argtypes = [vp, i32, vp]
    L.bns_layer_plan.restype = i32
    L.bns_layer_plan.argtypes = [vp, i32]
    L.bns_set_dropout.restype = i32
    L.bns_set_dropout.argtypes = [vp, C.c_double]
    L.bns_adam_update.restype = i32
    L.bns_adam_update.argtypes = [vp, vp, vp, vp, C.c_int64, C.c_float, C.c_float, C.c_float, C.c_float, i32, vp]
    L.bns_cache_input_aggregate.restype = i32
    L.bns_cache_input_aggregate.argtypes = [vp, vp, vp]
    L.bns_ws_view.restype = i32
    L.bns_ws_view.argtypes = [vp, i32, i32, C.POINTER(vp), C.POINTER(C.c_size_t)]
    L.bns_profile_enable.restype = i32
    L.bns_profile_enable.argtypes = [vp, u32, i32]
    L.bns_probe_gather.restype = i32
    L.bns_probe_gather.argtypes = [vp, C.c_int64, i32, vp, C.c_int64, i32, vp, vp]
    L.bns_probe_mfma.restype = i32
    L.bns_probe_mfma.argtypes = [i32, i32, i32, i32, vp, vp]
    L.bns_profile_read.restype = i32
    L.bns_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i32)]
    _lib = L
    return L


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr_array(tensors):
    arr = (C.c_void_p * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else t.data_ptr()
    return arr


def adam_update(W, dW, m, v, lr, beta1=0.9, beta2=0.999, eps=1e-8, t=1):
    """bns_adam_update on one weight tensor (in place)."""
    st = load_library().bns_adam_update(_ptr(W), _ptr(dW), _ptr(m), _ptr(v), W.numel(), lr, beta1, beta2,
                                        eps, t, _stream())
    if st != 0:
        raise BnsError(st, "bns_adam_update")


def sample_boundary_noalloc(halo_gid, n_halo, part_id, seed, epoch, p, kept_ids, remap, n_kept):
    """bns_sample_boundary_noalloc: needs no context and no workspace (fixed scratch inside the library)."""
    L = load_library()
    st = L.bns_sample_boundary_noalloc(_ptr(halo_gid), n_halo, part_id, seed, epoch, p, _ptr(kept_ids),
                                       _ptr(remap), _ptr(n_kept), _stream())
    if st != 0:
        raise BnsError(st, L.bns_last_error(None).decode())


def probe_gather(table, idx, per_wave, out):
    """bns_probe_gather: sums of randomly indexed rows of `table` [n_rows, d], per_wave rows per wavefront."""
    L = load_library()
    st = L.bns_probe_gather(_ptr(table), table.shape[0], table.shape[1], _ptr(idx), idx.numel(), per_wave, _ptr(out),
                            _stream())
    if st != 0:
        raise BnsError(st, "bns_probe_gather")


def probe_mfma(n_acc, waves_per_block, blocks, iters, out):
    """bns_probe_mfma: a loop of fp32 matrix instructions on n_acc accumulators per wavefront."""
    L = load_library()
    st = L.bns_probe_mfma(n_acc, waves_per_block, blocks, iters, _ptr(out), _stream())
    if st != 0:
        raise BnsError(st, "bns_probe_mfma")


class Context:
    """Owns the device copies of one partition's static arrays, the workspace and the bns_ctx."""

    def __init__(self, part, dims, loss_kind, device="cuda:0", layer_kind=0):
        L = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("the BNS-GCN library needs a GPU (there is no CPU fallback)")
        self._lib = L
        self.device = torch.device(device)
        self.n_in, self.n_halo, self.nnz0 = part.n_in, part.n_halo, part.nnz0
        self.dims = list(dims)
        self.n_layers = len(dims) - 1
        dev = self.device
        # keep the device arrays alive for the lifetime of the context
        self._static = {k: torch.from_numpy(getattr(part, k)).to(dev) for k in
                        ("row_ptr0", "col0", "t_in_ptr", "t_in_col", "halo_ptr", "halo_col",
                         "halo_gid", "deg_in", "deg_halo")}
        s = self._static
        self._pd = PartitionDesc(part.part_id, part.n_in, part.n_halo, part.nnz0, part.e_in, part.e_bd,
                                 s["row_ptr0"].data_ptr(), s["col0"].data_ptr(),
                                 s["t_in_ptr"].data_ptr(), s["t_in_col"].data_ptr(),
                                 s["halo_ptr"].data_ptr(), s["halo_col"].data_ptr(),
                                 s["halo_gid"].data_ptr(), s["deg_in"].data_ptr(),
                                 s["deg_halo"].data_ptr())
        self._dims_c = (C.c_int32 * len(dims))(*dims)
        self._md = ModelDesc(self.n_layers, self._dims_c, loss_kind, layer_kind)
        self.ws_bytes = int(L.bns_workspace_bytes(C.byref(self._pd), C.byref(self._md)))
        if self.ws_bytes == 0:
            raise BnsError(1, "invalid partition or model descriptor")
        self._ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device=dev)
        self._ctx = C.c_void_p()
        st = L.bns_create(C.byref(self._ctx), C.byref(self._pd), C.byref(self._md),
                          C.c_void_p(self._ws.data_ptr()), self.ws_bytes, _stream())
        self._check(st)

    def _check(self, st):
        if st != 0:
            msg = self._lib.bns_last_error(self._ctx).decode() if self._ctx else ""
            raise BnsError(st, msg)

    def close(self):
        if getattr(self, "_ctx", None):
            self._lib.bns_destroy(self._ctx)
            self._ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the calls of include/bns_gcn.h, same names and argument order ----------------------
    def sample_boundary(self, seed, epoch, p, kept_ids, remap, n_kept):
        self._check(self._lib.bns_sample_boundary(self._ctx, seed, epoch, p, _ptr(kept_ids), _ptr(remap),
                                                  _ptr(n_kept), _stream()))

    def build_sampled_csr(self, remap, kept_ids, n_kept, row_ptr, col_idx, t_row_ptr, t_col_idx, nnz):
        self._check(self._lib.bns_build_sampled_csr(self._ctx, _ptr(remap), _ptr(kept_ids), _ptr(n_kept),
                                                    _ptr(row_ptr), _ptr(col_idx),
                                                    _ptr(t_row_ptr), _ptr(t_col_idx), _ptr(nnz),
                                                    _stream()))

    def gcn_layer_fwd(self, layer, p, H_in, halo_h, W, A_saved, H_out, relu):
        self._check(self._lib.bns_gcn_layer_fwd(self._ctx, layer, p, _ptr(H_in), _ptr(halo_h), _ptr(W),
                                                _ptr(A_saved), _ptr(H_out), int(relu), _stream()))

    def gcn_layer_bwd(self, layer, p, dH_out, H_out, A_saved, H_in, W, dW, dH_in, dhalo):
        self._check(self._lib.bns_gcn_layer_bwd(self._ctx, layer, p, _ptr(dH_out), _ptr(H_out),
                                                _ptr(A_saved), _ptr(H_in), _ptr(W), _ptr(dW),
                                                _ptr(dH_in), _ptr(dhalo), _stream()))

    def train_step(self, seed, epoch, p, X, halo_h, labels, W, dW, dhalo, loss, lr=0.0):
        self._check(self._lib.bns_train_step(
            self._ctx, seed, epoch, p, _ptr(X), _ptr_array(halo_h), _ptr(labels), _ptr_array(W),
            _ptr_array(dW), None if dhalo is None else _ptr_array(dhalo), _ptr(loss), lr, _stream()))

    def graph_capture(self, seed, first_epoch, p, X, halo_h, labels, W, dW, dhalo, loss, lr=0.0):
        """Records one train_step on the CURRENT torch stream (must not be the default stream)."""
        self._check(self._lib.bns_graph_capture(
            self._ctx, seed, first_epoch, p, _ptr(X), _ptr_array(halo_h), _ptr(labels), _ptr_array(W),
            _ptr_array(dW), None if dhalo is None else _ptr_array(dhalo), _ptr(loss), lr, _stream()))

    def graph_replay(self, n_epochs):
        self._check(self._lib.bns_graph_replay(self._ctx, n_epochs, _stream()))

    def layer_plan(self, layer):
        """LAYER_TWO_KERNELS / LAYER_ONE_KERNEL / LAYER_UPDATE_FIRST: how train_step runs the layer."""
        return int(self._lib.bns_layer_plan(self._ctx, layer))

    def set_dropout(self, q):
        self._check(self._lib.bns_set_dropout(self._ctx, float(q)))

    def cache_input_aggregate(self, X):
        self._check(self._lib.bns_cache_input_aggregate(self._ctx, _ptr(X), _stream()))

    def profile_enable(self, phase_mask, max_records):
        self._check(self._lib.bns_profile_enable(self._ctx, phase_mask, max_records))

    def profile_read(self):
        """-> {phase name: (summed ms, number of brackets)} since the last read."""
        ms = (C.c_double * len(PHASES))()
        cnt = (C.c_int32 * len(PHASES))()
        self._check(self._lib.bns_profile_read(self._ctx, ms, cnt))
        return {name: (ms[i], cnt[i]) for i, name in enumerate(PHASES)}

    def ws_view(self, which, layer=0):
        """Device pointer and byte size of one of bns_train_step's intermediates."""
        p, n = C.c_void_p(), C.c_size_t()
        self._check(self._lib.bns_ws_view(self._ctx, which, layer, C.byref(p), C.byref(n)))
        return p.value, n.value

    def ws_tensor(self, which, layer=0, dtype=torch.int32):
        """A torch view (no copy) of an intermediate inside the workspace."""
        ptr, nbytes = self.ws_view(which, layer)
        off = ptr - self._ws.data_ptr()
        return self._ws[off:off + nbytes].view(dtype)
