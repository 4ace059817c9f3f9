// C ABI of the BNS-GCN partition step: context, workspace carving, argument checks and the
// sequencing of the kernels.  See include/bns_gcn.h for the contract of every entry point.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/bns_gcn.h"
#include "kernels.hpp"

using namespace bns;

const char *bns_noalloc_last_error();  // noalloc.hip: error text of the context-free calls on this thread

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Walks the workspace once; used both to size it and to hand out pointers.
struct Carver {
  char *base;
  size_t off = 0;
  explicit Carver(void *b) : base(static_cast<char *>(b)) {}
  template <typename T> T *take(size_t count) {
    T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off += align_up(count * sizeof(T));
    return p;
  }
};

struct Layout {
  // static, filled at set-up
  float *dis_in, *dis_halo;
  StaticSplit split;
  // scratch shared by all calls
  int32_t *tile_sums, *kept_start;
  uint64_t *ballots;
  int32_t *kpos;
  float *Hu, *Hu2, *G0, *G1, *G2, *partials, *loss_partials;  // Hu2: boundary rows at the output width
  int2 *halo_rec;  // per kept boundary node: (boundary index, weight) for the aggregates that read the rows in place
  float *inv_deg;            // 1 / (full-graph degree) of the inner nodes, for the mean aggregator
  SegPlan plan_f, plan_b;   // segmentation of the static CSR and of the transposed inner block
  int32_t *seg_tmp_a, *seg_tmp_b;
  float *spmm_partials;
  float *C0;                // cached inner part of layer 1's aggregate (n_in x d_0)
  // state of bns_train_step
  int32_t *kept_ids, *remap, *counters;
  int32_t *row_ptr, *col_idx, *t_row_ptr, *t_col_idx;
  std::vector<float *> A, H;  // index 1..L
  std::vector<float *> dZ;    // index 1..L: gradient w.r.t. the pre-activation of layer l (bns_train_step)
};

}  // namespace

// Optional instrumentation: HIP events around every kernel class of bns_train_step.
struct Profiler {
  uint32_t mask = 0;
  std::vector<hipEvent_t> start, stop;
  std::vector<int> phase;
  size_t used = 0;
  ~Profiler() {
    for (hipEvent_t e : start) (void)hipEventDestroy(e);
    for (hipEvent_t e : stop) (void)hipEventDestroy(e);
  }
};

struct bns_ctx {
  Profiler prof;
  bns_partition_desc part;
  std::vector<int32_t> dims;
  int32_t n_layers, loss_kind, layer_kind;
  Layout ws;
  // latest sample / subgraph the layer calls work on
  const int32_t *cur_kept = nullptr, *cur_remap = nullptr, *cur_n_kept = nullptr;
  const int32_t *cur_row_ptr = nullptr, *cur_col_idx = nullptr, *cur_t_row_ptr = nullptr,
                *cur_t_col_idx = nullptr;
  const float *cache_X = nullptr;  // features whose inner aggregate sits in ws.C0 (nullptr: none)
  double drop_q = 0.0;             // dropout rate on hidden activations (0: none)
  uint64_t cur_seed = 0;           // seed / epoch of the latest boundary sample: the dropout draw uses them
  uint32_t cur_epoch = 0;
  const uint32_t *cur_epoch_dev = nullptr;
  hipGraphExec_t graph_exec = nullptr;  // captured training step (bns_graph_capture)
  std::string err;
};

namespace {

// A GCN layer that shrinks its width by a quarter or more is run update first in bns_train_step:
// (P (H W)) instead of ((P H) W), so that the aggregate moves d_out instead of d_in floats per entry.
bool update_first_shape(int layer_kind, int d_in, int d_out) {
  return layer_kind == 0 && (int64_t)d_out * 4 <= (int64_t)d_in * 3;
}

// Row stride of an operand that is gathered at the output width d_out of a layer: a narrow width
// that is not a multiple of 4 is padded to one (the aggregate then reads 16 bytes per lane and
// several neighbours per load instruction) as long as the padded rows fit the buffers, which are
// sized for the input width.
int gather_stride(int d_in, int d_out) {
  const int ld = (d_out + 3) & ~3;
  return (d_out % 4 != 0 && ld < 128 && ld <= d_in) ? ld : d_out;
}

// Aggregate and update of a layer in one kernel?  The kernel's two phases (gather, product) do not
// overlap, so it pays only while the product is short beside the gather: measured on the five
// workloads, up to about 6.5 multiply-adds of the update per gathered feature element (GCN layers of
// workload 5: 4.4 and 6.0, faster in one kernel; mean-aggregator layers, whose update is twice as
// deep: workload 3 at 5.1 faster, workload 5 at 8.9 and 11.9 slower).
bool one_kernel_layer(const bns_partition_desc &part, int layer_kind, int d_in, int d_out) {
  if (layer_kind == 0) return spmm_gemm_fwd_supported(d_in);  // every GCN shape measured so far gains
  if (!spmm_gemm_fwd_concat_supported(d_in, d_out)) return false;
  const double avg_len = (double)part.nnz0 / (double)part.n_in;
  return 2.0 * d_out <= 6.5 * avg_len;
}

bool valid_desc(const bns_partition_desc *p, const bns_model_desc *m) {
  if (!p || !m || !m->dims) return false;
  if (p->n_in < 1 || p->n_halo < 0 || p->nnz0 < p->n_in || p->e_in < p->n_in || p->e_bd < 0) return false;
  if (p->e_in + p->e_bd != p->nnz0) return false;
  if (m->n_layers < 1 || (m->loss_kind != 0 && m->loss_kind != 1)) return false;
  if (m->layer_kind != 0 && m->layer_kind != 1) return false;
  for (int l = 0; l <= m->n_layers; ++l) {
    // the aggregate holds a row in at most 8 pieces of 64 lanes x (4, 2 or 1) floats
    const int d = m->dims[l], cap = d % 4 == 0 ? 2048 : d % 2 == 0 ? 1024 : 512;
    if (d < 1 || d > cap) return false;
  }
  return true;
}

bool fits_int32(const bns_partition_desc *p, const bns_model_desc *m) {
  const int64_t lim = INT32_MAX;
  if (p->nnz0 >= lim || (int64_t)p->n_in + p->n_halo + 1 >= lim) return false;
  int64_t dmax = 0;
  for (int l = 0; l <= m->n_layers; ++l) dmax = std::max<int64_t>(dmax, m->dims[l]);
  return ((int64_t)p->n_in + p->n_halo) * dmax < (int64_t)1 << 40;  // byte offsets are 64-bit
}

size_t carve(Carver &c, const bns_partition_desc *p, const bns_model_desc *m, Layout *out) {
  const size_t n_in = p->n_in, B = p->n_halo, L = m->n_layers;
  size_t d_in_max = 0, d_max = 0, part_max = 0, d_first_max = 0;
  for (size_t l = 0; l <= L; ++l) d_max = std::max<size_t>(d_max, m->dims[l]);
  for (size_t l = 0; l < L; ++l) {
    d_in_max = std::max<size_t>(d_in_max, m->dims[l]);
    const size_t mn = (size_t)m->dims[l] * m->dims[l + 1];
    part_max = std::max(part_max, mn * (size_t)splitk_splits(m->dims[l], m->dims[l + 1], p->n_in));
    if (m->layer_kind == 1)  // [A | H]^T dZ as one product of twice the height
      part_max = std::max(part_max, 2 * mn * (size_t)splitk_splits(2 * m->dims[l], m->dims[l + 1], p->n_in));
    if (update_first_shape(m->layer_kind, m->dims[l], m->dims[l + 1])) {
      d_first_max = std::max<size_t>(d_first_max, gather_stride(m->dims[l], m->dims[l + 1]));
      if (p->n_halo > 0)
        part_max = std::max(part_max, mn * (size_t)splitk_splits(m->dims[l], m->dims[l + 1], p->n_halo));
    }
  }
  Layout w;
  w.dis_in = c.take<float>(n_in);
  w.dis_halo = c.take<float>(B);
  w.split.n_inner = c.take<int32_t>(n_in);
  w.split.inner_ptr = c.take<int32_t>(n_in + 1);
  w.split.bd_ptr = c.take<int32_t>(n_in + 1);
  w.split.in_col = c.take<int32_t>(p->e_in);
  w.split.in_bdp = c.take<int32_t>(p->e_in);
  w.split.bd_b = c.take<int32_t>(p->e_bd);
  w.split.bd_row = c.take<int32_t>(p->e_bd);
  w.tile_sums = c.take<int32_t>(scan_tiles(p->nnz0 + n_in + B) + 4);
  w.kept_start = c.take<int32_t>((int64_t)B + 1);
  w.ballots = c.take<uint64_t>((B + 63) / 64 + 1);
  w.kpos = c.take<int32_t>(p->e_bd + 1);
  w.Hu = c.take<float>(B * d_in_max);
  w.Hu2 = c.take<float>(B * d_first_max);
  w.halo_rec = c.take<int2>(B + 1);
  w.G0 = c.take<float>(n_in * d_max);
  w.G1 = c.take<float>(n_in * d_max);
  w.G2 = c.take<float>(n_in * d_max);
  w.inv_deg = c.take<float>(n_in);
  w.partials = c.take<float>(part_max);
  w.loss_partials = c.take<float>(kLossBlocks);
  for (int k = 0; k < 2; ++k) {
    SegPlan &pl = k == 0 ? w.plan_f : w.plan_b;
    const int64_t nnz = k == 0 ? p->nnz0 : p->e_in;
    pl.seg_ptr = c.take<int32_t>(n_in + 1);
    pl.seg_row = c.take<int32_t>(seg_max_segments(n_in, nnz));
    pl.part_ptr = c.take<int32_t>(n_in + 1);
    pl.mrow = c.take<int32_t>(seg_max_multi(nnz));
    pl.part_row = c.take<int32_t>(seg_max_parts(nnz));
    pl.n_seg = pl.n_part = pl.n_multi = 0;
  }
  w.seg_tmp_a = c.take<int32_t>(n_in + 1);
  w.seg_tmp_b = c.take<int32_t>(n_in + 2);
  w.spmm_partials = c.take<float>((size_t)seg_max_parts(p->nnz0) * d_max);
  w.C0 = c.take<float>(n_in * (size_t)m->dims[0]);
  w.kept_ids = c.take<int32_t>(B + 1);
  w.remap = c.take<int32_t>(B + 1);
  w.counters = c.take<int32_t>(64);
  w.row_ptr = c.take<int32_t>(n_in + 1);
  w.col_idx = c.take<int32_t>(p->nnz0);
  w.t_row_ptr = c.take<int32_t>(n_in + B + 1);
  w.t_col_idx = c.take<int32_t>(p->nnz0);
  w.A.assign(L + 1, nullptr);
  w.H.assign(L + 1, nullptr);
  w.dZ.assign(L + 1, nullptr);
  for (size_t l = 1; l <= L; ++l) {
    w.A[l] = c.take<float>(n_in * (size_t)m->dims[l - 1]);
    w.H[l] = c.take<float>(n_in * (size_t)m->dims[l]);
    w.dZ[l] = c.take<float>(n_in * (size_t)m->dims[l]);
  }
  if (out) *out = w;
  return c.off;
}

bns_status fail(bns_ctx *ctx, bns_status st, const std::string &msg) {
  if (ctx) ctx->err = msg;
  return st;
}

bns_status hip_fail(bns_ctx *ctx, const char *what, hipError_t e) {
  // the runtime also keeps a failed call's code as its "last error": take it away, or the next
  // launcher's hipGetLastError() would report this failure once more as its own
  (void)hipGetLastError();
  return fail(ctx, BNS_EHIP, std::string(what) + ": " + hipGetErrorString(e));
}

#define BNS_TRY(what, expr)                                   \
  do {                                                        \
    hipError_t _e = (expr);                                   \
    if (_e != hipSuccess) return hip_fail(ctx, what, _e);     \
  } while (0)

// Brackets the kernels enqueued during its lifetime with two events (only if the phase is enabled).
struct PhaseTimer {
  Profiler *p = nullptr;
  hipStream_t s;
  size_t slot = 0;
  PhaseTimer(bns_ctx *ctx, int phase, hipStream_t stream) : s(stream) {
    Profiler &pr = ctx->prof;
    if (!((pr.mask >> phase) & 1u) || pr.used >= pr.start.size()) return;
    p = &pr;
    slot = pr.used++;
    pr.phase[slot] = phase;
    (void)hipEventRecord(pr.start[slot], s);
  }
  ~PhaseTimer() {
    if (p) (void)hipEventRecord(p->stop[slot], s);
  }
};

bool bad_p(double p) { return !(p >= 0.0 && p <= 1.0); }
float halo_scale(double p) { return p > 0.0 ? (float)(1.0 / p) : 0.f; }  // 1/p is never formed at p = 0

// Dropout of hidden layer `layer` in the current epoch (off when the rate is 0 or the layer has no ReLU).
Dropout dropout_of(const bns_ctx *ctx, int layer, bool relu) {
  Dropout d;
  if (!relu || ctx->drop_q <= 0.0) return d;
  d.threshold = (uint64_t)std::floor((1.0 - ctx->drop_q) * 4294967296.0);
  d.scale = (float)(1.0 / (1.0 - ctx->drop_q));
  d.k0 = (uint32_t)ctx->cur_seed;
  d.k1 = (uint32_t)(ctx->cur_seed >> 32) ^ 0x64726F70u;
  d.c2 = ((uint32_t)ctx->part.part_id << 8) | (uint32_t)layer;
  d.epoch = ctx->cur_epoch;
  d.epoch_dev = ctx->cur_epoch_dev;
  return d;
}
// Slope of a surviving hidden unit: 1/(1-q) under dropout, else 1.
float mask_scale_of(const bns_ctx *ctx) {
  return ctx->drop_q > 0.0 ? (float)(1.0 / (1.0 - ctx->drop_q)) : 1.f;
}

// update_first: H_out = act(P [H_in W ; Hu W]) instead of act((P [H_in ; Hu]) W); A_saved then
// receives H_in W (the aggregate of the inputs is never formed).
// How bns_train_step runs the forward pass of `layer` when its first-layer input is X.
int layer_plan(const bns_ctx *ctx, int layer, const float *X) {
  const int d_in = ctx->dims[layer - 1], d_out = ctx->dims[layer];
  const bool cached = layer == 1 && ctx->cache_X != nullptr && ctx->cache_X == X;
  // worth its extra launches only when the aggregate is big: at least 2^24 fewer floats gathered
  const bool big = (int64_t)ctx->part.nnz0 * (d_in - d_out) >= ((int64_t)1 << 24);
  if (!cached && big && update_first_shape(ctx->layer_kind, d_in, d_out)) return BNS_LAYER_UPDATE_FIRST;
  if (one_kernel_layer(ctx->part, ctx->layer_kind, d_in, d_out)) return BNS_LAYER_ONE_KERNEL;
  return BNS_LAYER_TWO_KERNELS;
}

// update_first: H_out = act(P [H_in W ; Hu W]) instead of act((P [H_in ; Hu]) W); A_saved then
// receives H_in W (the aggregate of the inputs is never formed).
bns_status layer_fwd_impl(bns_ctx *ctx, int layer, double p, const float *H_in, const float *halo_h,
                          const float *W, float *A_saved, float *H_out, bool relu, bool update_first,
                          hipStream_t s) {
  const int n_in = ctx->part.n_in, B = ctx->part.n_halo;
  const int d_in = ctx->dims[layer - 1], d_out = ctx->dims[layer];
  const bool sage = ctx->layer_kind == 1;
  if (update_first) {
    const int ld = gather_stride(d_in, d_out);  // row stride of H W and H_U W
    {
      PhaseTimer t(ctx, BNS_PHASE_GATHER, s);
      BNS_TRY("halo_gather", halo_gather(halo_h, ctx->cur_kept, ctx->cur_n_kept, B, ctx->ws.dis_halo, halo_scale(p),
                                         d_in, ctx->ws.Hu, s));
    }
    {
      PhaseTimer t(ctx, BNS_PHASE_GEMM_FWD, s);
      BNS_TRY("gemm_nn(inner)", gemm_nn(n_in, d_out, d_in, H_in, W, A_saved, false, false, Dropout{}, nullptr, s, ld));
      if (B > 0)
        BNS_TRY("gemm_nn(boundary)", gemm_nn(B, d_out, d_in, ctx->ws.Hu, W, ctx->ws.Hu2, false, false, Dropout{},
                                             ctx->cur_n_kept, s, ld));
    }
    PhaseTimer t(ctx, BNS_PHASE_SPMM_FWD, s);
    BNS_TRY("spmm_fwd", spmm_fwd(ctx->ws.plan_f, n_in, ld, ctx->cur_row_ptr, ctx->cur_col_idx, ctx->ws.dis_in,
                                 ctx->ws.dis_in, A_saved, ctx->ws.Hu2, ctx->ws.spmm_partials, H_out, SpmmRowPart{},
                                 false, relu, s, d_out));
    BNS_TRY("dropout_inplace", dropout_inplace(n_in, d_out, H_out, dropout_of(ctx, layer, relu), s));
    return BNS_OK;
  }
  {
    // The aggregate reads the kept boundary rows where the caller holds them; it only needs, per
    // kept node, the row index and the weight S_uu = 1/p (GCN: times d~^-1/2).  A gathered, scaled
    // copy of the rows would cost a read and a write of every kept row on top of the same reads.
    PhaseTimer t(ctx, BNS_PHASE_GATHER, s);
    BNS_TRY("halo_records", halo_records(ctx->cur_kept, ctx->cur_n_kept, B, sage ? nullptr : ctx->ws.dis_halo,
                                         halo_scale(p), ctx->ws.halo_rec, s));
  }
  SpmmRowPart part;
  part.halo_rec = B > 0 ? ctx->ws.halo_rec : nullptr;
  part.skip_self = sage;
  if (layer == 1 && ctx->cache_X != nullptr && ctx->cache_X == H_in) {
    // inner neighbours are the same every epoch: their sum is cached, only the kept boundary
    // tail of each row is aggregated now
    part.row_skip = ctx->ws.split.n_inner;
    part.init = ctx->ws.C0;
  }
  const float *w_col = sage ? nullptr : ctx->ws.dis_in;
  const float *row_scale = sage ? ctx->ws.inv_deg : ctx->ws.dis_in;
  if (one_kernel_layer(ctx->part, ctx->layer_kind, d_in, d_out)) {
    // aggregate and update in one kernel; the rows cut into several segments are finished first
    {
      PhaseTimer t(ctx, BNS_PHASE_SPMM_LONG, s);
      BNS_TRY("spmm_fwd(long rows)", spmm_fwd(ctx->ws.plan_f, n_in, d_in, ctx->cur_row_ptr, ctx->cur_col_idx, w_col,
                                              row_scale, H_in, halo_h, ctx->ws.spmm_partials, A_saved, part,
                                              true, false, s));
    }
    PhaseTimer t(ctx, BNS_PHASE_SPMM_FWD, s);
    BNS_TRY("spmm_gemm_fwd", spmm_gemm_fwd(ctx->ws.plan_f, n_in, d_in, d_out, ctx->cur_row_ptr, ctx->cur_col_idx,
                                           w_col, row_scale, H_in, halo_h, ctx->ws.spmm_partials, A_saved,
                                           part, W, H_out, relu, dropout_of(ctx, layer, relu), s, sage));
    return BNS_OK;
  }
  {
    PhaseTimer t(ctx, BNS_PHASE_SPMM_FWD, s);
    BNS_TRY("spmm_fwd", spmm_fwd(ctx->ws.plan_f, n_in, d_in, ctx->cur_row_ptr, ctx->cur_col_idx, w_col, row_scale,
                                 H_in, halo_h, ctx->ws.spmm_partials, A_saved, part, false, false, s));
  }
  {
    PhaseTimer t(ctx, BNS_PHASE_GEMM_FWD, s);
    if (!sage) {
      BNS_TRY("gemm_nn", gemm_nn(n_in, d_out, d_in, A_saved, W, H_out, relu, false, dropout_of(ctx, layer, relu),
                                 nullptr, s));
    } else if (d_in % 16 == 0) {  // [z | h] [W_n ; W_s] in one product
      BNS_TRY("gemm_nn_concat", gemm_nn_concat(n_in, d_out, d_in, A_saved, H_in, W, H_out, relu,
                                               dropout_of(ctx, layer, relu), s));
    } else {  // [z | h] [W_n ; W_s] = z W_n + h W_s
      BNS_TRY("gemm_nn(nbr)", gemm_nn(n_in, d_out, d_in, A_saved, W, H_out, false, false, Dropout{}, nullptr, s));
      BNS_TRY("gemm_nn(self)", gemm_nn(n_in, d_out, d_in, H_in, W + (size_t)d_in * d_out, H_out, relu, true,
                                       dropout_of(ctx, layer, relu), nullptr, s));
    }
  }
  return BNS_OK;
}

// dZ is the gradient of the layer's pre-activation.  mask_src (nullable): activations of the
// layer below; when given, dH_in receives the masked gradient (= dZ of the layer below).
// H_in is needed by the mean-aggregator layer only (its self half of the weight gradient).
// halo_first (nullable): the boundary features of an update-first layer (A_saved does not hold
// the aggregate then); the weight gradient is [H_in ; Hu]^T (P^T dZ) instead of A^T dZ.
bns_status layer_bwd_impl(bns_ctx *ctx, int layer, double p, const float *dZ, const float *A_saved,
                          const float *H_in, const float *W, float *dW, float *dH_in, float *dhalo,
                          const float *mask_src, bool update_first, const float *halo_first, hipStream_t s) {
  const int n_in = ctx->part.n_in, B = ctx->part.n_halo;
  const int d_in = ctx->dims[layer - 1], d_out = ctx->dims[layer];
  if (update_first) {
    float *G_in = ctx->ws.G1, *G_halo = B > 0 ? ctx->ws.Hu2 : nullptr;
    {  // G = P^T dZ at the output width, inner rows and kept boundary rows
      PhaseTimer t(ctx, BNS_PHASE_SPMM_BWD, s);
      const int ld = gather_stride(d_in, d_out);
      const float *dZ_g = dZ;
      if (ld != d_out) {  // the gathered operand with padded rows
        BNS_TRY("pad_rows", pad_rows(n_in, d_out, ld, dZ, ctx->ws.G2, s));
        dZ_g = ctx->ws.G2;
      }
      BNS_TRY("spmm_bwd", spmm_bwd(ctx->ws.plan_b, n_in, B, ld, ctx->cur_t_row_ptr, ctx->cur_t_col_idx,
                                   ctx->cur_kept, ctx->cur_n_kept, ctx->ws.dis_in, ctx->ws.dis_in, ctx->ws.dis_halo,
                                   halo_scale(p), dZ_g, nullptr, nullptr, false, ctx->ws.spmm_partials, G_in, G_halo,
                                   s, d_out));
    }
    if (B > 0) {  // the kept boundary features once more, unscaled: G_halo carries the 1/p and degree factors
      PhaseTimer t(ctx, BNS_PHASE_GATHER, s);
      BNS_TRY("halo_gather", halo_gather(halo_first, ctx->cur_kept, ctx->cur_n_kept, B, nullptr, 1.f, d_in,
                                         ctx->ws.Hu, s));
    }
    {
      PhaseTimer t(ctx, BNS_PHASE_GEMM_DW, s);
      BNS_TRY("gemm_tn_splitk(inner)", gemm_tn_splitk(d_in, d_out, n_in, H_in, G_in, dW, ctx->ws.partials, false,
                                                      nullptr, s));
      if (B > 0)
        BNS_TRY("gemm_tn_splitk(boundary)", gemm_tn_splitk(d_in, d_out, B, ctx->ws.Hu, G_halo, dW, ctx->ws.partials,
                                                           true, ctx->cur_n_kept, s));
    }
    if (dH_in) {
      PhaseTimer t(ctx, BNS_PHASE_GEMM_DA, s);
      const float ms1 = mask_src ? mask_scale_of(ctx) : 1.f;
      BNS_TRY("gemm_nt", gemm_nt(n_in, d_in, d_out, G_in, W, dH_in, mask_src, ms1, nullptr, s));
      if (dhalo && B > 0)
        BNS_TRY("gemm_nt(halo)", gemm_nt(B, d_in, d_out, G_halo, W, dhalo, nullptr, 1.f, ctx->cur_n_kept, s));
    }
    return BNS_OK;
  }
  // slope of the surviving hidden units of the layer below (dropout); it multiplies the masked
  // gradient only.  Where the transposed aggregate applies the mask, the factor rides on its
  // input (the product with W^T) and is divided out of the boundary rows, which are not masked.
  const float ms = mask_src ? mask_scale_of(ctx) : 1.f;
  if (ctx->layer_kind == 1) {
    const size_t half = (size_t)d_in * d_out;
    {
      PhaseTimer t(ctx, BNS_PHASE_GEMM_DW, s);
      if (gemm_tn_concat_supported(d_in)) {  // [A | H]^T dZ in one product: dZ is read once
        BNS_TRY("gemm_tn_splitk_concat", gemm_tn_splitk_concat(d_in, d_out, n_in, A_saved, H_in, dZ, dW,
                                                               ctx->ws.partials, false, nullptr, s));
      } else {
        BNS_TRY("gemm_tn_splitk(nbr)", gemm_tn_splitk(d_in, d_out, n_in, A_saved, dZ, dW, ctx->ws.partials, false,
                                                      nullptr, s));
        BNS_TRY("gemm_tn_splitk(self)", gemm_tn_splitk(d_in, d_out, n_in, H_in, dZ, dW + half, ctx->ws.partials, false,
                                                       nullptr, s));
      }
    }
    if (dH_in) {
      {
        PhaseTimer t(ctx, BNS_PHASE_GEMM_DA, s);
        if (gemm_nt_pair_supported(d_in)) {  // dZ [W_n ; W_s]^T in one product, split into the two halves
          BNS_TRY("gemm_nt_pair", gemm_nt_pair(n_in, d_in, d_out, dZ, W, ctx->ws.G1, ctx->ws.G2, ms, s));
        } else {
          BNS_TRY("gemm_nt(nbr)", gemm_nt(n_in, d_in, d_out, dZ, W, ctx->ws.G1, nullptr, ms, nullptr, s));
          BNS_TRY("gemm_nt(self)", gemm_nt(n_in, d_in, d_out, dZ, W + half, ctx->ws.G2, nullptr, ms, nullptr, s));
        }
      }
      // dH_in = (gradient through the node's own feature) + mean^T (gradient of the neighbour mean)
      PhaseTimer t(ctx, BNS_PHASE_SPMM_BWD, s);
      BNS_TRY("spmm_bwd", spmm_bwd(ctx->ws.plan_b, n_in, B, d_in, ctx->cur_t_row_ptr, ctx->cur_t_col_idx,
                                   ctx->cur_kept, ctx->cur_n_kept, ctx->ws.inv_deg, nullptr, nullptr,
                                   halo_scale(p) / ms, ctx->ws.G1, mask_src, ctx->ws.G2, true,
                                   ctx->ws.spmm_partials, dH_in, dhalo, s));
    }
    return BNS_OK;
  }
  {
    PhaseTimer t(ctx, BNS_PHASE_GEMM_DW, s);
    BNS_TRY("gemm_tn_splitk", gemm_tn_splitk(d_in, d_out, n_in, A_saved, dZ, dW, ctx->ws.partials, false, nullptr, s));
  }
  if (dH_in && d_out < d_in) {
    // (P^T dZ) W^T instead of P^T (dZ W^T): the transposed aggregate runs at the narrower width
    float *G_in = ctx->ws.G1, *G_halo = dhalo ? ctx->ws.Hu : nullptr;
    {
      PhaseTimer t(ctx, BNS_PHASE_SPMM_BWD, s);
      const int ld = gather_stride(d_in, d_out);
      const float *dZ_g = dZ;
      if (ld != d_out) {  // the gathered operand with padded rows
        BNS_TRY("pad_rows", pad_rows(n_in, d_out, ld, dZ, ctx->ws.G2, s));
        dZ_g = ctx->ws.G2;
      }
      BNS_TRY("spmm_bwd", spmm_bwd(ctx->ws.plan_b, n_in, B, ld, ctx->cur_t_row_ptr, ctx->cur_t_col_idx,
                                   ctx->cur_kept, ctx->cur_n_kept, ctx->ws.dis_in, ctx->ws.dis_in,
                                   ctx->ws.dis_halo, halo_scale(p), dZ_g, nullptr, nullptr, false,
                                   ctx->ws.spmm_partials, G_in, G_halo, s, d_out));
    }
    PhaseTimer t(ctx, BNS_PHASE_GEMM_DA, s);
    BNS_TRY("gemm_nt", gemm_nt(n_in, d_in, d_out, G_in, W, dH_in, mask_src, ms, nullptr, s));
    if (G_halo && B > 0)
      BNS_TRY("gemm_nt(halo)", gemm_nt(B, d_in, d_out, G_halo, W, dhalo, nullptr, 1.f, ctx->cur_n_kept, s));
  } else if (dH_in) {
    {
      PhaseTimer t(ctx, BNS_PHASE_GEMM_DA, s);
      BNS_TRY("gemm_nt", gemm_nt(n_in, d_in, d_out, dZ, W, ctx->ws.G1, nullptr, ms, nullptr, s));
    }
    PhaseTimer t(ctx, BNS_PHASE_SPMM_BWD, s);
    BNS_TRY("spmm_bwd", spmm_bwd(ctx->ws.plan_b, n_in, B, d_in, ctx->cur_t_row_ptr, ctx->cur_t_col_idx,
                                 ctx->cur_kept, ctx->cur_n_kept, ctx->ws.dis_in, ctx->ws.dis_in,
                                 ctx->ws.dis_halo, halo_scale(p) / ms, ctx->ws.G1, mask_src, nullptr, false,
                                 ctx->ws.spmm_partials, dH_in, dhalo, s));
  }
  return BNS_OK;
}

bns_status sample_impl(bns_ctx *ctx, uint64_t seed, uint32_t epoch, const uint32_t *epoch_dev, double p,
                       int32_t *kept_ids, int32_t *remap, int32_t *n_kept, hipStream_t s) {
  const uint64_t threshold = (uint64_t)std::floor(p * 4294967296.0);
  PhaseTimer t(ctx, BNS_PHASE_SAMPLE, s);
  BNS_TRY("sample_boundary",
          sample_boundary(ctx->part.halo_gid, ctx->part.n_halo, seed, epoch, epoch_dev, (uint32_t)ctx->part.part_id,
                          threshold, ctx->ws.ballots, ctx->ws.tile_sums, kept_ids, remap, n_kept, ctx->part.halo_ptr,
                          (int32_t)ctx->part.e_in, ctx->ws.kept_start, s));
  ctx->cur_kept = kept_ids;
  ctx->cur_remap = remap;
  ctx->cur_n_kept = n_kept;
  ctx->cur_seed = seed;
  ctx->cur_epoch = epoch;
  ctx->cur_epoch_dev = epoch_dev;
  return BNS_OK;
}

bns_status build_impl(bns_ctx *ctx, int32_t *row_ptr, int32_t *col_idx, int32_t *t_row_ptr,
                      int32_t *t_col_idx, int32_t *nnz, hipStream_t s) {
  const bns_partition_desc &P = ctx->part;
  PhaseTimer t(ctx, BNS_PHASE_BUILD, s);
  BNS_TRY("build_sampled_csr",
          build_sampled_csr(P.n_in, P.e_in, P.e_bd, ctx->ws.split, ctx->ws.ballots, ctx->cur_remap, ctx->ws.kpos,
                            ctx->ws.tile_sums, row_ptr, col_idx, nnz, s));
  BNS_TRY("build_transposed_csr",
          build_transposed_csr(P.n_in, P.n_halo, P.e_in, P.t_in_ptr, P.t_in_col, P.halo_ptr, P.halo_col,
                               ctx->cur_kept, ctx->cur_n_kept, ctx->ws.kept_start,
                               t_row_ptr, t_col_idx,
                               // the workspace arrays hold the static rows since bns_create
                               !(t_row_ptr == ctx->ws.t_row_ptr && t_col_idx == ctx->ws.t_col_idx), true, s));
  ctx->cur_row_ptr = row_ptr;
  ctx->cur_col_idx = col_idx;
  ctx->cur_t_row_ptr = t_row_ptr;
  ctx->cur_t_col_idx = t_col_idx;
  return BNS_OK;
}

// Selection step + subgraph step of a training step, into the workspace arrays: one launch for a
// small partition (timed as the sample phase), else the two calls above.
bns_status sample_and_build_impl(bns_ctx *ctx, uint64_t seed, uint32_t epoch, const uint32_t *epoch_dev, double p,
                                 hipStream_t s) {
  Layout &w = ctx->ws;
  const bns_partition_desc &P = ctx->part;
  if (!sample_build_small_fits(P.n_in, P.n_halo, P.e_in, P.e_bd)) {
    const bns_status st = sample_impl(ctx, seed, epoch, epoch_dev, p, w.kept_ids, w.remap, w.counters, s);
    if (st != BNS_OK) return st;
    return build_impl(ctx, w.row_ptr, w.col_idx, w.t_row_ptr, w.t_col_idx, w.counters + 1, s);
  }
  const uint64_t threshold = (uint64_t)std::floor(p * 4294967296.0);
  PhaseTimer t(ctx, BNS_PHASE_SAMPLE, s);
  BNS_TRY("sample_build_small",
          sample_build_small(P.halo_gid, P.n_halo, seed, epoch, epoch_dev, (uint32_t)P.part_id, threshold, w.ballots,
                             w.kept_ids, w.remap, w.counters, w.kept_start, P.n_in, P.e_in, P.e_bd, w.split, w.kpos,
                             w.row_ptr, w.col_idx, w.counters + 1, P.halo_ptr, P.halo_col, w.t_row_ptr, w.t_col_idx,
                             s));
  ctx->cur_kept = w.kept_ids;
  ctx->cur_remap = w.remap;
  ctx->cur_n_kept = w.counters;
  ctx->cur_seed = seed;
  ctx->cur_epoch = epoch;
  ctx->cur_epoch_dev = epoch_dev;
  ctx->cur_row_ptr = w.row_ptr;
  ctx->cur_col_idx = w.col_idx;
  ctx->cur_t_row_ptr = w.t_row_ptr;
  ctx->cur_t_col_idx = w.t_col_idx;
  return BNS_OK;
}

}  // namespace

extern "C" {

size_t bns_workspace_bytes(const bns_partition_desc *part, const bns_model_desc *model) {
  if (!valid_desc(part, model) || !fits_int32(part, model)) return 0;
  Carver c(nullptr);
  return carve(c, part, model, nullptr);
}

bns_status bns_create(bns_ctx **out, const bns_partition_desc *part, const bns_model_desc *model,
                      void *dev_ws, size_t ws_bytes, void *stream) {
  if (!out) return BNS_EINVAL;
  *out = nullptr;
  if (!valid_desc(part, model)) return BNS_EINVAL;
  if (!fits_int32(part, model)) return BNS_EOVERFLOW;
  if (!part->row_ptr0 || !part->col0 || !part->t_in_ptr || !part->t_in_col || !part->deg_in) return BNS_EINVAL;
  if (part->n_halo > 0 && (!part->halo_ptr || !part->halo_col || !part->halo_gid || !part->deg_halo))
    return BNS_EINVAL;
  if (!dev_ws || ((uintptr_t)dev_ws % kAlign) != 0) return BNS_EWORKSPACE;
  bns_ctx *ctx = new (std::nothrow) bns_ctx();
  if (!ctx) return BNS_EINVAL;
  ctx->part = *part;
  ctx->n_layers = model->n_layers;
  ctx->loss_kind = model->loss_kind;
  ctx->layer_kind = model->layer_kind;
  ctx->dims.assign(model->dims, model->dims + model->n_layers + 1);
  Carver c(dev_ws);
  const size_t need = carve(c, part, model, &ctx->ws);
  if (need > ws_bytes) { delete ctx; return BNS_EWORKSPACE; }
  *out = ctx;  // handed out even if set-up fails, so that the caller can read the error text
  hipStream_t s = static_cast<hipStream_t>(stream);
  BNS_TRY("degree_rsqrt(in)", degree_rsqrt(part->deg_in, part->n_in, ctx->ws.dis_in, s));
  BNS_TRY("degree_inverse", degree_inverse(part->deg_in, part->n_in, ctx->ws.inv_deg, s));
  BNS_TRY("degree_rsqrt(halo)", degree_rsqrt(part->deg_halo, part->n_halo, ctx->ws.dis_halo, s));
  BNS_TRY("build_static_split", build_static_split(part->n_in, part->row_ptr0, part->col0, ctx->ws.split,
                                                   ctx->ws.tile_sums, s));
  BNS_TRY("build_seg_plan(fwd)", build_seg_plan(part->n_in, part->nnz0, part->row_ptr0, &ctx->ws.plan_f, ctx->ws.seg_tmp_a,
                                                 ctx->ws.seg_tmp_b, ctx->ws.tile_sums, s));
  BNS_TRY("build_seg_plan(bwd)", build_seg_plan(part->n_in, part->e_in, part->t_in_ptr, &ctx->ws.plan_b, ctx->ws.seg_tmp_a,
                                                 ctx->ws.seg_tmp_b, ctx->ws.tile_sums, s));
  // the rows of the inner nodes in the workspace's transposed CSR are the same in every epoch
  BNS_TRY("build_transposed_csr(static rows)",
          build_transposed_csr(part->n_in, part->n_halo, part->e_in, part->t_in_ptr, part->t_in_col, part->halo_ptr,
                               part->halo_col, nullptr, nullptr, ctx->ws.kept_start, ctx->ws.t_row_ptr,
                               ctx->ws.t_col_idx, true, false, s));
  BNS_TRY("set-up sync", hipStreamSynchronize(s));
  return BNS_OK;
}

void bns_destroy(bns_ctx *ctx) {
  if (ctx && ctx->graph_exec) (void)hipGraphExecDestroy(ctx->graph_exec);
  delete ctx;
}

const char *bns_last_error(const bns_ctx *ctx) {
  if (ctx) return ctx->err.c_str();
  const char *e = bns_noalloc_last_error();
  return e[0] ? e : "null context";
}

bns_status bns_sample_boundary(bns_ctx *ctx, uint64_t seed, uint32_t epoch, double p, int32_t *kept_ids,
                               int32_t *remap, int32_t *n_kept, void *stream) {
  if (!ctx) return BNS_EINVAL;
  if (bad_p(p)) return fail(ctx, BNS_EINVAL, "p must lie in [0, 1]");
  if (!n_kept || (ctx->part.n_halo > 0 && (!kept_ids || !remap)))
    return fail(ctx, BNS_EINVAL, "null output pointer");
  return sample_impl(ctx, seed, epoch, nullptr, p, kept_ids, remap, n_kept, static_cast<hipStream_t>(stream));
}

bns_status bns_build_sampled_csr(bns_ctx *ctx, const int32_t *remap, const int32_t *kept_ids, const int32_t *n_kept,
                                 int32_t *row_ptr, int32_t *col_idx, int32_t *t_row_ptr, int32_t *t_col_idx,
                                 int32_t *nnz, void *stream) {
  if (!ctx) return BNS_EINVAL;
  if (!row_ptr || !col_idx || !t_row_ptr || !t_col_idx || !nnz)
    return fail(ctx, BNS_EINVAL, "null output pointer");
  if (!ctx->cur_n_kept) return fail(ctx, BNS_EINVAL, "bns_sample_boundary has not been called");
  // the keep bits of the latest sample sit in the workspace: the three arrays must be that sample's
  if (remap != ctx->cur_remap || kept_ids != ctx->cur_kept || n_kept != ctx->cur_n_kept)
    return fail(ctx, BNS_EINVAL, "remap / kept_ids / n_kept are not the outputs of the latest bns_sample_boundary");
  return build_impl(ctx, row_ptr, col_idx, t_row_ptr, t_col_idx, nnz, static_cast<hipStream_t>(stream));
}

bns_status bns_gcn_layer_fwd(bns_ctx *ctx, int32_t layer, double p, const float *H_in, const float *halo_h,
                             const float *W, float *A_saved, float *H_out, int32_t relu, void *stream) {
  if (!ctx) return BNS_EINVAL;
  if (layer < 1 || layer > ctx->n_layers) return fail(ctx, BNS_EINVAL, "layer out of range");
  if (bad_p(p)) return fail(ctx, BNS_EINVAL, "p must lie in [0, 1]");
  if (!H_in || !W || !A_saved || !H_out || (ctx->part.n_halo > 0 && !halo_h))
    return fail(ctx, BNS_EINVAL, "null pointer");
  if (!ctx->cur_row_ptr) return fail(ctx, BNS_EINVAL, "bns_build_sampled_csr has not been called");
  return layer_fwd_impl(ctx, layer, p, H_in, halo_h, W, A_saved, H_out, relu != 0, false,
                        static_cast<hipStream_t>(stream));
}

bns_status bns_gcn_layer_bwd(bns_ctx *ctx, int32_t layer, double p, const float *dH_out, const float *H_out,
                             const float *A_saved, const float *H_in, const float *W, float *dW, float *dH_in,
                             float *dhalo, void *stream) {
  if (!ctx) return BNS_EINVAL;
  if (layer < 1 || layer > ctx->n_layers) return fail(ctx, BNS_EINVAL, "layer out of range");
  if (bad_p(p)) return fail(ctx, BNS_EINVAL, "p must lie in [0, 1]");
  if (!dH_out || !A_saved || !W || !dW) return fail(ctx, BNS_EINVAL, "null pointer");
  if (ctx->layer_kind == 1 && !H_in) return fail(ctx, BNS_EINVAL, "the mean-aggregator layer needs H_in");
  if (!dH_in && dhalo) return fail(ctx, BNS_EINVAL, "dhalo needs dH_in");
  if (!ctx->cur_t_row_ptr) return fail(ctx, BNS_EINVAL, "bns_build_sampled_csr has not been called");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const float *dZ = dH_out;
  if (H_out) {
    const int64_t n = (int64_t)ctx->part.n_in * ctx->dims[layer];
    BNS_TRY("relu_mask", relu_mask(n, dH_out, H_out, mask_scale_of(ctx), ctx->ws.G0, s));
    dZ = ctx->ws.G0;
  }
  return layer_bwd_impl(ctx, layer, p, dZ, A_saved, H_in, W, dW, dH_in, dhalo, nullptr, false, nullptr, s);
}

static bns_status train_step_impl(bns_ctx *ctx, uint64_t seed, uint32_t epoch, const uint32_t *epoch_dev, double p,
                                  const float *X, const float *const *halo_h, const void *labels,
                                  float *const *W, float *const *dW, float *const *dhalo, float *loss, float lr,
                                  void *stream) {
  if (!ctx) return BNS_EINVAL;
  if (bad_p(p)) return fail(ctx, BNS_EINVAL, "p must lie in [0, 1]");
  if (!X || !labels || !W || !dW || !loss || (ctx->part.n_halo > 0 && !halo_h))
    return fail(ctx, BNS_EINVAL, "null pointer");
  const int L = ctx->n_layers, n_in = ctx->part.n_in;
  for (int l = 0; l < L; ++l)
    if (!W[l] || !dW[l] || (ctx->part.n_halo > 0 && !halo_h[l])) return fail(ctx, BNS_EINVAL, "null layer pointer");
  hipStream_t s = static_cast<hipStream_t>(stream);
  Layout &w = ctx->ws;

  bns_status st = sample_and_build_impl(ctx, seed, epoch, epoch_dev, p, s);
  if (st != BNS_OK) return st;

  const float *H_prev = X;
  for (int l = 1; l <= L; ++l) {
    st = layer_fwd_impl(ctx, l, p, H_prev, ctx->part.n_halo > 0 ? halo_h[l - 1] : nullptr, W[l - 1], w.A[l],
                        w.H[l], l < L, layer_plan(ctx, l, X) == BNS_LAYER_UPDATE_FIRST, s);
    if (st != BNS_OK) return st;
    H_prev = w.H[l];
  }

  const int C = ctx->dims[L];
  {
    PhaseTimer t(ctx, BNS_PHASE_LOSS, s);
    if (ctx->loss_kind == 0)
      BNS_TRY("loss_softmax_ce", loss_softmax_ce(n_in, C, w.H[L], static_cast<const int32_t *>(labels), w.dZ[L],
                                                 w.loss_partials, loss, s));
    else
      BNS_TRY("loss_sigmoid_bce", loss_sigmoid_bce(n_in, C, w.H[L], static_cast<const uint8_t *>(labels), w.dZ[L],
                                                   w.loss_partials, loss, s));
  }

  // dZ[l] is the gradient w.r.t. the pre-activation of layer l; the backward pass of layer l writes
  // dZ[l-1], already masked by the activations of the layer below.  Every layer keeps its own buffer
  // (BNS_VIEW_DZ), so that each stage of the backward pass can be inspected with its exact inputs.
  for (int l = L; l >= 1; --l) {
    float *dh = (dhalo && l > 1) ? dhalo[l - 1] : nullptr;
    st = layer_bwd_impl(ctx, l, p, w.dZ[l], w.A[l], l > 1 ? w.H[l - 1] : X, W[l - 1], dW[l - 1],
                        l > 1 ? w.dZ[l - 1] : nullptr, dh,
                        l > 1 ? w.H[l - 1] : nullptr, layer_plan(ctx, l, X) == BNS_LAYER_UPDATE_FIRST,
                        ctx->part.n_halo > 0 ? halo_h[l - 1] : nullptr, s);
    if (st != BNS_OK) return st;
  }
  if (lr > 0.f) {
    PhaseTimer t(ctx, BNS_PHASE_SGD, s);
    for (int l = 0; l < L; ++l)
      BNS_TRY("sgd_update", sgd_update((int64_t)(ctx->layer_kind == 1 ? 2 : 1) * ctx->dims[l] * ctx->dims[l + 1], W[l],
                                       dW[l], lr, s));
  }
  return BNS_OK;
}

bns_status bns_train_step(bns_ctx *ctx, uint64_t seed, uint32_t epoch, double p, const float *X,
                          const float *const *halo_h, const void *labels, float *const *W, float *const *dW,
                          float *const *dhalo, float *loss, float lr, void *stream) {
  return train_step_impl(ctx, seed, epoch, nullptr, p, X, halo_h, labels, W, dW, dhalo, loss, lr, stream);
}

bns_status bns_graph_capture(bns_ctx *ctx, uint64_t seed, uint32_t first_epoch, double p, const float *X,
                             const float *const *halo_h, const void *labels, float *const *W, float *const *dW,
                             float *const *dhalo, float *loss, float lr, void *stream) {
  if (!ctx) return BNS_EINVAL;
  if (!stream) return fail(ctx, BNS_EINVAL, "graph capture needs a stream other than the null stream");
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (ctx->graph_exec) { (void)hipGraphExecDestroy(ctx->graph_exec); ctx->graph_exec = nullptr; }
  uint32_t *epoch_dev = reinterpret_cast<uint32_t *>(ctx->ws.counters + 2);
  BNS_TRY("set_counter", set_counter(epoch_dev, first_epoch, s));
  BNS_TRY("hipStreamBeginCapture", hipStreamBeginCapture(s, hipStreamCaptureModeThreadLocal));
  // event brackets are not part of the graph: the phase timers are off between here and the end
  // of the capture, and there is no return in between
  const uint32_t saved_mask = ctx->prof.mask;
  ctx->prof.mask = 0;
  bns_status st = train_step_impl(ctx, seed, 0, epoch_dev, p, X, halo_h, labels, W, dW, dhalo, loss, lr, stream);
  hipError_t e_bump = st == BNS_OK ? bump_counter(epoch_dev, s) : hipSuccess;
  hipGraph_t graph = nullptr;
  hipError_t e_end = hipStreamEndCapture(s, &graph);
  ctx->prof.mask = saved_mask;
  if (st != BNS_OK) { if (graph) (void)hipGraphDestroy(graph); return st; }
  if (e_bump != hipSuccess) { if (graph) (void)hipGraphDestroy(graph); return hip_fail(ctx, "bump_counter", e_bump); }
  if (e_end != hipSuccess) return hip_fail(ctx, "hipStreamEndCapture", e_end);
  hipError_t e_inst = hipGraphInstantiate(&ctx->graph_exec, graph, nullptr, nullptr, 0);
  (void)hipGraphDestroy(graph);
  if (e_inst != hipSuccess) { ctx->graph_exec = nullptr; return hip_fail(ctx, "hipGraphInstantiate", e_inst); }
  return BNS_OK;
}

bns_status bns_graph_replay(bns_ctx *ctx, int32_t n_epochs, void *stream) {
  if (!ctx || n_epochs < 0) return BNS_EINVAL;
  if (!ctx->graph_exec) return fail(ctx, BNS_EINVAL, "bns_graph_capture has not been called");
  for (int i = 0; i < n_epochs; ++i)
    BNS_TRY("hipGraphLaunch", hipGraphLaunch(ctx->graph_exec, static_cast<hipStream_t>(stream)));
  return BNS_OK;
}

int32_t bns_layer_plan(const bns_ctx *ctx, int32_t layer) {
  if (!ctx || layer < 1 || layer >= (int32_t)ctx->dims.size()) return -1;
  return layer_plan(ctx, layer, ctx->cache_X);
}

bns_status bns_set_dropout(bns_ctx *ctx, double q) {
  if (!ctx) return BNS_EINVAL;
  if (!(q >= 0.0 && q < 1.0)) return fail(ctx, BNS_EINVAL, "dropout rate must lie in [0, 1)");
  ctx->drop_q = q;
  return BNS_OK;
}

bns_status bns_adam_update(float *W, const float *dW, float *m, float *v, int64_t n, float lr, float beta1,
                           float beta2, float eps, int32_t t, void *stream) {
  if (!W || !dW || !m || !v || n < 0 || t < 1) return BNS_EINVAL;
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps > 0.f)) return BNS_EINVAL;
  return adam_update(n, W, dW, m, v, lr, beta1, beta2, eps, t, static_cast<hipStream_t>(stream)) == hipSuccess
             ? BNS_OK
             : BNS_EHIP;
}

bns_status bns_cache_input_aggregate(bns_ctx *ctx, const float *X, void *stream) {
  if (!ctx) return BNS_EINVAL;
  ctx->cache_X = nullptr;
  if (!X) return BNS_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // C0[v,:] = sum over the inner neighbours u of v of d~_u^-1/2 X[u,:] (GCN layer) or of X[u,:]
  // without the self-loop (mean aggregator): static CSR, inner entries only, no row factor
  const bool sage = ctx->layer_kind == 1;
  SpmmRowPart part;
  part.row_take = ctx->ws.split.n_inner;
  part.skip_self = sage;
  BNS_TRY("spmm_fwd(cache)", spmm_fwd(ctx->ws.plan_f, ctx->part.n_in, ctx->dims[0], ctx->part.row_ptr0,
                                      ctx->part.col0, sage ? nullptr : ctx->ws.dis_in, nullptr, X, nullptr,
                                      ctx->ws.spmm_partials, ctx->ws.C0, part, false, false, s));
  ctx->cache_X = X;
  return BNS_OK;
}

bns_status bns_profile_enable(bns_ctx *ctx, uint32_t phase_mask, int32_t max_records) {
  if (!ctx || max_records < 0) return BNS_EINVAL;
  Profiler &pr = ctx->prof;
  pr.mask = phase_mask;
  pr.used = 0;
  while (pr.start.size() < (size_t)max_records) {
    hipEvent_t a, b;
    BNS_TRY("hipEventCreate", hipEventCreate(&a));
    pr.start.push_back(a);
    BNS_TRY("hipEventCreate", hipEventCreate(&b));
    pr.stop.push_back(b);
  }
  pr.phase.assign(pr.start.size(), 0);
  return BNS_OK;
}

bns_status bns_profile_read(bns_ctx *ctx, double *ms_per_phase, int32_t *records_per_phase) {
  if (!ctx || !ms_per_phase || !records_per_phase) return BNS_EINVAL;
  Profiler &pr = ctx->prof;
  for (int i = 0; i < BNS_PHASE_COUNT; ++i) { ms_per_phase[i] = 0.0; records_per_phase[i] = 0; }
  for (size_t k = 0; k < pr.used; ++k) {
    BNS_TRY("hipEventSynchronize", hipEventSynchronize(pr.stop[k]));
    float ms = 0.f;
    BNS_TRY("hipEventElapsedTime", hipEventElapsedTime(&ms, pr.start[k], pr.stop[k]));
    ms_per_phase[pr.phase[k]] += ms;
    records_per_phase[pr.phase[k]] += 1;
  }
  pr.used = 0;
  return BNS_OK;
}

bns_status bns_ws_view(const bns_ctx *ctx, bns_view which, int32_t layer, void **dev_ptr, size_t *bytes) {
  if (!ctx || !dev_ptr || !bytes) return BNS_EINVAL;
  const Layout &w = ctx->ws;
  const size_t n_in = ctx->part.n_in, B = ctx->part.n_halo, nnz0 = ctx->part.nnz0;
  switch (which) {
    case BNS_VIEW_KEPT_IDS: *dev_ptr = w.kept_ids; *bytes = 4 * B; break;
    case BNS_VIEW_REMAP: *dev_ptr = w.remap; *bytes = 4 * B; break;
    case BNS_VIEW_N_KEPT: *dev_ptr = w.counters; *bytes = 4; break;
    case BNS_VIEW_ROW_PTR: *dev_ptr = w.row_ptr; *bytes = 4 * (n_in + 1); break;
    case BNS_VIEW_COL_IDX: *dev_ptr = w.col_idx; *bytes = 4 * nnz0; break;
    case BNS_VIEW_T_ROW_PTR: *dev_ptr = w.t_row_ptr; *bytes = 4 * (n_in + B + 1); break;
    case BNS_VIEW_T_COL_IDX: *dev_ptr = w.t_col_idx; *bytes = 4 * nnz0; break;
    case BNS_VIEW_NNZ: *dev_ptr = w.counters + 1; *bytes = 4; break;
    case BNS_VIEW_A:
    case BNS_VIEW_H:
    case BNS_VIEW_DZ:
      if (layer < 1 || layer > ctx->n_layers) return BNS_EINVAL;
      if (which == BNS_VIEW_A) { *dev_ptr = w.A[layer]; *bytes = 4 * n_in * (size_t)ctx->dims[layer - 1]; }
      else if (which == BNS_VIEW_H) { *dev_ptr = w.H[layer]; *bytes = 4 * n_in * (size_t)ctx->dims[layer]; }
      else { *dev_ptr = w.dZ[layer]; *bytes = 4 * n_in * (size_t)ctx->dims[layer]; }
      break;
    default: return BNS_EINVAL;
  }
  return BNS_OK;
}

}  // extern "C"
