/*
 * bns_gcn.h -- C ABI of the MI355X (gfx950) BNS-GCN partition step.
 *
 * One partition's full-graph GCN training iteration with random boundary-node
 * sampling (Algorithm 1, per-partition view), without the exchange steps: the
 * features of boundary nodes are supplied by the caller as preloaded buffers,
 * one per layer, standing in for what the other partitions would send.
 *
 * Conventions
 *  - "dev" pointers are device (HBM) pointers owned by the caller; "host"
 *    pointers are ordinary host memory.  The library never allocates or frees
 *    device memory: everything it needs lives in the caller's workspace.
 *  - All matrices are dense row-major fp32 without padding.
 *  - `stream` is a hipStream_t passed as void*.  Every call validates its
 *    arguments on the host, enqueues its kernels on `stream` and returns; it
 *    does not synchronise (bns_create is the one exception).  Counts produced
 *    on the device (|U|, nnz) stay on the device.
 *  - Every function returns a bns_status; nothing throws or aborts.  After a
 *    failure bns_last_error(ctx) describes it.
 *  - Calls on one context must be issued on one stream at a time: they share
 *    the workspace.
 *
 * Layout of a partition (Section 3.1: inner node set V_i, boundary node set B_i)
 *  - inner nodes have local ids 0..n_in-1; boundary node b (0..n_halo-1)
 *    appears as column n_in+b.  Only inner rows exist.
 *  - row_ptr0/col0: CSR of the local graph incl. one self-loop per row, columns
 *    strictly ascending in a row (so boundary columns form the row's tail).
 *  - t_in_ptr/t_in_col: CSR of the transpose of the inner-inner block.
 *  - halo_ptr/halo_col: for boundary node b, the ascending list of inner rows
 *    that contain column n_in+b.
 *  - deg_in/deg_halo: FULL-GRAPH degree + 1 (the diagonal of D~ in Appendix A),
 *    static over epochs; the normalisation never uses sampled degrees.
 */
#ifndef BNS_GCN_H
#define BNS_GCN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bns_ctx bns_ctx; /* opaque; host-side; holds descriptors and workspace offsets */

typedef enum {
  BNS_OK = 0,
  BNS_EINVAL = 1,     /* null pointer, bad size, p outside [0,1] or NaN, bad layer index      */
  BNS_EOVERFLOW = 2,  /* an index range does not fit int32                                    */
  BNS_EWORKSPACE = 3, /* workspace too small or misaligned                                    */
  BNS_EHIP = 4        /* a HIP call or kernel launch failed                                   */
} bns_status;

typedef struct {
  int32_t part_id;          /* i: enters the random draw, partitions sample independently */
  int32_t n_in;             /* |V_i|                                                      */
  int32_t n_halo;           /* |B_i|  (0 is legal)                                        */
  int64_t nnz0;             /* entries of col0   = e_in + e_bd                            */
  int64_t e_in;             /* entries of t_in_col (inner-inner block incl. self-loops)   */
  int64_t e_bd;             /* entries of halo_col (inner-boundary block)                 */
  const int32_t *row_ptr0;  /* dev int32[n_in+1]                                          */
  const int32_t *col0;      /* dev int32[nnz0]                                            */
  const int32_t *t_in_ptr;  /* dev int32[n_in+1]                                          */
  const int32_t *t_in_col;  /* dev int32[e_in]                                            */
  const int32_t *halo_ptr;  /* dev int32[n_halo+1]                                        */
  const int32_t *halo_col;  /* dev int32[e_bd]                                            */
  const int64_t *halo_gid;  /* dev int64[n_halo]  global node id of each boundary node    */
  const int32_t *deg_in;    /* dev int32[n_in]    full-graph degree + 1                   */
  const int32_t *deg_halo;  /* dev int32[n_halo]  full-graph degree + 1                   */
} bns_partition_desc;

typedef struct {
  int32_t n_layers;     /* L >= 1                                                          */
  const int32_t *dims;  /* host int32[L+1]: d_0 .. d_L (layer l maps d_{l-1} -> d_l); each
                           1..2048 if a multiple of 4, ..1024 if even, ..512 if odd       */
  int32_t loss_kind;    /* 0: softmax cross-entropy, labels dev int32[n_in] in [0, d_L); a
                              negative label marks a node outside the training set (the
                              splits of Table 2): no loss term, zero gradient
                           1: sigmoid binary cross-entropy, labels dev uint8[n_in*d_L] in
                              {0, 1}; the value 255 marks an entry outside the training set  */
  int32_t layer_kind;   /* 0: GCN layer of Appendix A, H' = sigma(P H W), W f32[d_in*d_out]
                           1: GraphSAGE with a mean aggregator (Section 2),
                              H' = sigma([mean of neighbours | H] W), W f32[2*d_in*d_out] with
                              the neighbour half first; kept boundary features are divided
                              by p and the mean keeps the full-graph neighbour count
                              (deg - 1 of the arrays below), Section 3.2                   */
} bns_model_desc;

/* Bytes of device workspace bns_create needs for this partition and model (sized for p = 1).
 * Returns 0 if a descriptor is invalid. */
size_t bns_workspace_bytes(const bns_partition_desc *part, const bns_model_desc *model);

/* Creates a context on the current device.  `dev_ws` (256-byte aligned, >= bns_workspace_bytes)
 * must stay valid, like every array named in `part`, until bns_destroy, and belongs to the
 * context from here on: the set-up leaves tables in it that every later call reads (d~^-1/2, the
 * inner/boundary split of the CSR, segment plans, the static rows of the transposed CSR), so the
 * caller must neither write to it nor hand it to a second context.  Runs the one-off set-up
 * kernels on `stream` and waits for them. */
bns_status bns_create(bns_ctx **out, const bns_partition_desc *part, const bns_model_desc *model,
                      void *dev_ws, size_t ws_bytes, void *stream);
void bns_destroy(bns_ctx *ctx);
const char *bns_last_error(const bns_ctx *ctx); /* never NULL; "" if no error so far.  ctx = NULL: the
                                                   error text of the latest context-free call
                                                   (bns_sample_boundary_noalloc) on this thread if
                                                   it failed, else "null context" */

/* Algorithm 1, selection step: U_i <- each b in B_i kept independently with probability p.
 * keep(b) <=> draw(seed, epoch, part_id, halo_gid[b]) < floor(p * 2^32), where draw is the
 * first output word of Philox-4x32-10 with counter (gid low, gid high, epoch, part_id) and key
 * (seed low, seed high): the same (seed, epoch, partition, node) always gives the same decision,
 * on any machine.  p = 1 keeps all, p = 0 none.
 *   kept_ids dev int32[n_halo] (capacity): the kept b, ascending, first *n_kept entries valid
 *   remap    dev int32[n_halo]: rank of b in kept_ids, or -1
 *   n_kept   dev int32[1]
 * The context remembers these three pointers for the calls below: the arrays must stay
 * allocated until a later bns_sample_boundary / bns_train_step replaces them. */
bns_status bns_sample_boundary(bns_ctx *ctx, uint64_t seed, uint32_t epoch, double p,
                               int32_t *kept_ids, int32_t *remap, int32_t *n_kept, void *stream);

/* The same selection step for callers that cannot allocate device memory and have no workspace to
 * hand over: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  It needs no context and calls no hipMalloc / hipFree or any routine that allocates:
 * the scratch of the kernels (one keep bit per boundary node, one count per 2048 nodes) lives in a
 * fixed array of about 0.5 MB inside the library's device code, of which every GPU the library runs
 * on holds its own copy until the process ends.  Inputs and outputs are the caller's, with the
 * meaning and layout of bns_sample_boundary (halo_gid dev int64[n_halo], part_id = the partition id
 * of the draw); the results are bit-identical to it.  n_halo > BNS_NOALLOC_MAX_HALO ->
 * BNS_EOVERFLOW; bad p or a null pointer -> BNS_EINVAL; bns_last_error(NULL) has the text.
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams,
 * two threads) race and give wrong results; calls that follow each other on one stream are fine,
 * nothing has to be cleared in between.  The first call on a device looks up the array's address
 * (a host-side query, no allocation); make that first call outside a stream capture. */
#define BNS_NOALLOC_MAX_HALO 4194304 /* 2^22 boundary nodes */
bns_status bns_sample_boundary_noalloc(const int64_t *halo_gid, int32_t n_halo, int32_t part_id,
                                       uint64_t seed, uint32_t epoch, double p, int32_t *kept_ids,
                                       int32_t *remap, int32_t *n_kept, void *stream);

/* Algorithm 1, subgraph step: the node-induced subgraph on V_i u U_i, in canonical CSR form, and
 * its transpose for the backward pass.
 *   remap, kept_ids, n_kept: the sample, exactly the three arrays the latest bns_sample_boundary on
 *             this context filled (that call also left the keep bits in the workspace, which this
 *             one reads); other pointers -> BNS_EINVAL
 *   row_ptr   dev int32[n_in+1], col_idx dev int32[nnz0] (capacity): inner columns unchanged,
 *             kept boundary column n_in+b renumbered n_in+remap[b], order preserved
 *   t_row_ptr dev int32[n_in+n_halo+1] (first n_in+*n_kept+1 valid), t_col_idx dev int32[nnz0]:
 *             for stacked column u the ascending inner rows holding u
 *   nnz       dev int32[1]
 * The layer calls below work on the subgraph of the most recent call: the context keeps the four
 * array pointers (and those of the sample), so the arrays must stay allocated until a later
 * bns_build_sampled_csr / bns_train_step replaces them. */
bns_status bns_build_sampled_csr(bns_ctx *ctx, const int32_t *remap, const int32_t *kept_ids,
                                 const int32_t *n_kept, int32_t *row_ptr, int32_t *col_idx,
                                 int32_t *t_row_ptr, int32_t *t_col_idx, int32_t *nnz, void *stream);

/* One layer forward, Eq. 1 then Eq. 2 in the sampled matrix form of Appendix A:
 *   A = [P_VV P_VU] S [H_in ; halo_h[kept_ids]],  S = diag(1 .. 1, 1/p .. 1/p),
 *   P_vu = (d~_v d~_u)^-1/2;   H_out = A W, followed by ReLU iff relu != 0.
 * layer in 1..L selects d_in = d_{layer-1}, d_out = d_layer.  Uses the latest sample and CSR.
 *   H_in dev f32[n_in*d_in]; halo_h dev f32[n_halo*d_in] (ALL boundary rows, unscaled; only
 *   kept rows are read; may be NULL iff n_halo == 0); W dev f32[d_in*d_out];
 *   A_saved dev f32[n_in*d_in] (out, kept for backward); H_out dev f32[n_in*d_out] (out). */
bns_status bns_gcn_layer_fwd(bns_ctx *ctx, int32_t layer, double p, const float *H_in,
                             const float *halo_h, const float *W, float *A_saved, float *H_out,
                             int32_t relu, void *stream);

/* One layer backward (Algorithm 1, backward step; Section 3.2: a partition returns feature
 * gradients of its selected boundary nodes).  With dZ = dH_out (.) [H_out > 0] (or dZ = dH_out
 * when H_out is NULL, i.e. no ReLU on this layer):
 *   dW = A_saved^T dZ;  dA = dZ W^T;  [dH_in ; dhalo] = S^T P^T dA.
 *   dW dev f32[d_in*d_out] (out); dH_in dev f32[n_in*d_in] (out, or NULL to skip dA and the
 *   transposed aggregate, as for layer 1); dhalo dev f32[n_halo*d_in] (capacity; first *n_kept
 *   rows valid: gradient w.r.t. the unscaled features of the kept boundary nodes; NULL to skip).
 * H_in (the layer's input, dev f32[n_in*d_in]) is read by the mean-aggregator layer only
 * (dW = [A_saved | H_in]^T dZ, f32[2*d_in*d_out]); it may be NULL for the GCN layer. */
bns_status bns_gcn_layer_bwd(bns_ctx *ctx, int32_t layer, double p, const float *dH_out,
                             const float *H_out, const float *A_saved, const float *H_in,
                             const float *W, float *dW, float *dH_in, float *dhalo, void *stream);

/* One iteration of Algorithm 1 for this partition: sample, induced subgraph (+ transpose), L
 * layers forward, loss summed over inner nodes, backward, optional SGD w <- w - lr * g.
 *   X dev f32[n_in*d_0]; halo_h host array of L dev pointers, halo_h[l] = f32[n_halo*d_l];
 *   labels dev (see loss_kind); W host array of L dev pointers f32[d_{l}*d_{l+1}], updated in
 *   place iff lr > 0; dW host array of L dev pointers (out); dhalo NULL, or host array of L dev
 *   pointers f32[n_halo*d_l] (entry 0 unused, NULL entries skipped); loss dev f32[1] (out).
 * Intermediate results stay in the workspace and can be located with bns_ws_view. */
bns_status bns_train_step(bns_ctx *ctx, uint64_t seed, uint32_t epoch, double p, const float *X,
                          const float *const *halo_h, const void *labels, float *const *W,
                          float *const *dW, float *const *dhalo, float *loss, float lr,
                          void *stream);

/* The epoch loop of Algorithm 1 as a HIP graph.  bns_graph_capture records one bns_train_step (same
 * arguments) on `stream`, which must be a created stream, not the null stream; inside the graph
 * the epoch index lives in device memory, starts at first_epoch and is advanced by one at the end
 * of every replay, so each replay draws a fresh boundary sample.  bns_graph_replay launches the
 * recorded step n_epochs times on `stream` without synchronising.  Every pointer passed at capture
 * time (and the arrays they name) must stay valid and in place until the graph is replaced by a
 * new capture or the context is destroyed.  With lr > 0 the weights are updated in place, i.e.
 * n replays run n epochs of Algorithm 1.  Event brackets (bns_profile_enable) are not recorded.
 * The dropout rate, the input-aggregate cache and the layer plans in effect at capture time are
 * part of the recording: change them (bns_set_dropout, bns_cache_input_aggregate) and capture again. */
bns_status bns_graph_capture(bns_ctx *ctx, uint64_t seed, uint32_t first_epoch, double p, const float *X,
                             const float *const *halo_h, const void *labels, float *const *W,
                             float *const *dW, float *const *dhalo, float *loss, float lr,
                             void *stream);
bns_status bns_graph_replay(bns_ctx *ctx, int32_t n_epochs, void *stream);

/* How bns_train_step runs layer `layer` (1..L); host-only query, -1 for a bad argument.  The
 * three plans give the same results up to rounding (Appendix A writes Z = P H W without
 * parentheses); they differ in kernel boundaries, in what BNS_VIEW_A holds and in what the phase
 * timers attribute to BNS_PHASE_SPMM_FWD / BNS_PHASE_GEMM_FWD.
 *   BNS_LAYER_TWO_KERNELS  aggregate (Eq. 1), then update (Eq. 2); BNS_VIEW_A = the aggregate.
 *   BNS_LAYER_ONE_KERNEL   the same two steps in one kernel: input width a multiple of 4 between 68
 *                          and 128; the mean-aggregator layer, whose update is twice as deep, only
 *                          with an output width of at most 256 and at most 3.25 times the average
 *                          number of entries per row (a longer update is faster as a kernel of its
 *                          own); BNS_VIEW_A = the aggregate.
 *   BNS_LAYER_UPDATE_FIRST a GCN layer whose output is at most 3/4 as wide as its input (and whose
 *                          aggregate thereby gathers at least 2^24 fewer floats) is run as
 *                          P (H W): the products H W and H_U W first, then the aggregate at the
 *                          output width; its backward pass forms the weight gradient as
 *                          [H ; H_U]^T (P^T dZ).  BNS_VIEW_A then holds H W: n_in rows of d_l
 *                          floats at a row stride of s floats, where s = d_l rounded up to a
 *                          multiple of 4 if d_l is not one and s < 128 and s <= d_{l-1} (the
 *                          aggregate gathers 16 bytes per lane; pad columns are zero), else
 *                          s = d_l.  Not used for layer 1 while bns_cache_input_aggregate is in
 *                          effect.
 * bns_gcn_layer_fwd / bns_gcn_layer_bwd always aggregate first (their A_saved is the aggregate). */
typedef enum { BNS_LAYER_TWO_KERNELS = 0, BNS_LAYER_ONE_KERNEL = 1, BNS_LAYER_UPDATE_FIRST = 2 } bns_layer_plan_kind;
int32_t bns_layer_plan(const bns_ctx *ctx, int32_t layer);

/* Dropout on the hidden activations, as in the training set-up of Section 4 (rates 0.1 - 0.5).
 * With rate q in (0, 1) every element of the output of a layer that has a ReLU (layers 1..L-1 of
 * bns_train_step, relu != 0 in bns_gcn_layer_fwd) is zeroed with probability q and multiplied by
 * 1/(1-q) otherwise, and the backward calls scale the gradient of the surviving elements
 * accordingly (an element that is zero after dropout passes no gradient).  The draw is counter
 * based, one per element and built like the boundary draw: the first output word of Philox-4x32-10
 * on the counter (row, column, part_id * 256 + layer, epoch) under the key (seed lo, seed hi xor
 * 0x64726F70), with the seed and epoch of the latest bns_sample_boundary / bns_train_step on this
 * context; kept iff the word is below floor((1-q) * 2^32).  Boundary features are used as handed in (their owners applied their
 * own dropout).  q = 0 (the default) switches dropout off; q outside [0, 1) -> BNS_EINVAL. */
bns_status bns_set_dropout(bns_ctx *ctx, double q);

/* Adam, the optimiser of the paper's experiments (Section 4; Kingma & Ba 2015), as an alternative
 * to the plain update of Algorithm 1: call bns_train_step with lr = 0, then this once per weight
 * matrix.  m, v: dev f32[n] moment buffers owned by the caller (zero before the first step);
 * t >= 1 is the step count (bias correction).  Needs no context. */
bns_status bns_adam_update(float *W, const float *dW, float *m, float *v, int64_t n, float lr,
                           float beta1, float beta2, float eps, int32_t t, void *stream);

/* Static-inner caching.  The input features X and the inner-inner edges are the same in every
 * epoch; sampling only changes the boundary entries of a row (Appendix D).  This call aggregates the
 * inner neighbours of layer 1 once, C[v,:] = sum_{u in V_i, u ~ v} d~_u^-1/2 X[u,:], into the
 * workspace.  Afterwards every layer-1 forward whose input pointer equals X (bns_gcn_layer_fwd with
 * layer 1, bns_train_step) aggregates only the kept boundary tail of each row and adds C.  The caller
 * promises not to change the contents of X while the cache is installed; X = NULL drops it. */
bns_status bns_cache_input_aggregate(bns_ctx *ctx, const float *X /* dev f32[n_in*d_0] */, void *stream);

/* Where bns_train_step keeps its intermediates inside the workspace (for inspection). */
typedef enum {
  BNS_VIEW_KEPT_IDS = 0,  /* int32[n_halo]            */
  BNS_VIEW_REMAP = 1,     /* int32[n_halo]            */
  BNS_VIEW_N_KEPT = 2,    /* int32[1]                 */
  BNS_VIEW_ROW_PTR = 3,   /* int32[n_in+1]            */
  BNS_VIEW_COL_IDX = 4,   /* int32[nnz0]              */
  BNS_VIEW_T_ROW_PTR = 5, /* int32[n_in+n_halo+1]     */
  BNS_VIEW_T_COL_IDX = 6, /* int32[nnz0]              */
  BNS_VIEW_NNZ = 7,       /* int32[1]                 */
  BNS_VIEW_A = 8,         /* layer l: f32[n_in*d_{l-1}], l = 1..L */
  BNS_VIEW_H = 9,         /* layer l: f32[n_in*d_l],     l = 1..L (H_L = logits) */
  BNS_VIEW_DZ = 10        /* layer l: f32[n_in*d_l],     l = 1..L: gradient of the loss w.r.t. the
                             pre-activation of layer l as the backward pass used it (for l < L
                             already masked by H_l > 0 and scaled by the dropout slope) */
} bns_view;
bns_status bns_ws_view(const bns_ctx *ctx, bns_view which, int32_t layer, void **dev_ptr,
                       size_t *bytes);

/* Instrumentation (no counterpart in the paper; its appendix on sampling overhead reports the
 * share of sampling in the training time, which these timers reproduce per kernel class).
 * While a phase's bit is set, bns_train_step and the layer calls bracket that phase's kernels
 * with two HIP events on the call's stream.  At most max_records brackets are kept between two
 * reads; further ones are dropped.  bns_profile_read waits for the recorded events, returns per
 * phase the summed milliseconds and the number of brackets since the last read, and clears them.
 * Events are host objects: no device memory is allocated. */
typedef enum {
  BNS_PHASE_SAMPLE = 0,   /* sample_boundary kernels; in bns_train_step on a small partition (at most 4096
                             boundary nodes, 8192 boundary entries, 16384 inner nodes + inner entries) the one
                             launch that runs the selection and the subgraph step together               */
  BNS_PHASE_BUILD = 1,    /* sampled CSR + transposed CSR (no bracket where the sample phase covers it)  */
  BNS_PHASE_GATHER = 2,   /* gather of kept boundary features (x 1/p)      */
  BNS_PHASE_SPMM_FWD = 3, /* aggregate                                     */
  BNS_PHASE_GEMM_FWD = 4, /* update  A W                                   */
  BNS_PHASE_LOSS = 5,
  BNS_PHASE_GEMM_DW = 6,  /* A^T dZ (split-K + reduction)                  */
  BNS_PHASE_GEMM_DA = 7,  /* dZ W^T                                        */
  BNS_PHASE_SPMM_BWD = 8, /* transposed aggregate                          */
  BNS_PHASE_SGD = 9,
  BNS_PHASE_SPMM_LONG = 10, /* forward aggregate of the rows longer than one segment, where it
                               runs as a pass of its own before a one-kernel layer */
  BNS_PHASE_COUNT = 11
} bns_phase;
bns_status bns_profile_enable(bns_ctx *ctx, uint32_t phase_mask, int32_t max_records);
bns_status bns_profile_read(bns_ctx *ctx, double *ms_per_phase /* host [BNS_PHASE_COUNT] */,
                            int32_t *records_per_phase /* host [BNS_PHASE_COUNT] */);

/* Instrumentation: the access pattern of the aggregate (Eq. 1) stripped of its arithmetic, to
 * measure what this machine delivers for it.  Every wavefront sums per_wave rows of `table`
 * (dev f32[n_rows*d], d in {16, 32, 64, 128, 256}) chosen by `idx` (dev int32[n_idx], values in
 * [0, n_rows); the caller's responsibility, they are not checked) and stores the sum as one row:
 * out dev f32[ceil(n_idx / per_wave) * d].  No weights, no row structure.  bench.py times it with
 * as many uniformly random indices as a layer has entries, over a table as large as the layer's
 * stacked features: the rate at which an aggregate on a graph without locality can gather. */
bns_status bns_probe_gather(const float *table, int64_t n_rows, int32_t d, const int32_t *idx,
                            int64_t n_idx, int32_t per_wave, float *out, void *stream);

/* Instrumentation: the fp32 matrix instruction of the update (Eq. 2), v_mfma_f32_32x32x2_f32, with
 * nothing else in the loop.  `blocks` workgroups of waves_per_block (1..16) wavefronts each issue
 * iters * 8 * n_acc of them on n_acc (1, 2, 3, 4 or 6) independent accumulators per wavefront:
 * 4096 * 8 * n_acc * iters * waves_per_block * blocks flops in all.  out dev f32[blocks] receives one
 * checksum per workgroup (1024-thread workgroups leave 128 registers per wavefront, enough for
 * every n_acc).  bench.py --mfma-regimes times it over wavefronts per SIMD x accumulators per
 * wavefront: the issue rates the GEMM tile shapes were chosen by. */
bns_status bns_probe_mfma(int32_t n_acc, int32_t waves_per_block, int32_t blocks, int32_t iters,
                          float *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BNS_GCN_H */
