/*
 * nf — the per-layer local training step of adaptive local learning on one AMD MI355X
 * (gfx950), as a C-ABI library of hand-written HIP kernels.
 *
 * Method: NeuroFlux (arXiv 2402.14139).  One local step is the body of Algorithm 2 for
 * one (batch, layer) pair:
 *     x_{n+1} = ReLU(P_n(theta_n * x_n))                         Eq. 1
 *     z       = gamma_n F_n beta_n x_{n+1}                       Eq. 2
 *     L       = mean_k CE(z_k, y_k)                              Eq. 3
 *     gradients of L w.r.t. (theta_n, beta_n, gamma_n) only, then the update,
 * plus the activation cache that carries a trained block's output to the next block at
 * that block's own batch size (section "Efficient Forward Propagation via Prefetching and
 * Adaptive Batching").
 *
 * ---- Data layout (all tensors dense fp32 unless stated, all pointers DEVICE pointers) ----
 *   activations  NHWC : x[n][h][w][c]
 *   conv weights KRSC : W[k][r][s][c]         (k = output channel)
 *   projection        : Wp[k][c]              (1x1, stride skip_stride, no bias)
 *   aux conv     ARSK : Wa[a][r][s][k]        (a = aux filter, k = layer output channel)
 *   linear            : Wf[q][f], f = (i*pool_ow + j)*A + a   (NHWC flatten of the pooled map)
 *   labels            : int32 in [0, n_classes)
 *   cache row         : one sample's emitted activation, H*W*C contiguous floats (NHWC)
 * These are index permutations of the paper-notation tensors (NCHW / OIHW / flatten a,i,j);
 * the library never transposes activations.
 *
 * ---- Ownership, streams, errors -----------------------------------------------------------
 *   The caller owns every buffer, including the workspace `ws` (size from
 *   nf_workspace_bytes, 256-byte aligned).  The library allocates nothing and keeps no
 *   state between calls (five documented exceptions: the static scratch array of
 *   nf_local_step_static, the event pool of the prefetch mode of nf_block_train_epoch, the
 *   graph handles of nf_block_graph_create, the process-wide contraction mode of nf_contraction,
 *   and the measurement aid nf_prof_begin/end).  `stream` is a hipStream_t passed as void*
 *   (NULL = default stream); every call only enqueues work on it and never synchronises the host.
 *   Every device pointer must be 16-byte aligned.
 *   Every call returns NF_OK (0) or a negative nf_status.  Arguments are validated before
 *   anything is enqueued, so a failing call has no side effects on device memory.
 *   Labels outside [0,n_classes) and cache indices outside [0,capacity) are NOT detected
 *   (they are data on the device); such a label contributes as if no class matched and
 *   such an index is clamped into range.
 *   Calls sharing a workspace must be ordered on one stream.
 */
#ifndef NF_H
#define NF_H
#include <stddef.h>
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  NF_OK = 0,
  NF_ERR_NULL = -1,        /* a required pointer is NULL                                   */
  NF_ERR_BAD_DESC = -2,    /* non-positive size, inconsistent shapes, misaligned pointer   */
  NF_ERR_UNSUPPORTED = -3, /* filter/stride/pool outside what the kernels implement        */
  NF_ERR_WORKSPACE = -4,   /* workspace NULL, misaligned or smaller than required          */
  NF_ERR_CACHE_RANGE = -5, /* first + B exceeds the cache capacity                         */
  NF_ERR_DEVICE = -6,      /* a HIP call failed (launch error)                             */
  NF_ERR_SCRATCH_LIMIT = -7 /* nf_local_step_static: the step needs more than NF_STATIC_SCRATCH_BYTES */
} nf_status;

/* Layer n of Eq. 1: conv theta_n (+bias, + optional shortcut), ReLU, optional max-pool P_n.
 * Supported: 1 <= R,S <= 15, 1 <= stride <= 4, 0 <= pad < R + S; max-pool with
 * 2*pool_pad <= pool_k <= 15 and any positive stride.  Anything else: NF_ERR_UNSUPPORTED. */
typedef struct {
  int32_t C_in, H_in, W_in;
  int32_t C_out, R, S, stride, pad;
  int32_t pool_kind; /* 0 none, 1 max */
  int32_t pool_k, pool_stride, pool_pad;
  int32_t skip_kind; /* 0 none; 1 identity (x_skip has the conv-output shape);
                        2 projection: + sum_c Wp[k][c] * x_skip[n][i*skip_stride][j*skip_stride][c] */
  int32_t skip_C, skip_H, skip_W, skip_stride;
} nf_layer_desc;

/* Auxiliary head A_n of Eq. 2: conv beta_n (R x S, stride 1, pad, + bias, ReLU if relu),
 * adaptive pooling F_n to pool_oh x pool_ow (average or max: the two down-sampling mechanisms
 * the text below Eq. 1 names), linear gamma_n to n_classes.  The loss l of Eq. 3 is softmax
 * cross-entropy, or the mean squared error against the one-hot label (mean over the classes,
 * then over the batch).  C_in/H_in/W_in describe the tensor the layer emits (post-pool). */
enum { NF_HEAD_POOL_AVG = 0, NF_HEAD_POOL_MAX = 1 };
enum { NF_LOSS_CE = 0, NF_LOSS_MSE = 1 };
typedef struct {
  int32_t C_in, H_in, W_in;
  int32_t A, R, S, pad, relu;
  int32_t pool_oh, pool_ow;
  int32_t n_classes;
  int32_t head_pool; /* NF_HEAD_POOL_*; ties of the max go to the first element in row-major order */
  int32_t loss_kind; /* NF_LOSS_* */
} nf_aux_desc;

typedef struct {
  float lr, momentum;
} nf_sgd_desc;

/* Parameters of the layer (theta_n) and of its head (beta_n, gamma_n).  The same structs
 * carry gradients and momentum buffers.  Wp is ignored unless skip_kind == 2. */
typedef struct {
  float *W, *b, *Wp;
} nf_layer_params;
typedef struct {
  float *Wa, *ba, *Wf, *bf;
} nf_aux_params;

const char *nf_strerror(int32_t status);

/* How the wide contractions (the convolution of Eq. 1 and its weight gradient in Algorithm 2, for
 * layers with at least 128 filters) are carried out.  Operands, results and accumulation are fp32
 * in both modes.
 *   NF_CONTRACT_F32     (default) fp32 matrix-core instructions (v_mfma_f32_32x32x2_f32).
 *   NF_CONTRACT_BF16X6  each fp32 operand element is cut into three bfloat16 pieces that sum to it
 *                       exactly; six of the nine piece products are accumulated in fp32 by bf16
 *                       matrix-core instructions.  The three left out are together below 2^-21 of
 *                       the product in the worst case and about 2^-24 of it in the root mean
 *                       square, i.e. of the size of an fp32 rounding; over the reductions of this
 *                       library (36 ... 4608 terms) the measured error against fp64 equals that of
 *                       the fp32 instructions.  An operand element that is +-inf gives NaN
 *                       instead of +-inf.
 *   NF_CONTRACT_BF16X9  the same with all nine piece products: every product x*w enters the fp32
 *                       accumulation exactly, as with the fp32 instructions; 1.5x the matrix-core
 *                       work of BF16X6.
 * Process-wide (read when a call enqueues its kernels); returns the previous mode, or
 * NF_ERR_BAD_DESC for an unknown mode.  mode = -1 only queries. */
enum { NF_CONTRACT_F32 = 0, NF_CONTRACT_BF16X6 = 1, NF_CONTRACT_BF16X9 = 2 };
int32_t nf_contraction(int32_t mode);

/* Emitted sizes: conv output (Ho,Wo) and post-pool (Hp,Wp).  Any out pointer may be NULL. */
int32_t nf_layer_out_dims(const nf_layer_desc *d, int32_t *Ho, int32_t *Wo, int32_t *Hp, int32_t *Wp);

/* Bytes of workspace the calls below need for this (layer, head, batch).  `a` may be NULL
 * when only nf_layer_fwd will be called. */
int32_t nf_workspace_bytes(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B, size_t *out);

/* Where two intermediates of the step live inside the workspace (byte offset and size), for
 * callers that want to inspect them after nf_aux_fwd_loss / nf_local_step (tests compare the
 * ReLU and max-pool decisions the kernels took):
 *   NF_WS_AUX_ACT   the head's convolution output after its ReLU (Eq. 2, beta_n), fp32
 *                   [B][Hu][Wu][A];
 *   NF_WS_POOL_ARG  one byte per emitted element [B][Hp][Wp][C_out]: index u*pool_k+v of the
 *                   window cell the max-pool P_n of Eq. 1 selected (size 0 when un-pooled);
 *   NF_WS_HEAD_ARG  int32 [B][pool_oh][pool_ow][A]: flat position h*Wu+w inside the head's
 *                   convolution output that a max-pooling F_n selected (size 0 when F_n averages). */
enum { NF_WS_AUX_ACT = 0, NF_WS_POOL_ARG = 1, NF_WS_HEAD_ARG = 2 };
int32_t nf_workspace_region(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B, int32_t which,
                            size_t *offset, size_t *bytes);

/* Eq. 1.  x [B,H_in,W_in,C_in], x_skip per skip_kind (NULL if 0), y OUT [B,Hp,Wp,C_out].
 * Records in ws what the backward needs (pool arg-max). */
int32_t nf_layer_fwd(const nf_layer_desc *d, int32_t B, const float *x, const float *x_skip,
                     const nf_layer_params *p, float *y, void *ws, size_t ws_bytes, void *stream);

/* Eq. 2 + Eq. 3.  y is the emitted activation [B,Hp,Wp,C_out]; *loss_out (device float)
 * receives the batch-mean cross-entropy.  Leaves the head's activations and dL/dz in ws.
 * `d` is the layer the head is attached to (it fixes where the head's data sits in ws). */
int32_t nf_aux_fwd_loss(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B, const float *y,
                        const int32_t *labels, const nf_aux_params *ap, float *loss_out, void *ws,
                        size_t ws_bytes, void *stream);

/* Algorithm 2, gradient line: gradients of the local loss w.r.t. theta_n, beta_n, gamma_n.
 * Must follow nf_layer_fwd and nf_aux_fwd_loss on the same ws.  gp/ga are OVERWRITTEN
 * (not accumulated).  No gradient is formed for x or x_skip. */
int32_t nf_local_bwd_wgrad(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B,
                           const float *x, const float *x_skip, const float *y,
                           const nf_layer_params *p, const nf_aux_params *ap,
                           const nf_layer_params *gp, const nf_aux_params *ga, void *ws,
                           size_t ws_bytes, void *stream);

/* Algorithm 2, update line, for n_tensors (<= 16) tensors in one launch:
 *   v = momentum*v + g ; w = w - lr*v      (v == NULL or momentum == 0: w = w - lr*g)
 * w, g, v are HOST arrays of device pointers; numel a HOST array of element counts. */
int32_t nf_sgd_update(const nf_sgd_desc *s, int32_t n_tensors, float *const *w, const float *const *g,
                      float *const *v, const int64_t *numel, void *stream);

/* Activation cache.  cache [capacity][sample_elems], cache_labels [capacity] (may be NULL
 * together with labels).  Write stores batch rows at [first, first+B).  Read gathers B rows:
 * idx == NULL -> rows first..first+B-1, else rows idx[0..B) (device int64) — B is the
 * CONSUMING block's batch size and need not equal the batch size used for writing. */
int32_t nf_cache_write(float *cache, int32_t *cache_labels, int64_t capacity, int64_t sample_elems,
                       int64_t first, int32_t B, const float *y, const int32_t *labels, void *stream);
int32_t nf_cache_read(const float *cache, const int32_t *cache_labels, int64_t capacity,
                      int64_t sample_elems, int64_t first, const int64_t *idx, int32_t B, float *x_out,
                      int32_t *labels_out, void *stream);

/* The whole Algorithm 2 body for one (batch, layer): forward, head, loss, gradients, update
 * of p/ap in place, and y_out = the activation emitted with the PRE-update weights (it is
 * the next layer's input).  gp/ga receive the gradients; vp/va are momentum buffers (may be
 * NULL when s->momentum == 0). */
int32_t nf_local_step(const nf_layer_desc *d, const nf_aux_desc *a, const nf_sgd_desc *s, int32_t B,
                      const float *x, const float *x_skip, const int32_t *labels,
                      const nf_layer_params *p, const nf_aux_params *ap, const nf_layer_params *gp,
                      const nf_aux_params *ga, const nf_layer_params *vp, const nf_aux_params *va,
                      float *y_out, float *loss_out, void *ws, size_t ws_bytes, void *stream);

/* nf_local_step for callers that cannot allocate device memory or hand in a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-for-bit the same results as nf_local_step, but the scratch lives in a
 * file-scope device array of NF_STATIC_SCRATCH_BYTES inside the library (one copy per GPU the
 * library runs on, held until the process ends) instead of a caller workspace.  The call
 * allocates nothing (no hipMalloc / hipFree, no allocating library routine).
 * A (layer, head, B) whose nf_workspace_bytes exceeds NF_STATIC_SCRATCH_BYTES is rejected with
 * NF_ERR_SCRATCH_LIMIT before anything is enqueued (a 512-channel 3x3 layer at batch 512 on 4x4
 * maps needs 89 MiB, the largest layer of the VGG-16-style workload 115 MiB).
 * Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (two
 * streams, two threads) race; order them on one stream.  The array keeps the previous call's
 * contents, which is harmless: every region is written by the step before it is read.  The
 * intermediates nf_workspace_region describes are not reachable through this entry point. */
#define NF_STATIC_SCRATCH_BYTES (128u << 20)
int32_t nf_local_step_static(const nf_layer_desc *d, const nf_aux_desc *a, const nf_sgd_desc *s, int32_t B,
                             const float *x, const float *x_skip, const int32_t *labels,
                             const nf_layer_params *p, const nf_aux_params *ap, const nf_layer_params *gp,
                             const nf_aux_params *ga, const nf_layer_params *vp, const nf_aux_params *va,
                             float *y_out, float *loss_out, void *stream);

/* ---- a block of consecutive local layers (the paper's partition of the network into blocks,
 * each trained at its own batch size; Worker loop of Algorithm 2; "Efficient Forward Propagation
 * via Prefetching and Adaptive Batching") ---------------------------------------------------------
 * All arrays are HOST arrays with n_layers entries; the pointers inside the parameter structs
 * are device pointers.  Layer n+1 reads what layer n emits, so its C_in/H_in/W_in must equal
 * layer n's C_out/Hp/Wp.  skip_src (NULL = no shortcuts) gives per layer -1, or the position
 * m <= n of the layer whose INPUT tensor is layer n's shortcut (0 = the block's input batch);
 * that tensor's shape must equal the layer's skip_C/skip_H/skip_W.  aux/ap/gp/ga are not read by
 * nf_block_fill_cache and may be NULL there; vp/va may be NULL when momentum == 0.  gp/ga are
 * scratch of the pass (they hold the last batch's gradients afterwards).  The block calls validate
 * every descriptor, shape, pointer and alignment of every layer before the first enqueue, so an
 * argument error has no side effects; only a HIP error (NF_ERR_DEVICE) can surface mid-pass, and
 * then the prefetch stream, if any, is joined back into `stream` before the call returns. */
typedef struct {
  int32_t n_layers;
  const nf_layer_desc *layers;
  const nf_aux_desc *aux;
  const int32_t *skip_src;
  const nf_layer_params *p;
  const nf_aux_params *ap;
  const nf_layer_params *gp;
  const nf_aux_params *ga;
  const nf_layer_params *vp;
  const nf_aux_params *va;
} nf_block;

/* Workspace of the two block calls at batch size B: two input batches (double buffer), every
 * layer's emitted batch, and the largest single-layer workspace. */
int32_t nf_block_workspace_bytes(const nf_block *blk, int32_t B, size_t *out);

/* One pass of the block over n_items cached samples in batches of B (the last one may be
 * smaller): per batch, nf_cache_read (rows idx[j], device int64 [n_items], or rows 0..n_items-1
 * when idx == NULL; cache [capacity][C_in*H_in*W_in of layer 0], cache_labels [capacity]), then
 * nf_local_step layer by layer, each layer handing on the activations it emitted BEFORE its
 * update.  losses (device, [ceil(n_items/B)][n_layers]) receives every local loss.
 * prefetch_stream != NULL: the read of batch j+1 is enqueued there and overlaps the training of
 * batch j (the paper's prefetching); it is ordered after everything already enqueued on `stream`
 * and joined back into `stream` before the call's last batch, so `stream` alone orders the
 * result.  That mode uses four process-wide HIP events per device, created on first use: calls
 * with a prefetch stream must not overlap in time on one device.  Both streams must have the
 * default priority. */
int32_t nf_block_train_epoch(const nf_block *blk, const nf_sgd_desc *s, int32_t B, int64_t n_items,
                             const float *cache, const int32_t *cache_labels, int64_t capacity,
                             const int64_t *idx, float *losses, void *ws, size_t ws_bytes,
                             void *stream, void *prefetch_stream);

/* The same pass (Algorithm 2, the Worker's loop over the batches of a block) as a HIP graph the
 * library captures itself (the per-batch work of a block is a few
 * hundred short launches; replayed from a graph they are enqueued by one call and the gaps between
 * them shrink).  nf_block_graph_create takes the arguments of nf_block_train_epoch without the
 * streams, validates them the same way (same error codes, nothing captured on error), captures the
 * whole pass over the n_items samples on a private stream and instantiates it; *out is the handle.
 * The graph is a snapshot of the ARGUMENTS: every pointer, B, n_items, lr, momentum, the descriptors
 * and the contraction mode in force at creation are fixed; what the pointers point at (cache rows,
 * the index list idx, weights, momentum) is read when the graph runs, so an epoch with a new shuffle
 * is: rewrite idx on the device, launch again.  All buffers must stay alive until the handle is
 * destroyed.  nf_block_graph_launch enqueues one pass on `stream` (default priority) of the device
 * the graph was created on (another current device: NF_ERR_BAD_DESC); results are bit-identical to
 * nf_block_train_epoch with prefetch_stream == NULL.  Launches of one handle must not overlap in
 * time (they share ws).  nf_block_graph_destroy frees the handle (NULL is accepted).  Creation
 * between nf_prof_begin and nf_prof_end is refused with NF_ERR_UNSUPPORTED.  These three calls are
 * the only ones in the library that allocate: the graph objects and the handle, host side. */
typedef struct nf_block_graph nf_block_graph;
int32_t nf_block_graph_create(const nf_block *blk, const nf_sgd_desc *s, int32_t B, int64_t n_items,
                              const float *cache, const int32_t *cache_labels, int64_t capacity,
                              const int64_t *idx, float *losses, void *ws, size_t ws_bytes,
                              nf_block_graph **out);
int32_t nf_block_graph_launch(nf_block_graph *g, void *stream);
int32_t nf_block_graph_destroy(nf_block_graph *g);

/* After the block is trained: forward-only sweep with its final weights over rows [0, n_items)
 * of its input cache in batches of B (last one partial), writing the last layer's emitted
 * activations and the labels to rows [0, n_items) of the next block's cache
 * (cache_out [capacity_out][C_out*Hp*Wp of the last layer]). */
int32_t nf_block_fill_cache(const nf_block *blk, int32_t B, int64_t n_items, const float *cache_in,
                            const int32_t *labels_in, int64_t capacity_in, float *cache_out,
                            int32_t *labels_out, int64_t capacity_out, void *ws, size_t ws_bytes,
                            void *stream);

/* ---- early-exit evaluation ("Trained Output CNN") ---------------------------------------------
 * nf_aux_predict: forward of the head only on emitted activations y [B,Hp,Wp,C_out]; pred_out
 * (device int32 [B]) receives the class with the largest logit (lowest index among equal maxima);
 * with labels, *n_correct (device int32) receives the number of correct predictions of the batch,
 * added to its previous value when accumulate != 0 (labels and n_correct are given together or
 * both NULL); logits_out (device [B][n_classes]) is optional.
 * nf_block_evaluate: the early-exit model that leaves the block after layer exit_layer: rows
 * [0, n_items) of the block's input cache in batches of B (last one partial), forward through
 * layers 0..exit_layer, that layer's head; pred_out [n_items], *n_correct the total (cache_labels
 * and n_correct may both be NULL: plain prediction).  The block's aux and ap arrays are required,
 * gp/ga/vp/va are not read.
 * nf_select_exit (host): index of the exit with the most correct validation predictions; among
 * equals the one whose model has the fewest parameters; among those the earliest. */
int32_t nf_aux_predict(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B, const float *y,
                       const int32_t *labels, const nf_aux_params *ap, int32_t *pred_out, int32_t *n_correct,
                       int32_t accumulate, float *logits_out, void *ws, size_t ws_bytes, void *stream);
int32_t nf_block_evaluate(const nf_block *blk, int32_t exit_layer, int32_t B, int64_t n_items,
                          const float *cache, const int32_t *cache_labels, int64_t capacity,
                          int32_t *pred_out, int32_t *n_correct, void *ws, size_t ws_bytes, void *stream);
int32_t nf_select_exit(int32_t n_exits, const int64_t *n_correct, const int64_t *n_params, int32_t *exit_out);

/* ---- Profiler and Partitioner ("Modules", Algorithm 1): host functions, no device work ---------
 * The Profiler's measured memory is replaced by the exact device bytes of one local step with
 * this library: parameters + gradients (+ momentum buffers) of the layer and its head, the input,
 * shortcut and emitted batches, labels, and nf_workspace_bytes.  nf_fit_linear is the Profiler's
 * linear model (least squares: bytes ~ intercept + slope * batch); nf_profile_layer evaluates the
 * byte count at n (2..64) batch sizes and fits it.  nf_partition is Algorithm 1: per layer the
 * largest batch size whose model stays within the budget M (same unit as the models), capped at
 * B_limit; then consecutive layers are grouped into one block while
 * |b[i+1] - b[i]| <= rho * b[i], a block taking the smallest batch size of its layers.
 * Outputs: layer_batch[n_layers] (optional), block_first[k] = index of the first layer of block
 * k and block_batch[k] (arrays of n_layers entries), *n_blocks.  A layer that does not fit at
 * batch size 1 gets batch size 0. */
typedef struct {
  double slope, intercept;
} nf_linear_model;
int32_t nf_layer_step_bytes(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B, int32_t with_momentum,
                            size_t *out);
int32_t nf_fit_linear(int32_t n, const double *batch, const double *bytes, nf_linear_model *out);
int32_t nf_profile_layer(const nf_layer_desc *d, const nf_aux_desc *a, int32_t with_momentum, int32_t n,
                         const int32_t *batches, nf_linear_model *out);
int32_t nf_partition(int32_t n_layers, const nf_linear_model *R, double M, int32_t B_limit, double rho,
                     int32_t *layer_batch, int32_t *block_first, int32_t *block_batch, int32_t *n_blocks);

/* ---- measurement aid (not a step of the method) ---------------------------------------------
 * Between nf_prof_begin and nf_prof_end every kernel the library enqueues is bracketed by a
 * HIP-event pair on the caller's stream.  nf_prof_end waits for those events (the only call
 * that blocks the host), and returns one record per kernel: launches, summed duration (ms),
 * summed algorithmic FLOPs and bytes.  Records are sorted by duration, at most `cap` are
 * written, *n receives the number of distinct kernels.  Process-wide state (one recording at a time;
 * the record list is guarded by a mutex so that launches from several host threads may be recorded),
 * creates HIP events: keep it out of production loops. */
typedef struct {
  char kernel[48];
  int64_t launches;
  double ms, flops, bytes;
} nf_prof_record;
/* Compute units and peak shader clock (kHz) of the current device, as the runtime reports them
 * (the fp32 MFMA peak is compute_units x 4 SIMDs x 64 flop/clk x clock). */
int32_t nf_device_info(int32_t *compute_units, int32_t *clock_khz);
int32_t nf_prof_begin(void);
int32_t nf_prof_end(nf_prof_record *out, int32_t cap, int32_t *n);

#ifdef __cplusplus
}
#endif
#endif
