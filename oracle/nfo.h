/*
 * nfo — CPU oracle for the per-layer local training step of adaptive local learning
 * (NeuroFlux, arXiv 2402.14139: Eq. 1-3, Algorithm 2, and the activation cache of
 * the "Efficient Forward Propagation via Prefetching and Adaptive Batching" section).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, loop-by-loop
 * statement of what the method computes, used only to check the GPU library and as a
 * timed host baseline.  It shares no code with the GPU library.
 *
 * Conventions
 *   - logical NCHW activations, OIHW convolution weights, row-major [out][in] linear
 *     weights, int32 labels; every pointer is a HOST pointer owned by the caller.
 *   - every function exists for T = float (suffix _f32) and T = double (suffix _f64).
 *     Sums are always accumulated in double and rounded to T once when stored.
 *   - nothing is allocated that outlives a call; nothing is kept between calls.
 *
 * Parity pins (tests, CPU only): central finite differences of the loss in f64, a
 * PyTorch-autograd (f64, CPU) evaluation of the same step, the closed form
 * loss = ln(n_classes) at zero linear weights, the activation-size series of the
 * paper's Fig. 13 (left), and the invariants/special cases listed in the tests.  The
 * max-pooling head and the squared-error loss have the same two pins (finite differences,
 * autograd) plus loss = 1/n_classes at zero linear weights and quadrant maxima on even maps.
 * Unpinned: nothing below is "parity unpinned"; absolute values for any particular
 * seeded configuration are defined only by this oracle plus the input generator.
 */
#ifndef NFO_H
#define NFO_H
#include <stdint.h>
#ifdef __cplusplus
extern "C" {
#endif

/* Layer n of Eq. 1: x_{n+1} = ReLU( P_n ( theta_n * x_n + b [+ skip] ) ). */
typedef struct {
  int32_t C_in, H_in, W_in;      /* input x_n                                        */
  int32_t C_out, R, S, stride, pad; /* convolution theta_n                           */
  int32_t pool_kind;             /* P_n: 0 none, 1 max-pool                          */
  int32_t pool_k, pool_stride, pool_pad;
  int32_t skip_kind;             /* 0 none, 1 identity add, 2 1x1 strided projection */
  int32_t skip_C, skip_H, skip_W, skip_stride;
} nfo_layer_desc;

/* Auxiliary head A_n of Eq. 2: z = gamma_n F_n beta_n x_{n+1}:
 * conv (beta, + bias, optional ReLU), adaptive pooling F_n to pool_oh x pool_ow (average, or
 * max -- the two down-sampling mechanisms the paper names), one linear layer to n_classes.
 * C_in/H_in/W_in are the layer's emitted tensor.  The loss l of Eq. 3 is cross-entropy or the
 * mean squared error against the one-hot label (the two losses the paper names). */
typedef struct {
  int32_t C_in, H_in, W_in;
  int32_t A, R, S, pad, relu;
  int32_t pool_oh, pool_ow;
  int32_t n_classes;
  int32_t head_pool;             /* F_n: 0 adaptive average pool, 1 adaptive max pool */
  int32_t loss_kind;             /* l:   0 softmax cross-entropy, 1 mean squared error  */
} nfo_aux_desc;

/* conv output (Ho,Wo) and emitted, post-pool (Hp,Wp) sizes; returns 0, or -1 if the
 * descriptor is not meaningful (non-positive sizes, pool padding > pool_k/2, ...). */
int32_t nfo_layer_dims(const nfo_layer_desc *d, int32_t *Ho, int32_t *Wo, int32_t *Hp, int32_t *Wp);

int32_t nfo_num_threads(void);           /* threads the OpenMP loops will use */
void nfo_set_num_threads(int32_t n);

#define NFO_DECLARE(T, SUF)                                                                    \
  /* Eq. 1.  Z = conv + bias (+ skip), pre-activation [B,K,Ho,Wo]; Y emitted [B,K,Hp,Wp];   */ \
  /* arg[B,K,Hp,Wp] = flat index (h*Wo+w) of the first maximal element of each pool window  */ \
  /* (unused, may be NULL, when pool_kind==0).                                              */ \
  void nfo_layer_fwd_##SUF(const nfo_layer_desc *d, int32_t B, const T *x, const T *x_skip,    \
                           const T *W, const T *b, const T *Wp, T *Z, T *Y, int32_t *arg);     \
  /* Eq. 2 + Eq. 3 (batch mean of the loss).  U[B,A,H,W] post-ReLU aux conv output,         */ \
  /* Pq[B,A*oh*ow] pooled features (flatten order a,i,j), z[B,Cls] logits, *loss the batch  */ \
  /* mean, dz[B,Cls] = d loss / d z.  Upre (optional) receives the aux conv output before   */ \
  /* its ReLU; parg (optional, used when head_pool==1) [B,A*oh*ow] the flat position h*W+w  */ \
  /* of the first maximal element of each pooling window.                                   */ \
  void nfo_aux_fwd_loss_##SUF(const nfo_aux_desc *a, int32_t B, const T *y,                    \
                              const int32_t *labels, const T *Wa, const T *ba, const T *Wf,    \
                              const T *bf, T *U, T *Pq, T *z, double *loss, T *dz, T *Upre,    \
                              int32_t *parg);                                                  \
  /* Algorithm 2, "compute the gradient w.r.t. (theta_n, beta_n, gamma_n)".  Consumes what  */ \
  /* the two forward calls produced.  dY/dZ are optional outputs (may be NULL).  No         */ \
  /* gradient is formed for x or x_skip.  dWp may be NULL unless skip_kind==2.              */ \
  /* mask_u [B,A,Hu,Wu] / mask_z [B,K,Ho,Wo] (optional, 0/1 bytes) replace the decisions    */ \
  /* "U > 0" / "Z > 0" of the two ReLU derivatives; `arg` is an input in any case.  They let */ \
  /* a comparison hand over the branch taken by an implementation that accumulates in        */ \
  /* another precision, for pre-activations that are zero to within rounding.  parg is the   */ \
  /* max-pooling selection of the head (required when head_pool==1; ignored otherwise).      */ \
  void nfo_local_bwd_##SUF(const nfo_layer_desc *d, const nfo_aux_desc *a, int32_t B,          \
                           const T *x, const T *x_skip, const T *Z, const T *Y,                \
                           const int32_t *arg, const T *U, const T *Pq, const T *dz,           \
                           const T *Wa, const T *Wf, T *dW, T *db, T *dWp, T *dWa, T *dba,     \
                           T *dWf, T *dbf, T *dY, T *dZ, const uint8_t *mask_u,                \
                           const uint8_t *mask_z, const int32_t *parg);                        \
  /* Algorithm 2, "update": v = mu*v + g ; w = w - lr*v.  v==NULL or mu==0: w = w - lr*g.   */ \
  void nfo_sgd_update_##SUF(int64_t numel, T *w, const T *g, T *v, double lr, double mu);      \
  /* Activation cache: row r of `cache` is one sample (sample_elems values).               */  \
  void nfo_cache_write_##SUF(T *cache, int32_t *cache_labels, int64_t sample_elems,            \
                             int64_t first, int32_t B, const T *y, const int32_t *labels);     \
  void nfo_cache_read_##SUF(const T *cache, const int32_t *cache_labels, int64_t sample_elems, \
                            int64_t first, const int64_t *idx, int32_t B, T *x_out,            \
                            int32_t *labels_out);                                              \
  /* One whole pass of the Algorithm 2 body for one (batch, layer): forward, head, loss,    */ \
  /* gradients, update (in place), and the emitted Y computed with the PRE-update weights.  */ \
  /* Gradient outputs are optional (NULL to skip); momentum buffers NULL when mu==0.        */ \
  void nfo_local_step_##SUF(const nfo_layer_desc *d, const nfo_aux_desc *a, int32_t B,         \
                            const T *x, const T *x_skip, const int32_t *labels, T *W, T *b,    \
                            T *Wp, T *Wa, T *ba, T *Wf, T *bf, T *gW, T *gb, T *gWp, T *gWa,   \
                            T *gba, T *gWf, T *gbf, T *vW, T *vb, T *vWp, T *vWa, T *vba,      \
                            T *vWf, T *vbf, double lr, double mu, T *Y, double *loss);

NFO_DECLARE(float, f32)
NFO_DECLARE(double, f64)

#ifdef __cplusplus
}
#endif
#endif
