// C-ABI entry points of libnf (include/nf.h): argument validation, workspace layout and the
// order in which the kernels of one local training step are enqueued (body of Algorithm 2,
// NeuroFlux, arXiv 2402.14139).  No device work is enqueued before validation has passed.
#include <algorithm>
#include <atomic>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "nf_internal.h"

// Scratch of nf_local_step_static: one copy per GPU the library runs on, held until the process
// ends.  In host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[NF_STATIC_SCRATCH_BYTES];

namespace nf {

std::atomic<int> g_contraction{NF_CONTRACT_F32};
int contraction_mode() { return g_contraction.load(std::memory_order_relaxed); }
namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct LayerDims {
  int Ho, Wo, Hp, Wp;
};

int32_t check_layer(const nf_layer_desc *d, LayerDims *o) {
  if (!d) return NF_ERR_NULL;
  if (d->C_in <= 0 || d->H_in <= 0 || d->W_in <= 0 || d->C_out <= 0 || d->R <= 0 || d->S <= 0 || d->stride <= 0 ||
      d->pad < 0)
    return NF_ERR_BAD_DESC;
  if (d->R > 15 || d->S > 15 || d->stride > 4 || d->pad >= d->R + d->S) return NF_ERR_UNSUPPORTED;
  const int hn = d->H_in + 2 * d->pad - d->R, wn = d->W_in + 2 * d->pad - d->S;
  if (hn < 0 || wn < 0) return NF_ERR_BAD_DESC;
  o->Ho = hn / d->stride + 1;
  o->Wo = wn / d->stride + 1;
  o->Hp = o->Ho;
  o->Wp = o->Wo;
  if (d->pool_kind != 0) {
    if (d->pool_kind != 1) return NF_ERR_UNSUPPORTED;
    if (d->pool_k <= 0 || d->pool_stride <= 0 || d->pool_pad < 0 || 2 * d->pool_pad > d->pool_k)
      return NF_ERR_BAD_DESC;
    if (d->pool_k > 15) return NF_ERR_UNSUPPORTED;
    const int ph = o->Ho + 2 * d->pool_pad - d->pool_k, pw = o->Wo + 2 * d->pool_pad - d->pool_k;
    if (ph < 0 || pw < 0) return NF_ERR_BAD_DESC;
    o->Hp = ph / d->pool_stride + 1;
    o->Wp = pw / d->pool_stride + 1;
  }
  if (d->skip_kind == 1) {
    if (d->skip_C != d->C_out || d->skip_H != o->Ho || d->skip_W != o->Wo) return NF_ERR_BAD_DESC;
  } else if (d->skip_kind == 2) {
    if (d->skip_C <= 0 || d->skip_stride <= 0 || d->skip_H <= 0 || d->skip_W <= 0) return NF_ERR_BAD_DESC;
    if ((long long)(o->Ho - 1) * d->skip_stride >= d->skip_H || (long long)(o->Wo - 1) * d->skip_stride >= d->skip_W)
      return NF_ERR_BAD_DESC;
  } else if (d->skip_kind != 0) {
    return NF_ERR_BAD_DESC;
  }
  return NF_OK;
}

struct AuxDims {
  int Hu, Wu, F;
};

int32_t check_aux(const nf_aux_desc *a, AuxDims *o) {
  if (!a) return NF_ERR_NULL;
  if (a->C_in <= 0 || a->H_in <= 0 || a->W_in <= 0 || a->A <= 0 || a->R <= 0 || a->S <= 0 || a->pad < 0 ||
      a->pool_oh <= 0 || a->pool_ow <= 0 || a->n_classes <= 0)
    return NF_ERR_BAD_DESC;
  if (a->R != a->S || a->R > 15 || a->pad > a->R - 1) return NF_ERR_UNSUPPORTED;
  if (a->head_pool < 0 || a->head_pool > 1 || a->loss_kind < 0 || a->loss_kind > 1) return NF_ERR_UNSUPPORTED;
  o->Hu = a->H_in + 2 * a->pad - a->R + 1;
  o->Wu = a->W_in + 2 * a->pad - a->S + 1;
  if (o->Hu <= 0 || o->Wu <= 0) return NF_ERR_BAD_DESC;
  const long long F = (long long)a->A * a->pool_oh * a->pool_ow;
  if (F > 4096 || a->n_classes > 4096) return NF_ERR_UNSUPPORTED;
  o->F = (int)F;
  return NF_OK;
}

// every index the kernels form in 32-bit must fit
int32_t check_sizes(const nf_layer_desc *d, const LayerDims &ld, int32_t B) {
  if (B <= 0) return NF_ERR_BAD_DESC;
  const long long lim = (1ll << 31) - 1;
  const long long pix_in = (long long)B * d->H_in * d->W_in, pix_out = (long long)B * ld.Ho * ld.Wo;
  const long long pix_skip = d->skip_kind == 2 ? (long long)B * d->skip_H * d->skip_W : 0;
  if (pix_in > lim || pix_out > lim || pix_skip > lim) return NF_ERR_UNSUPPORTED;
  if ((long long)d->R * d->S * d->C_in + d->skip_C > lim / 4) return NF_ERR_UNSUPPORTED;
  if (B > 65535) return NF_ERR_UNSUPPORTED;
  return NF_OK;
}

// shape part of the aux convolution's weight-gradient problem (pointers and splits left to the caller)
WgradProblem aux_wgrad_shape(const nf_aux_desc *a, const AuxDims &ad, int B) {
  WgradProblem g;
  std::memset((void *)&g, 0, sizeof(g));
  g.H = a->H_in, g.W = a->W_in, g.C = a->C_in, g.R = a->R, g.S = a->S, g.stride = 1, g.pad = a->pad, g.Ho = ad.Hu,
  g.Wo = ad.Wu;
  g.P = a->A, g.M = B * ad.Hu * ad.Wu, g.RSC = a->R * a->S * a->C_in, g.Q = g.RSC;
  g.div_howo = FastDiv(ad.Hu * ad.Wu), g.div_wo = FastDiv(ad.Wu);
  return g;
}

HeadShape head_shape(const nf_aux_desc *a, const AuxDims &ad, int B) {
  HeadShape h;
  h.B = B, h.Hu = ad.Hu, h.Wu = ad.Wu, h.A = a->A, h.oh = a->pool_oh, h.ow = a->pool_ow, h.F = ad.F,
  h.Cls = a->n_classes, h.relu = a->relu, h.pmax = a->head_pool == 1, h.mse = a->loss_kind == 1;
  return h;
}

// beta_n of Eq. 2 as a forward-type contraction (pointers left null)
FwdProblem aux_fwd_problem(const nf_aux_desc *a, const AuxDims &ad, int B) {
  FwdProblem f;
  std::memset((void *)&f, 0, sizeof(f));
  f.H = a->H_in, f.W = a->W_in, f.C = a->C_in, f.N = a->A, f.R = a->R, f.S = a->S, f.stride = 1, f.pad = a->pad,
  f.Ho = ad.Hu, f.Wo = ad.Wu;
  f.relu = a->relu ? 1 : 0;
  f.M = B * ad.Hu * ad.Wu, f.RSC = a->R * a->S * a->C_in, f.Kg = f.RSC;
  f.div_howo = FastDiv(ad.Hu * ad.Wu), f.div_wo = FastDiv(ad.Wu);
  return f;
}

struct WsLayout {
  size_t T_dZ, arg, U, Pq, parg, dz, loss_n, dPq, dU, WaT, dY, part, part_b, part_aux, part_b_aux, ppart, total;
  int splits_aux, splits_layer, Qld_aux, Qld_layer;
  // reduction splits of the forward-type contractions (1 = none); their partial sums alias `part`
  int ksplits_aux, ksplits_layer, ksplits_dgrad;
  // 1: the head's per-sample chain (pooling ... dU) runs as one launch right after its convolution;
  // 2: as two (pooling; everything else).  In both the batch-reducing rest (gamma_n's gradient,
  // batch-mean loss) rides on the reduction launch.  0: pooling, linear layer + loss, backward.
  int head_fused;
  // head_fused == 2 only: F_n is formed from column sums left by the aux convolution's epilogue
  // (region ppart), no pooling launch
  int pool_fused;
};

WsLayout ws_layout(const nf_layer_desc *d, const LayerDims &ld, const nf_aux_desc *a, const AuxDims &ad, int B) {
  WsLayout w;
  std::memset(&w, 0, sizeof(w));
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t at = off;
    off += up(bytes);
    return at;
  };
  const size_t f = sizeof(float);
  const bool pooled = d->pool_kind != 0;
  const size_t conv_out = (size_t)B * ld.Ho * ld.Wo * d->C_out, emitted = (size_t)B * ld.Hp * ld.Wp * d->C_out;
  // pre-pool activation in the forward, dL/d(conv output) in the backward: never live together
  w.T_dZ = take((pooled || a) ? conv_out * f : 0);
  w.arg = take(pooled ? emitted : 0);
  const int Kl = d->R * d->S * d->C_in + (d->skip_kind == 2 ? d->skip_C : 0);
  w.ksplits_layer = igemm_fwd_pick_ksplits(B * ld.Ho * ld.Wo, d->C_out, Kl, d->C_in, d->R * d->S);
  size_t pmax = w.ksplits_layer > 1 ? (size_t)w.ksplits_layer * conv_out : 0;
  w.ksplits_aux = w.ksplits_dgrad = 1;
  if (a) {
    const size_t u = (size_t)B * ad.Hu * ad.Wu * a->A;
    w.U = take(u * f);
    w.Pq = take((size_t)B * ad.F * f);
    w.parg = take(a->head_pool == 1 ? (size_t)B * ad.F * sizeof(int32_t) : 0);
    w.dz = take((size_t)B * a->n_classes * f);
    w.loss_n = take((size_t)B * f);
    w.dPq = take((size_t)B * ad.F * f);
    w.dU = take(u * f);
    w.WaT = take((size_t)a->A * a->R * a->S * a->C_in * f);
    w.dY = take(pooled ? emitted * f : 0);
    const int Qa = a->R * a->S * a->C_in;
    w.Qld_aux = (Qa + 3) / 4 * 4;
    w.Qld_layer = (Kl + 3) / 4 * 4;
    w.splits_aux = igemm_wgrad_small_applicable(aux_wgrad_shape(a, ad, B))
                       ? igemm_wgrad_small_splits(a->A, a->C_in, B, a->H_in)
                       : wgrad_pick_splits(a->A, Qa, B * ad.Hu * ad.Wu);
    w.splits_layer = wgrad_pick_splits(d->C_out, Kl, B * ld.Ho * ld.Wo);
    // split partials of the two weight gradients live side by side: one launch reduces both
    const size_t pa = (size_t)w.splits_aux * a->A * w.Qld_aux, pl = (size_t)w.splits_layer * d->C_out * w.Qld_layer;
    if (pl > pmax) pmax = pl;
    // partials of the aux forward are dead before the backward; those of the data gradient are
    // dead before the layer's weight gradient overwrites them
    w.ksplits_aux = igemm_fwd_pick_ksplits(B * ad.Hu * ad.Wu, a->A, Qa, a->C_in, a->R * a->S);
    if (w.ksplits_aux > 1 && (size_t)w.ksplits_aux * u > pmax) pmax = (size_t)w.ksplits_aux * u;
    w.ksplits_dgrad = igemm_fwd_pick_ksplits(B * a->H_in * a->W_in, a->C_in, a->R * a->S * a->A, a->A, a->R * a->S);
    if (w.ksplits_dgrad > 1 && (size_t)w.ksplits_dgrad * emitted > pmax) pmax = (size_t)w.ksplits_dgrad * emitted;
    w.head_fused = head_sample_applicable(head_shape(a, ad, B)) ? 1 : head_wide_applicable(head_shape(a, ad, B)) ? 2 : 0;
    if (w.head_fused == 2 && head_pool_partials_applicable(head_shape(a, ad, B))) {
      // (a reduction split in two gives way: the pooling launch it would need costs more than it gains)
      FwdProblem fp = aux_fwd_problem(a, ad, B);
      fp.ksplits = w.ksplits_aux <= 2 ? 1 : w.ksplits_aux;
      w.pool_fused = fwd_pool_partials_applicable(fp) ? 1 : 0;
      if (w.pool_fused) w.ksplits_aux = 1;
    }
    w.ppart = take(w.pool_fused ? (size_t)B * ad.Hu * ad.Wu / 16 * 2 * a->A * f : 0);
    w.part_b = take((size_t)w.splits_layer * d->C_out * f);
    w.part_aux = take(pa * f);
    w.part_b_aux = take((size_t)w.splits_aux * a->A * f);
  }
  w.part = take(pmax * f);
  w.total = off ? off : ALIGN;
  return w;
}

int32_t check_ws(const void *ws, size_t have, size_t need) {
  if (!ws) return NF_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) % ALIGN) return NF_ERR_WORKSPACE;
  if (have < need) return NF_ERR_WORKSPACE;
  return NF_OK;
}

inline float *wsf(void *ws, size_t off) { return reinterpret_cast<float *>(static_cast<char *>(ws) + off); }

// A HIP error while enqueueing is reported on stderr with the failing expression (the status code
// alone cannot say which launch it was), then returned as NF_ERR_DEVICE.
#define NF_HIP(expr)                                                                     \
  do {                                                                                   \
    const hipError_t e_ = (expr);                                                        \
    if (e_ != hipSuccess) {                                                              \
      std::fprintf(stderr, "libnf: %s: %s\n", hipGetErrorString(e_), #expr);             \
      return NF_ERR_DEVICE;                                                              \
    }                                                                                    \
  } while (0)

// ---- optional kernel timing (nf_prof_begin / nf_prof_end): one HIP-event pair per launch ----
struct ProfEvent {
  const char *name;
  hipEvent_t a, b;
  double flops, bytes;
};
struct ProfState {
  bool on = false;
  std::vector<ProfEvent> ev;
  std::mutex mu;  // guards ev: launches from several host threads may record while profiling is on
};
ProfState g_prof;

struct ProfScope {
  hipStream_t st;
  hipEvent_t a = nullptr, b = nullptr;
  bool on;
  explicit ProfScope(hipStream_t s) : st(s), on(g_prof.on) {
    if (on) {
      on = hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess && hipEventRecord(a, st) == hipSuccess;
    }
  }
  void done(const char *name, double flops, double bytes) {
    if (on && hipEventRecord(b, st) == hipSuccess) {
      std::lock_guard<std::mutex> lk(g_prof.mu);
      g_prof.ev.push_back({name, a, b, flops, bytes});
    }
  }
};

// ---- enqueue helpers (arguments already validated) ----

#define NF_RUN(st, name, flops, bytes, call) \
  do {                                       \
    ProfScope sc_(st);                       \
    NF_HIP(call);                            \
    sc_.done(name, flops, bytes);            \
  } while (0)

// algorithmic work of the two contractions (dense formula: padding taps counted, tile padding not)
int32_t enqueue_fwd(const FwdProblem &f, hipStream_t st) {
  const double B = (double)f.M / ((double)f.Ho * f.Wo);
  const double flops = 2.0 * f.M * f.N * f.Kg;
  double elems = B * f.H * f.W * f.C + (double)f.N * f.Kg + (double)f.M * f.N;
  if (f.Cs) elems += B * f.Hs * f.Ws * f.Cs;
  if (f.addsrc) elems += (double)f.M * f.N;
  if (f.mask) elems += (double)f.M * f.N;
  ProfScope sc(st);
  const char *kn = "igemm_fwd";
  NF_HIP(launch_igemm_fwd(f, st, &kn));
  sc.done(kn, flops, 4.0 * elems);
  return NF_OK;
}

// forward-type contraction into `out`; with ksplits > 1 (and the fast path available) the
// reduction is split into `part` and a small kernel applies the epilogue
int32_t enqueue_fwd_split(FwdProblem f, float *out, int ksplits, float *part, hipStream_t st) {
  if (ksplits > 1 && igemm_fwd_fast_applicable(f)) {
    const float *bias = f.bias, *addsrc = f.addsrc, *mask = f.mask;
    const int relu = f.relu;
    f.ksplits = ksplits, f.out = part;
    const int32_t rc = enqueue_fwd(f, st);
    if (rc) return rc;
    const double mn = (double)f.M * f.N;
    NF_RUN(st, "fwd_finish", 0.0, 4.0 * mn * (ksplits + 1.0 + (addsrc ? 1.0 : 0.0) + (mask ? 1.0 : 0.0)),
           launch_fwd_finish(part, ksplits, f.M, f.N, bias, addsrc, mask, relu, out, st));
    return NF_OK;
  }
  f.ksplits = 0, f.out = out;
  return enqueue_fwd(f, st);
}

int32_t enqueue_wgrad(const WgradProblem &g, hipStream_t st) {
  const double B = (double)g.M / ((double)g.Ho * g.Wo);
  const double flops = 2.0 * g.M * g.P * g.Q;
  double elems = (double)g.M * g.P + B * g.H * g.W * g.C + (double)g.P * g.Q;
  if (g.Cs) elems += B * g.Hs * g.Ws * g.Cs;
  ProfScope sc(st);
  const char *kn = "igemm_wgrad";
  NF_HIP(launch_igemm_wgrad(g, st, &kn));
  sc.done(kn, flops, 4.0 * elems);
  return NF_OK;
}

WgradReduce reduce_job(const WgradProblem &g, float *out0, float *out1, float *ob) {
  WgradReduce j;
  std::memset((void *)&j, 0, sizeof(j));
  j.part = g.part, j.part_b = g.part_b, j.splits = g.splits, j.P = g.P, j.Q = g.Q, j.Qld = g.Qld, j.Q0 = g.RSC;
  j.out0 = out0, j.out1 = out1, j.ob = ob;
  return j;
}

int32_t run_layer_fwd(const nf_layer_desc *d, const LayerDims &ld, int B, const float *x, const float *xs,
                      const nf_layer_params *p, float *y, void *ws, const WsLayout &w, hipStream_t st) {
  const bool pooled = d->pool_kind != 0;
  FwdProblem f;
  std::memset((void *)&f, 0, sizeof(f));
  f.x = x, f.w = p->W, f.bias = p->b;
  f.H = d->H_in, f.W = d->W_in, f.C = d->C_in, f.N = d->C_out, f.R = d->R, f.S = d->S, f.stride = d->stride,
  f.pad = d->pad, f.Ho = ld.Ho, f.Wo = ld.Wo;
  if (d->skip_kind == 1) f.addsrc = xs;
  if (d->skip_kind == 2) f.xs = xs, f.wp = p->Wp, f.Cs = d->skip_C, f.Hs = d->skip_H, f.Ws = d->skip_W, f.ss = d->skip_stride;
  f.relu = 1;
  f.M = B * ld.Ho * ld.Wo, f.RSC = d->R * d->S * d->C_in, f.Kg = f.RSC + f.Cs;
  f.div_howo = FastDiv(ld.Ho * ld.Wo), f.div_wo = FastDiv(ld.Wo);
  float *conv_out = pooled ? wsf(ws, w.T_dZ) : y;
  int32_t rc = enqueue_fwd_split(f, conv_out, w.ksplits_layer, wsf(ws, w.part), st);
  if (rc) return rc;
  if (pooled) {
    const double pre = (double)B * ld.Ho * ld.Wo * d->C_out, post = (double)B * ld.Hp * ld.Wp * d->C_out;
    NF_RUN(st, "maxpool_fwd", 0.0, 4.0 * pre + 5.0 * post,
           launch_maxpool_fwd(wsf(ws, w.T_dZ), y, reinterpret_cast<uint8_t *>(wsf(ws, w.arg)), B, ld.Ho, ld.Wo,
                              d->C_out, ld.Hp, ld.Wp, d->pool_k, d->pool_stride, d->pool_pad, st));
  }
  return NF_OK;
}

// beta_n and F_n of Eq. 2: the head's convolution (+ bias, ReLU) and its pooling; leaves U and Pq
// (and the max-pooling selection) in the workspace
int32_t run_aux_features(const nf_aux_desc *a, const AuxDims &ad, int B, const float *y, const nf_aux_params *ap,
                         void *ws, const WsLayout &w, hipStream_t st, bool partials_only = false) {
  FwdProblem f = aux_fwd_problem(a, ad, B);
  f.x = y, f.w = ap->Wa, f.bias = ap->ba;
  // skinny head, long reduction: split it; the pooling kernel adds the parts, bias and ReLU
  const int ks = (w.ksplits_aux > 1 && igemm_fwd_fast_applicable(f)) ? w.ksplits_aux : 0;
  f.ksplits = ks;
  f.out = ks ? wsf(ws, w.part) : wsf(ws, w.U);
  // partials_only (the caller's next launch forms F_n itself): the convolution's epilogue leaves
  // the column sums per 16 pixels, and there is no pooling launch
  const bool fused = partials_only && w.pool_fused;
  if (fused) f.pool_part = wsf(ws, w.ppart), f.pool_split = ad.Wu == 16 ? 1 : 0;
  int32_t rc = enqueue_fwd(f, st);
  if (rc) return rc;
  if (fused) return NF_OK;
  const HeadShape hs = head_shape(a, ad, B);
  const double u = (double)B * ad.Hu * ad.Wu * a->A;
  NF_RUN(st, "head_pool", 0.0, 4.0 * (u * (ks ? ks + 1.0 : 1.0) + (double)B * ad.F),
         launch_head_pool(hs, wsf(ws, w.U), wsf(ws, w.part), ks, ap->ba, wsf(ws, w.Pq),
                          reinterpret_cast<int32_t *>(wsf(ws, w.parg)), st));
  return NF_OK;
}

// loss_out == nullptr: the batch mean is left to the backward launch that follows (run_bwd)
int32_t run_aux_fwd(const nf_aux_desc *a, const AuxDims &ad, int B, const float *y, const int32_t *labels,
                    const nf_aux_params *ap, float *loss_out, void *ws, const WsLayout &w, hipStream_t st) {
  const HeadShape hs = head_shape(a, ad, B);
  if (w.head_fused == 1) {
    // small activation map: the convolution, then ONE launch for the head's whole per-sample chain
    // (F_n, gamma_n, loss, dL/dz, dPq, dU) and the re-laid filter the data gradient will read
    FwdProblem f;
    std::memset((void *)&f, 0, sizeof(f));
    f.x = y, f.w = ap->Wa, f.bias = ap->ba;
    f.H = a->H_in, f.W = a->W_in, f.C = a->C_in, f.N = a->A, f.R = a->R, f.S = a->S, f.stride = 1, f.pad = a->pad,
    f.Ho = ad.Hu, f.Wo = ad.Wu;
    f.relu = a->relu ? 1 : 0;
    f.M = B * ad.Hu * ad.Wu, f.RSC = a->R * a->S * a->C_in, f.Kg = f.RSC;
    f.div_howo = FastDiv(ad.Hu * ad.Wu), f.div_wo = FastDiv(ad.Wu);
    // skinny head, long reduction: split it; the per-sample launch adds the parts, bias and ReLU
    const int ks = (w.ksplits_aux > 1 && igemm_fwd_fast_applicable(f)) ? w.ksplits_aux : 0;
    f.ksplits = ks;
    f.out = ks ? wsf(ws, w.part) : wsf(ws, w.U);
    int32_t rc = enqueue_fwd(f, st);
    if (rc) return rc;
    const double u = (double)B * ad.Hu * ad.Wu * a->A, fc = (double)a->n_classes * ad.F;
    const double wa = (double)a->A * a->R * a->S * a->C_in;
    NF_RUN(st, "head_sample", 4.0 * B * fc,
           4.0 * ((3.0 + ks) * u + 2.0 * B * fc + (double)B * (ad.F + a->n_classes + 1.0)) + 8.0 * wa,
           launch_head_sample(hs, wsf(ws, w.U), wsf(ws, w.part), ks, ap->ba, labels, ap->Wf, ap->bf, wsf(ws, w.Pq),
                              reinterpret_cast<int32_t *>(wsf(ws, w.parg)), wsf(ws, w.dz), wsf(ws, w.loss_n),
                              wsf(ws, w.dU), ap->Wa, wsf(ws, w.WaT), a->R, a->S, a->C_in, st));
    if (loss_out) NF_RUN(st, "loss_mean", 0.0, 4.0 * B, launch_loss_mean(wsf(ws, w.loss_n), B, loss_out, st));
    return NF_OK;
  }
  int32_t rc = run_aux_features(a, ad, B, y, ap, ws, w, st, w.head_fused == 2);
  if (rc) return rc;
  const double fc = (double)a->n_classes * ad.F;
  if (w.head_fused == 2) {
    // large activation map, small linear layer: ONE more launch for gamma_n, loss, dL/dz, dPq and dU
    const double u = (double)B * ad.Hu * ad.Wu * a->A, wa = (double)a->A * a->R * a->S * a->C_in;
    NF_RUN(st, "head_wide", 4.0 * B * fc, 4.0 * (2.0 * u + (double)B * (ad.F + a->n_classes + 1.0)) + 8.0 * wa,
           launch_head_wide(hs, wsf(ws, w.U), wsf(ws, w.Pq), w.pool_fused ? wsf(ws, w.ppart) : nullptr, labels, ap->Wf, ap->bf, wsf(ws, w.dz), wsf(ws, w.loss_n),
                            reinterpret_cast<const int32_t *>(wsf(ws, w.parg)), wsf(ws, w.dU), ap->Wa, wsf(ws, w.WaT),
                            a->R, a->S, a->C_in, st));
    if (loss_out) NF_RUN(st, "loss_mean", 0.0, 4.0 * B, launch_loss_mean(wsf(ws, w.loss_n), B, loss_out, st));
    return NF_OK;
  }
  NF_RUN(st, "head_fc", 4.0 * B * fc, 4.0 * (2.0 * B * fc + (double)B * (2.0 * ad.F + a->n_classes)),
         launch_head_fc(hs, wsf(ws, w.Pq), labels, ap->Wf, ap->bf, wsf(ws, w.dz), wsf(ws, w.loss_n), wsf(ws, w.dPq), st));
  if (loss_out) NF_RUN(st, "loss_mean", 0.0, 4.0 * B, launch_loss_mean(wsf(ws, w.loss_n), B, loss_out, st));
  return NF_OK;
}

int32_t run_bwd(const nf_layer_desc *d, const LayerDims &ld, const nf_aux_desc *a, const AuxDims &ad, int B,
                const float *x, const float *xs, const float *y, const nf_layer_params *p,
                const nf_aux_params *ap, const nf_layer_params *gp, const nf_aux_params *ga, float *loss_out,
                const nf_sgd_desc *sgd, const nf_layer_params *vp, const nf_aux_params *va, void *ws,
                const WsLayout &w, hipStream_t st) {
  // sgd != nullptr: the update line of Algorithm 2 is applied by the launch that finishes the
  // gradients (nothing reads the parameters after the data gradient)
  ReduceSgd red;
  std::memset((void *)&red, 0, sizeof(red));
  const bool pooled = d->pool_kind != 0;
  const HeadShape hs = head_shape(a, ad, B);
  float *dU = wsf(ws, w.dU), *dZ = wsf(ws, w.T_dZ);
  // gamma_n weight gradient, back through F_n and the aux ReLU (dPq came with the forward)
  const double u = (double)B * ad.Hu * ad.Wu * a->A, fc = (double)a->n_classes * ad.F;
  const double wa = (double)a->A * a->R * a->S * a->C_in;
  if (!w.head_fused)
    NF_RUN(st, "head_bwd", 2.0 * B * fc, 4.0 * (fc + (double)B * (2.0 * ad.F + a->n_classes) + 2.0 * u) + 8.0 * wa,
           launch_head_bwd(hs, wsf(ws, w.Pq), wsf(ws, w.dz), ga->Wf, ga->bf, wsf(ws, w.U), wsf(ws, w.dPq), dU, ap->Wa,
                           wsf(ws, w.WaT), a->R, a->S, a->C_in, wsf(ws, w.loss_n), loss_out,
                           reinterpret_cast<const int32_t *>(wsf(ws, w.parg)), st));
  // beta_n: weight + bias gradient
  {
    WgradProblem g = aux_wgrad_shape(a, ad, B);
    g.d = dU, g.x = y, g.part = wsf(ws, w.part_aux), g.part_b = wsf(ws, w.part_b_aux);
    g.Qld = w.Qld_aux;
    g.splits = w.splits_aux;
    g.m_per_split = ((g.M + g.splits - 1) / g.splits + 31) / 32 * 32;  // whole 32-row steps
    g.div_howo = FastDiv(ad.Hu * ad.Wu), g.div_wo = FastDiv(ad.Wu);
    const int32_t rc = enqueue_wgrad(g, st);
    if (rc) return rc;
    red.job[1] = reduce_job(g, ga->Wa, nullptr, ga->ba);
  }
  // beta_n: data gradient w.r.t. the emitted activation, layer ReLU mask fused when un-pooled
  {
    FwdProblem f;
    std::memset((void *)&f, 0, sizeof(f));
    f.x = dU, f.w = wsf(ws, w.WaT);
    f.H = ad.Hu, f.W = ad.Wu, f.C = a->A, f.N = a->C_in, f.R = a->R, f.S = a->S, f.stride = 1,
    f.pad = a->R - 1 - a->pad, f.Ho = a->H_in, f.Wo = a->W_in;
    f.M = B * a->H_in * a->W_in, f.RSC = a->R * a->S * a->A, f.Kg = f.RSC;
    f.div_howo = FastDiv(a->H_in * a->W_in), f.div_wo = FastDiv(a->W_in);
    f.mask = pooled ? nullptr : y;
    const int32_t rc = enqueue_fwd_split(f, pooled ? wsf(ws, w.dY) : dZ, w.ksplits_dgrad, wsf(ws, w.part), st);
    if (rc) return rc;
    if (pooled) {
      const double pre = (double)B * ld.Ho * ld.Wo * d->C_out, post = (double)B * ld.Hp * ld.Wp * d->C_out;
      NF_RUN(st, "maxpool_bwd", 0.0, 4.0 * pre + 9.0 * post,
             launch_maxpool_bwd(wsf(ws, w.dY), y, reinterpret_cast<const uint8_t *>(wsf(ws, w.arg)), dZ, B, ld.Ho,
                                ld.Wo, d->C_out, ld.Hp, ld.Wp, d->pool_k, d->pool_stride, d->pool_pad, st));
    }
  }
  // theta_n: weight, bias and projection gradients; nothing flows to x or x_skip
  {
    WgradProblem g;
    std::memset((void *)&g, 0, sizeof(g));
    g.d = dZ, g.x = x, g.part = wsf(ws, w.part), g.part_b = wsf(ws, w.part_b);
    g.H = d->H_in, g.W = d->W_in, g.C = d->C_in, g.R = d->R, g.S = d->S, g.stride = d->stride, g.pad = d->pad,
    g.Ho = ld.Ho, g.Wo = ld.Wo;
    if (d->skip_kind == 2) g.xs = xs, g.Cs = d->skip_C, g.Hs = d->skip_H, g.Ws = d->skip_W, g.ss = d->skip_stride;
    g.P = d->C_out, g.M = B * ld.Ho * ld.Wo, g.RSC = d->R * d->S * d->C_in, g.Q = g.RSC + g.Cs, g.Qld = w.Qld_layer;
    g.splits = w.splits_layer;
    g.m_per_split = ((g.M + g.splits - 1) / g.splits + 31) / 32 * 32;  // whole 32-row steps
    g.div_howo = FastDiv(ld.Ho * ld.Wo), g.div_wo = FastDiv(ld.Wo);
    const int32_t rc = enqueue_wgrad(g, st);
    if (rc) return rc;
    red.job[0] = reduce_job(g, gp->W, gp->Wp, gp->b);
  }
  red.njobs = 2;
  double nred = 0, nsgd = 0;
  for (int j = 0; j < 2; ++j) nred += ((double)red.job[j].splits + 1.0) * red.job[j].P * (red.job[j].Q + 1.0);
  if (sgd) {
    const bool mom = sgd->momentum != 0.f;
    red.lr = sgd->lr, red.mu = sgd->momentum;
    red.job[0].w0 = p->W, red.job[0].w1 = p->Wp, red.job[0].wb = p->b;
    red.job[1].w0 = ap->Wa, red.job[1].wb = ap->ba;
    if (mom) {
      red.job[0].v0 = vp->W, red.job[0].v1 = vp->Wp, red.job[0].vb = vp->b;
      red.job[1].v0 = va->Wa, red.job[1].vb = va->ba;
    }
    if (!w.head_fused) {
      red.nx = 2;
      red.xw[0] = ap->Wf, red.xg[0] = ga->Wf, red.xv[0] = mom ? va->Wf : nullptr, red.xn[0] = (long long)a->n_classes * ad.F;
      red.xw[1] = ap->bf, red.xg[1] = ga->bf, red.xv[1] = mom ? va->bf : nullptr, red.xn[1] = a->n_classes;
    }
    for (int j = 0; j < 2; ++j) nsgd += (double)red.job[j].P * (red.job[j].Q + 1.0);
    nsgd += fc + a->n_classes;
    nsgd *= mom ? 16.0 : 8.0;  // bytes beyond the gradient write
  }
  if (w.head_fused) {
    // gamma_n's gradient (a sum over the batch), its update and the batch-mean loss as extra
    // workgroups of this launch: the per-sample launch left Pq, dz and the per-sample losses
    GammaJob &gj = red.gamma;
    gj.B = B, gj.F = ad.F, gj.Cls = a->n_classes, gj.Pq = wsf(ws, w.Pq), gj.dz = wsf(ws, w.dz);
    gj.dWf = ga->Wf, gj.dbf = ga->bf;
    if (sgd) {
      gj.Wf = ap->Wf, gj.bf = ap->bf, gj.lr = sgd->lr, gj.mu = sgd->momentum;
      if (sgd->momentum != 0.f) gj.vWf = va->Wf, gj.vbf = va->bf;
    }
    gj.loss_n = wsf(ws, w.loss_n), gj.loss_out = loss_out;
    nred += (double)B * (ad.F + a->n_classes) + fc;
  }
  NF_RUN(st, sgd ? "wgrad_reduce_sgd" : "wgrad_reduce", 0.0, 4.0 * nred + nsgd, launch_wgrad_reduce_sgd(red, st));
  return NF_OK;
}

int32_t enqueue_sgd(const SgdTensors &t, hipStream_t st) {
  double n = 0;
  for (int i = 0; i < t.n; ++i) n += (double)t.numel[i];
  const bool mom = t.mu != 0.f && t.v[0] != nullptr;
  NF_RUN(st, "sgd", (mom ? 4.0 : 2.0) * n, (mom ? 20.0 : 12.0) * n, launch_sgd(t, st));
  return NF_OK;
}

int32_t enqueue_cache_copy(const char *name, const float *src, float *dst, const int32_t *sl, int32_t *dl,
                           long long se, long long sfirst, long long dfirst, const long long *idx, long long cap,
                           int B, hipStream_t st) {
  NF_RUN(st, name, 0.0, 8.0 * (double)se * B + (sl ? 8.0 * B : 0.0) + (idx ? 8.0 * B : 0.0),
         launch_cache_copy(src, dst, sl, dl, se, sfirst, dfirst, idx, cap, B, st));
  return NF_OK;
}

int32_t check_layer_ptrs(const nf_layer_desc *d, const float *x, const float *xs, const nf_layer_params *p) {
  if (!x || !p || !p->W || !p->b) return NF_ERR_NULL;
  if (d->skip_kind != 0 && !xs) return NF_ERR_NULL;
  if (d->skip_kind == 2 && !p->Wp) return NF_ERR_NULL;
  if (!aligned16(x) || !aligned16(xs) || !aligned16(p->W) || !aligned16(p->b) ||
      (d->skip_kind == 2 && !aligned16(p->Wp)))
    return NF_ERR_BAD_DESC;
  return NF_OK;
}

int32_t check_aux_ptrs(const nf_aux_params *ap) {
  if (!ap || !ap->Wa || !ap->ba || !ap->Wf || !ap->bf) return NF_ERR_NULL;
  if (!aligned16(ap->Wa) || !aligned16(ap->ba) || !aligned16(ap->Wf) || !aligned16(ap->bf)) return NF_ERR_BAD_DESC;
  return NF_OK;
}

int32_t check_pair(const nf_layer_desc *d, const LayerDims &ld, const nf_aux_desc *a) {
  if (a->C_in != d->C_out || a->H_in != ld.Hp || a->W_in != ld.Wp) return NF_ERR_BAD_DESC;
  return NF_OK;
}

// Device address of `scratch` on the current device: looked up once per device (each GPU holds
// its own copy at its own address) and kept.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];

int32_t static_scratch(void **out) {
  int dev = -1;
  NF_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return NF_ERR_DEVICE;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    NF_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return NF_ERR_DEVICE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return NF_OK;
}

// nf_local_step with the workspace given (ws != nullptr) or taken from the static array
int32_t local_step_impl(const nf_layer_desc *d, const nf_aux_desc *a, const nf_sgd_desc *s, int32_t B,
                        const float *x, const float *x_skip, const int32_t *labels, const nf_layer_params *p,
                        const nf_aux_params *ap, const nf_layer_params *gp, const nf_aux_params *ga,
                        const nf_layer_params *vp, const nf_aux_params *va, float *y_out, float *loss_out,
                        void *ws, size_t ws_bytes, bool use_static, void *stream) {
  LayerDims ld;
  AuxDims ad;
  int32_t rc = check_layer(d, &ld);
  if (rc) return rc;
  if ((rc = check_aux(a, &ad))) return rc;
  if ((rc = check_pair(d, ld, a))) return rc;
  if ((rc = check_sizes(d, ld, B))) return rc;
  if (!s || !labels || !y_out || !loss_out) return NF_ERR_NULL;
  if ((rc = check_layer_ptrs(d, x, x_skip, p))) return rc;
  if ((rc = check_aux_ptrs(ap))) return rc;
  if ((rc = check_layer_ptrs(d, x, x_skip, gp))) return rc;
  if ((rc = check_aux_ptrs(ga))) return rc;
  if (s->momentum != 0.f) {
    if (!vp || !va) return NF_ERR_NULL;
    if ((rc = check_layer_ptrs(d, x, x_skip, vp))) return rc;
    if ((rc = check_aux_ptrs(va))) return rc;
  }
  if (!aligned16(y_out)) return NF_ERR_BAD_DESC;
  const WsLayout w = ws_layout(d, ld, a, ad, B);
  if (use_static) {
    if (w.total > (size_t)NF_STATIC_SCRATCH_BYTES) return NF_ERR_SCRATCH_LIMIT;
    if ((rc = static_scratch(&ws))) return rc;
  } else if ((rc = check_ws(ws, ws_bytes, w.total))) {
    return rc;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  // Algorithm 2: forward with the current weights (this y_out is what the next layer reads),
  // head + loss, local gradients, update.
  if ((rc = run_layer_fwd(d, ld, B, x, x_skip, p, y_out, ws, w, st))) return rc;
  // the batch-mean loss rides on the head's backward launch
  if ((rc = run_aux_fwd(a, ad, B, y_out, labels, ap, nullptr, ws, w, st))) return rc;
  // ... and the update on the launch that finishes the weight gradients
  return run_bwd(d, ld, a, ad, B, x, x_skip, y_out, p, ap, gp, ga, loss_out, s, vp, va, ws, w, st);
}

}  // namespace

bool prof_active() { return g_prof.on; }
}  // namespace nf

using namespace nf;

extern "C" {

int32_t nf_contraction(int32_t mode) {
  if (mode == -1) return nf::g_contraction.load();
  if (mode != NF_CONTRACT_F32 && mode != NF_CONTRACT_BF16X6 && mode != NF_CONTRACT_BF16X9) return NF_ERR_BAD_DESC;
  return nf::g_contraction.exchange(mode);
}

const char *nf_strerror(int32_t s) {
  switch (s) {
    case NF_OK: return "ok";
    case NF_ERR_NULL: return "a required pointer is NULL";
    case NF_ERR_BAD_DESC: return "bad descriptor (non-positive or inconsistent sizes, or misaligned pointer)";
    case NF_ERR_UNSUPPORTED: return "configuration outside what the kernels implement";
    case NF_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case NF_ERR_CACHE_RANGE: return "cache range exceeds capacity";
    case NF_ERR_DEVICE: return "HIP error while enqueueing";
    case NF_ERR_SCRATCH_LIMIT: return "the step needs more scratch than the static buffer of nf_local_step_static holds";
    default: return "unknown status";
  }
}

int32_t nf_layer_out_dims(const nf_layer_desc *d, int32_t *Ho, int32_t *Wo, int32_t *Hp, int32_t *Wp) {
  LayerDims ld;
  const int32_t rc = check_layer(d, &ld);
  if (rc) return rc;
  if (Ho) *Ho = ld.Ho;
  if (Wo) *Wo = ld.Wo;
  if (Hp) *Hp = ld.Hp;
  if (Wp) *Wp = ld.Wp;
  return NF_OK;
}

int32_t nf_workspace_bytes(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B, size_t *out) {
  if (!out) return NF_ERR_NULL;
  LayerDims ld;
  AuxDims ad = {0, 0, 0};
  int32_t rc = check_layer(d, &ld);
  if (rc) return rc;
  if ((rc = check_sizes(d, ld, B))) return rc;
  if (a) {
    if ((rc = check_aux(a, &ad))) return rc;
    if ((rc = check_pair(d, ld, a))) return rc;
  }
  *out = ws_layout(d, ld, a, ad, B).total;
  return NF_OK;
}

int32_t nf_workspace_region(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B, int32_t which,
                            size_t *offset, size_t *bytes) {
  if (!offset || !bytes) return NF_ERR_NULL;
  LayerDims ld;
  AuxDims ad = {0, 0, 0};
  int32_t rc = check_layer(d, &ld);
  if (rc) return rc;
  if ((rc = check_sizes(d, ld, B))) return rc;
  if (a) {
    if ((rc = check_aux(a, &ad))) return rc;
    if ((rc = check_pair(d, ld, a))) return rc;
  }
  const WsLayout w = ws_layout(d, ld, a, ad, B);
  if (which == NF_WS_AUX_ACT) {
    if (!a) return NF_ERR_NULL;
    *offset = w.U;
    *bytes = (size_t)B * ad.Hu * ad.Wu * a->A * sizeof(float);
  } else if (which == NF_WS_POOL_ARG) {
    *offset = w.arg;
    *bytes = d->pool_kind ? (size_t)B * ld.Hp * ld.Wp * d->C_out : 0;
  } else if (which == NF_WS_HEAD_ARG) {
    if (!a) return NF_ERR_NULL;
    *offset = w.parg;
    *bytes = a->head_pool == 1 ? (size_t)B * ad.F * sizeof(int32_t) : 0;
  } else {
    return NF_ERR_BAD_DESC;
  }
  return NF_OK;
}

int32_t nf_layer_fwd(const nf_layer_desc *d, int32_t B, const float *x, const float *x_skip,
                     const nf_layer_params *p, float *y, void *ws, size_t ws_bytes, void *stream) {
  LayerDims ld;
  AuxDims ad = {0, 0, 0};
  int32_t rc = check_layer(d, &ld);
  if (rc) return rc;
  if ((rc = check_sizes(d, ld, B))) return rc;
  if ((rc = check_layer_ptrs(d, x, x_skip, p))) return rc;
  if (!y) return NF_ERR_NULL;
  if (!aligned16(y)) return NF_ERR_BAD_DESC;
  // the layout with a head is a superset that starts with the same regions, so a workspace
  // sized for the full step is accepted as well
  const WsLayout w = ws_layout(d, ld, nullptr, ad, B);
  if ((rc = check_ws(ws, ws_bytes, w.total))) return rc;
  return run_layer_fwd(d, ld, B, x, x_skip, p, y, ws, w, static_cast<hipStream_t>(stream));
}

int32_t nf_aux_fwd_loss(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B, const float *y,
                        const int32_t *labels, const nf_aux_params *ap, float *loss_out, void *ws,
                        size_t ws_bytes, void *stream) {
  LayerDims ld;
  AuxDims ad;
  int32_t rc = check_layer(d, &ld);
  if (rc) return rc;
  if ((rc = check_aux(a, &ad))) return rc;
  if ((rc = check_pair(d, ld, a))) return rc;
  if ((rc = check_sizes(d, ld, B))) return rc;
  if (!y || !labels || !loss_out) return NF_ERR_NULL;
  if ((rc = check_aux_ptrs(ap))) return rc;
  if (!aligned16(y)) return NF_ERR_BAD_DESC;
  const WsLayout w = ws_layout(d, ld, a, ad, B);
  if ((rc = check_ws(ws, ws_bytes, w.total))) return rc;
  return run_aux_fwd(a, ad, B, y, labels, ap, loss_out, ws, w, static_cast<hipStream_t>(stream));
}

int32_t nf_aux_predict(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B, const float *y,
                       const int32_t *labels, const nf_aux_params *ap, int32_t *pred_out, int32_t *n_correct,
                       int32_t accumulate, float *logits_out, void *ws, size_t ws_bytes, void *stream) {
  LayerDims ld;
  AuxDims ad;
  int32_t rc = check_layer(d, &ld);
  if (rc) return rc;
  if ((rc = check_aux(a, &ad))) return rc;
  if ((rc = check_pair(d, ld, a))) return rc;
  if ((rc = check_sizes(d, ld, B))) return rc;
  if (!y || !pred_out) return NF_ERR_NULL;
  if ((labels == nullptr) != (n_correct == nullptr)) return NF_ERR_NULL;
  if ((rc = check_aux_ptrs(ap))) return rc;
  if (!aligned16(y)) return NF_ERR_BAD_DESC;
  const WsLayout w = ws_layout(d, ld, a, ad, B);
  if ((rc = check_ws(ws, ws_bytes, w.total))) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if ((rc = run_aux_features(a, ad, B, y, ap, ws, w, st))) return rc;
  const HeadShape hs = head_shape(a, ad, B);
  const double fc = (double)a->n_classes * ad.F;
  int32_t *hit = reinterpret_cast<int32_t *>(wsf(ws, w.loss_n));  // one flag per sample
  NF_RUN(st, "head_predict", 2.0 * B * fc, 4.0 * (B * fc + (double)B * (ad.F + 2.0)),
         launch_head_predict(hs, wsf(ws, w.Pq), labels, ap->Wf, ap->bf, logits_out, pred_out, hit, st));
  if (labels) NF_RUN(st, "count_hits", 0.0, 4.0 * B, launch_count_hits(hit, B, n_correct, accumulate != 0, st));
  return NF_OK;
}

int32_t nf_local_bwd_wgrad(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B, const float *x,
                           const float *x_skip, const float *y, const nf_layer_params *p,
                           const nf_aux_params *ap, const nf_layer_params *gp, const nf_aux_params *ga,
                           void *ws, size_t ws_bytes, void *stream) {
  LayerDims ld;
  AuxDims ad;
  int32_t rc = check_layer(d, &ld);
  if (rc) return rc;
  if ((rc = check_aux(a, &ad))) return rc;
  if ((rc = check_pair(d, ld, a))) return rc;
  if ((rc = check_sizes(d, ld, B))) return rc;
  if ((rc = check_layer_ptrs(d, x, x_skip, p))) return rc;
  if ((rc = check_aux_ptrs(ap))) return rc;
  if ((rc = check_layer_ptrs(d, x, x_skip, gp))) return rc;
  if ((rc = check_aux_ptrs(ga))) return rc;
  if (!y) return NF_ERR_NULL;
  if (!aligned16(y)) return NF_ERR_BAD_DESC;
  const WsLayout w = ws_layout(d, ld, a, ad, B);
  if ((rc = check_ws(ws, ws_bytes, w.total))) return rc;
  return run_bwd(d, ld, a, ad, B, x, x_skip, y, p, ap, gp, ga, nullptr, nullptr, nullptr, nullptr, ws, w,
                 static_cast<hipStream_t>(stream));
}

int32_t nf_sgd_update(const nf_sgd_desc *s, int32_t n_tensors, float *const *w, const float *const *g,
                      float *const *v, const int64_t *numel, void *stream) {
  if (!s || !w || !g || !numel) return NF_ERR_NULL;
  if (n_tensors <= 0 || n_tensors > 16) return NF_ERR_BAD_DESC;
  const bool use_v = s->momentum != 0.f;
  if (use_v && !v) return NF_ERR_NULL;
  SgdTensors t;
  std::memset(&t, 0, sizeof(t));
  for (int i = 0; i < n_tensors; ++i) {
    if (!w[i] || !g[i] || (use_v && !v[i])) return NF_ERR_NULL;
    if (numel[i] <= 0) return NF_ERR_BAD_DESC;
    if (!aligned16(w[i]) || !aligned16(g[i]) || (use_v && !aligned16(v[i]))) return NF_ERR_BAD_DESC;
    t.w[i] = w[i], t.g[i] = g[i], t.v[i] = use_v ? v[i] : nullptr, t.numel[i] = numel[i];
  }
  t.n = n_tensors, t.lr = s->lr, t.mu = s->momentum;
  return enqueue_sgd(t, static_cast<hipStream_t>(stream));
}

static int32_t check_cache(const void *cache, const void *clab, int64_t capacity, int64_t se, int64_t first,
                           int32_t B, const void *buf, const void *lab) {
  if (!cache || !buf) return NF_ERR_NULL;
  if ((clab == nullptr) != (lab == nullptr)) return NF_ERR_NULL;
  if (capacity <= 0 || se <= 0 || B <= 0 || B > 65535) return NF_ERR_BAD_DESC;
  if (!aligned16(cache) || !aligned16(buf)) return NF_ERR_BAD_DESC;
  if (first < 0 || first + B > capacity) return NF_ERR_CACHE_RANGE;
  return NF_OK;
}

int32_t nf_cache_write(float *cache, int32_t *cache_labels, int64_t capacity, int64_t sample_elems,
                       int64_t first, int32_t B, const float *y, const int32_t *labels, void *stream) {
  const int32_t rc = check_cache(cache, cache_labels, capacity, sample_elems, first, B, y, labels);
  if (rc) return rc;
  return enqueue_cache_copy("cache_write", y, cache, labels, cache_labels, sample_elems, 0, first, nullptr, capacity, B,
                            static_cast<hipStream_t>(stream));
}

int32_t nf_cache_read(const float *cache, const int32_t *cache_labels, int64_t capacity, int64_t sample_elems,
                      int64_t first, const int64_t *idx, int32_t B, float *x_out, int32_t *labels_out,
                      void *stream) {
  const int32_t rc = check_cache(cache, cache_labels, capacity, sample_elems, idx ? 0 : first, idx ? 1 : B, x_out,
                                 labels_out);
  if (rc) return rc;
  if (B <= 0 || B > 65535) return NF_ERR_BAD_DESC;
  return enqueue_cache_copy("cache_read", cache, x_out, cache_labels, labels_out, sample_elems, first, 0,
                            reinterpret_cast<const long long *>(idx), capacity, B, static_cast<hipStream_t>(stream));
}

int32_t nf_local_step(const nf_layer_desc *d, const nf_aux_desc *a, const nf_sgd_desc *s, int32_t B,
                      const float *x, const float *x_skip, const int32_t *labels, const nf_layer_params *p,
                      const nf_aux_params *ap, const nf_layer_params *gp, const nf_aux_params *ga,
                      const nf_layer_params *vp, const nf_aux_params *va, float *y_out, float *loss_out,
                      void *ws, size_t ws_bytes, void *stream) {
  return local_step_impl(d, a, s, B, x, x_skip, labels, p, ap, gp, ga, vp, va, y_out, loss_out, ws, ws_bytes, false,
                         stream);
}

int32_t nf_local_step_static(const nf_layer_desc *d, const nf_aux_desc *a, const nf_sgd_desc *s, int32_t B,
                             const float *x, const float *x_skip, const int32_t *labels,
                             const nf_layer_params *p, const nf_aux_params *ap, const nf_layer_params *gp,
                             const nf_aux_params *ga, const nf_layer_params *vp, const nf_aux_params *va,
                             float *y_out, float *loss_out, void *stream) {
  return local_step_impl(d, a, s, B, x, x_skip, labels, p, ap, gp, ga, vp, va, y_out, loss_out, nullptr, 0, true,
                         stream);
}

int32_t nf_device_info(int32_t *compute_units, int32_t *clock_khz) {
  if (!compute_units || !clock_khz) return NF_ERR_NULL;
  int dev = 0, cu = 0, khz = 0;
  NF_HIP(hipGetDevice(&dev));
  NF_HIP(hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev));
  NF_HIP(hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev));
  *compute_units = cu, *clock_khz = khz;
  return NF_OK;
}

int32_t nf_prof_begin(void) {
  std::lock_guard<std::mutex> lk(g_prof.mu);
  for (auto &e : g_prof.ev) {
    (void)hipEventDestroy(e.a);
    (void)hipEventDestroy(e.b);
  }
  g_prof.ev.clear();
  g_prof.on = true;
  return NF_OK;
}

int32_t nf_prof_end(nf_prof_record *out, int32_t cap, int32_t *n) {
  g_prof.on = false;
  if (!n || (cap > 0 && !out)) return NF_ERR_NULL;
  std::lock_guard<std::mutex> lk(g_prof.mu);
  std::vector<nf_prof_record> agg;
  int32_t rc = NF_OK;
  for (auto &e : g_prof.ev) {
    float ms = 0.f;
    if (hipEventSynchronize(e.b) != hipSuccess || hipEventElapsedTime(&ms, e.a, e.b) != hipSuccess) rc = NF_ERR_DEVICE;
    (void)hipEventDestroy(e.a);
    (void)hipEventDestroy(e.b);
    auto it = std::find_if(agg.begin(), agg.end(), [&](const nf_prof_record &r) { return !std::strcmp(r.kernel, e.name); });
    if (it == agg.end()) {
      nf_prof_record r;
      std::memset(&r, 0, sizeof(r));
      std::strncpy(r.kernel, e.name, sizeof(r.kernel) - 1);
      agg.push_back(r);
      it = agg.end() - 1;
    }
    it->launches += 1, it->ms += ms, it->flops += e.flops, it->bytes += e.bytes;
  }
  g_prof.ev.clear();
  std::sort(agg.begin(), agg.end(), [](const nf_prof_record &a, const nf_prof_record &b) { return a.ms > b.ms; });
  *n = (int32_t)agg.size();
  for (int32_t i = 0; i < *n && i < cap; ++i) out[i] = agg[i];
  return rc;
}

}  // extern "C"
