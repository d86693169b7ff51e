// nfo — CPU oracle for the local training step (see nfo.h).  TEST INFRASTRUCTURE ONLY.
//
// Every function is the written-out definition: direct loops, double accumulation,
// one rounding to the storage type per stored element.  OpenMP is applied only to loops
// over *output* elements, so no element's summation order depends on the thread count.
#include "nfo.h"

#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

struct Dims {
  int Ho, Wo, Hp, Wp;
};

bool layer_dims(const nfo_layer_desc &d, Dims &o) {
  if (d.C_in <= 0 || d.H_in <= 0 || d.W_in <= 0 || d.C_out <= 0 || d.R <= 0 || d.S <= 0 ||
      d.stride <= 0 || d.pad < 0)
    return false;
  const int hn = d.H_in + 2 * d.pad - d.R, wn = d.W_in + 2 * d.pad - d.S;
  if (hn < 0 || wn < 0) return false;
  o.Ho = hn / d.stride + 1;
  o.Wo = wn / d.stride + 1;
  if (d.pool_kind == 0) {
    o.Hp = o.Ho;
    o.Wp = o.Wo;
  } else {
    if (d.pool_k <= 0 || d.pool_stride <= 0 || d.pool_pad < 0 || 2 * d.pool_pad > d.pool_k)
      return false;
    const int ph = o.Ho + 2 * d.pool_pad - d.pool_k, pw = o.Wo + 2 * d.pool_pad - d.pool_k;
    if (ph < 0 || pw < 0) return false;
    o.Hp = ph / d.pool_stride + 1;
    o.Wp = pw / d.pool_stride + 1;
  }
  return true;
}

// ---------------------------------------------------------------------------------------
// Eq. 1: x_{n+1} = alpha P_n theta_n x_n   (conv + bias [+ skip], ReLU, max-pool).
// ReLU is applied before the max-pool; the two commute (both are monotone), see tests.
// ---------------------------------------------------------------------------------------
template <typename T>
void layer_fwd(const nfo_layer_desc &d, int B, const T *x, const T *xs, const T *W, const T *b,
               const T *Wp, T *Z, T *Y, int32_t *arg) {
  Dims o;
  if (!layer_dims(d, o)) return;
  const int C = d.C_in, H = d.H_in, Wd = d.W_in, K = d.C_out, R = d.R, S = d.S;
  const int st = d.stride, p = d.pad, Ho = o.Ho, Wo = o.Wo;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int k = 0; k < K; ++k)
      for (int i = 0; i < Ho; ++i)
        for (int j = 0; j < Wo; ++j) {
          double acc = b ? (double)b[k] : 0.0;
          for (int c = 0; c < C; ++c)
            for (int r = 0; r < R; ++r)
              for (int s = 0; s < S; ++s) {
                const int h = i * st + r - p, w = j * st + s - p;
                if (h < 0 || h >= H || w < 0 || w >= Wd) continue;  // zero padding
                acc += (double)W[((int64_t)(k * C + c) * R + r) * S + s] *
                       (double)x[((int64_t)(n * C + c) * H + h) * Wd + w];
              }
          if (d.skip_kind == 1) {  // identity shortcut: same shape as Z
            acc += (double)xs[((int64_t)(n * K + k) * Ho + i) * Wo + j];
          } else if (d.skip_kind == 2) {  // 1x1 strided projection of the shortcut, no bias
            const int ss = d.skip_stride;
            for (int c = 0; c < d.skip_C; ++c)
              acc += (double)Wp[(int64_t)k * d.skip_C + c] *
                     (double)xs[((int64_t)(n * d.skip_C + c) * d.skip_H + i * ss) * d.skip_W + j * ss];
          }
          Z[((int64_t)(n * K + k) * Ho + i) * Wo + j] = (T)acc;
        }
  if (d.pool_kind == 0) {
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < (int64_t)B * K * Ho * Wo; ++e) Y[e] = Z[e] > (T)0 ? Z[e] : (T)0;
    return;
  }
  const int pk = d.pool_k, ps = d.pool_stride, pp = d.pool_pad, Hp = o.Hp, Wp_ = o.Wp;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int k = 0; k < K; ++k) {
      const T *zp = Z + (int64_t)(n * K + k) * Ho * Wo;
      for (int i = 0; i < Hp; ++i)
        for (int j = 0; j < Wp_; ++j) {
          T best = -std::numeric_limits<T>::infinity();
          int32_t bi = -1;
          for (int u = 0; u < pk; ++u)
            for (int v = 0; v < pk; ++v) {
              const int h = i * ps + u - pp, w = j * ps + v - pp;
              if (h < 0 || h >= Ho || w < 0 || w >= Wo) continue;  // padding cells ignored
              const T t = zp[h * Wo + w] > (T)0 ? zp[h * Wo + w] : (T)0;  // ReLU
              if (t > best) {  // strict: first maximal element in row-major window order
                best = t;
                bi = h * Wo + w;
              }
            }
          const int64_t q = ((int64_t)(n * K + k) * Hp + i) * Wp_ + j;
          Y[q] = best;
          if (arg) arg[q] = bi;
        }
    }
}

// adaptive average-pool window [lo,hi) of output cell i for an input of length L
inline void adaptive_window(int i, int L, int O, int &lo, int &hi) {
  lo = (int)((int64_t)i * L / O);
  hi = (int)ceil_div((int64_t)(i + 1) * L, O);
}

// ---------------------------------------------------------------------------------------
// Eq. 2: z = gamma_n F_n beta_n x_{n+1};  Eq. 3 with cross-entropy (or mean squared error
// against the one-hot label), mean over the batch.  F_n is adaptive average or max pooling.
// ---------------------------------------------------------------------------------------
template <typename T>
void aux_fwd_loss(const nfo_aux_desc &a, int B, const T *y, const int32_t *labels, const T *Wa,
                  const T *ba, const T *Wf, const T *bf, T *U, T *Pq, T *z, double *loss, T *dz, T *Upre,
                  int32_t *parg) {
  const int K = a.C_in, H = a.H_in, Wd = a.W_in, A = a.A, R = a.R, S = a.S, p = a.pad;
  const int oh = a.pool_oh, ow = a.pool_ow, Cls = a.n_classes, F = A * oh * ow;
  // beta_n: stride-1 convolution, output has the input's spatial size when 2*pad = R-1
  const int Hu = H + 2 * p - R + 1, Wu = Wd + 2 * p - S + 1;
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int q = 0; q < A; ++q)
      for (int i = 0; i < Hu; ++i)
        for (int j = 0; j < Wu; ++j) {
          double acc = ba ? (double)ba[q] : 0.0;
          for (int k = 0; k < K; ++k)
            for (int r = 0; r < R; ++r)
              for (int s = 0; s < S; ++s) {
                const int h = i + r - p, w = j + s - p;
                if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                acc += (double)Wa[((int64_t)(q * K + k) * R + r) * S + s] *
                       (double)y[((int64_t)(n * K + k) * H + h) * Wd + w];
              }
          if (Upre) Upre[((int64_t)(n * A + q) * Hu + i) * Wu + j] = (T)acc;  // before the ReLU
          if (a.relu && acc < 0.0) acc = 0.0;
          U[((int64_t)(n * A + q) * Hu + i) * Wu + j] = (T)acc;
        }
  // F_n: adaptive pooling to oh x ow -- the mean of each window, or its maximum (then parg
  // records the flat position h*Wu+w of the first maximal element in row-major window order)
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int q = 0; q < A; ++q)
      for (int i = 0; i < oh; ++i)
        for (int j = 0; j < ow; ++j) {
          int h0, h1, w0, w1;
          adaptive_window(i, Hu, oh, h0, h1);
          adaptive_window(j, Wu, ow, w0, w1);
          const int64_t f = (int64_t)n * F + (q * oh + i) * ow + j;
          if (a.head_pool == 1) {
            T best = U[((int64_t)(n * A + q) * Hu + h0) * Wu + w0];
            int bi = h0 * Wu + w0;
            for (int h = h0; h < h1; ++h)
              for (int w = w0; w < w1; ++w) {
                const T u = U[((int64_t)(n * A + q) * Hu + h) * Wu + w];
                if (u > best) best = u, bi = h * Wu + w;
              }
            Pq[f] = best;
            if (parg) parg[f] = bi;
            continue;
          }
          double acc = 0.0;
          for (int h = h0; h < h1; ++h)
            for (int w = w0; w < w1; ++w) acc += (double)U[((int64_t)(n * A + q) * Hu + h) * Wu + w];
          Pq[f] = (T)(acc / (double)((h1 - h0) * (w1 - w0)));
        }
  // gamma_n: linear layer
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int c = 0; c < Cls; ++c) {
      double acc = bf ? (double)bf[c] : 0.0;
      for (int f = 0; f < F; ++f) acc += (double)Wf[(int64_t)c * F + f] * (double)Pq[(int64_t)n * F + f];
      z[(int64_t)n * Cls + c] = (T)acc;
    }
  double total = 0.0;
  if (a.loss_kind == 1) {
    // mean squared error against the one-hot label: mean over the classes, then over the batch
    for (int n = 0; n < B; ++n)
      for (int c = 0; c < Cls; ++c) {
        const double e = (double)z[(int64_t)n * Cls + c] - (c == labels[n] ? 1.0 : 0.0);
        total += e * e;
        dz[(int64_t)n * Cls + c] = (T)(2.0 * e / ((double)B * (double)Cls));
      }
    *loss = total / ((double)B * (double)Cls);
    return;
  }
  // softmax cross-entropy, mean over the batch, and its derivative w.r.t. the logits
  for (int n = 0; n < B; ++n) {
    const T *zn = z + (int64_t)n * Cls;
    double m = (double)zn[0];
    for (int c = 1; c < Cls; ++c) m = std::fmax(m, (double)zn[c]);
    double se = 0.0;
    for (int c = 0; c < Cls; ++c) se += std::exp((double)zn[c] - m);
    const double lse = m + std::log(se);
    total += lse - (double)zn[labels[n]];
    for (int c = 0; c < Cls; ++c) {
      const double sm = std::exp((double)zn[c] - lse);
      dz[(int64_t)n * Cls + c] = (T)((sm - (c == labels[n] ? 1.0 : 0.0)) / (double)B);
    }
  }
  *loss = total / (double)B;
}

// ---------------------------------------------------------------------------------------
// Gradients of the local loss w.r.t. (theta_n, beta_n, gamma_n) only.
// ---------------------------------------------------------------------------------------
template <typename T>
void local_bwd(const nfo_layer_desc &d, const nfo_aux_desc &a, int B, const T *x, const T *xs,
               const T *Z, const T *Y, const int32_t *arg, const T *U, const T *Pq, const T *dz,
               const T *Wa, const T *Wf, T *dW, T *db, T *dWp, T *dWa, T *dba, T *dWf, T *dbf,
               T *dY_out, T *dZ_out, const uint8_t *mask_u, const uint8_t *mask_z, const int32_t *parg) {
  // mask_u / mask_z (optional): the two ReLU decisions "U > 0" and "Z > 0" handed in by the
  // caller instead of being taken here.  They exist for comparisons against an implementation
  // that accumulates in another precision: where a pre-activation is zero to within rounding,
  // both sides must differentiate the same branch of the ReLU.
  Dims o;
  if (!layer_dims(d, o)) return;
  const int C = d.C_in, H = d.H_in, Wd = d.W_in, K = d.C_out, R = d.R, S = d.S, st = d.stride,
            p = d.pad, Ho = o.Ho, Wo = o.Wo, Hp = o.Hp, Wp_ = o.Wp;
  const int A = a.A, Ra = a.R, Sa = a.S, pa = a.pad, oh = a.pool_oh, ow = a.pool_ow,
            Cls = a.n_classes, F = A * oh * ow;
  const int Hu = Hp + 2 * pa - Ra + 1, Wu = Wp_ + 2 * pa - Sa + 1;

  // gamma_n
#pragma omp parallel for schedule(static)
  for (int c = 0; c < Cls; ++c) {
    double sb = 0.0;
    for (int n = 0; n < B; ++n) sb += (double)dz[(int64_t)n * Cls + c];
    dbf[c] = (T)sb;
    for (int f = 0; f < F; ++f) {
      double acc = 0.0;
      for (int n = 0; n < B; ++n) acc += (double)dz[(int64_t)n * Cls + c] * (double)Pq[(int64_t)n * F + f];
      dWf[(int64_t)c * F + f] = (T)acc;
    }
  }
  std::vector<T> dPq((size_t)B * F);
#pragma omp parallel for schedule(static)
  for (int n = 0; n < B; ++n)
    for (int f = 0; f < F; ++f) {
      double acc = 0.0;
      for (int c = 0; c < Cls; ++c) acc += (double)dz[(int64_t)n * Cls + c] * (double)Wf[(int64_t)c * F + f];
      dPq[(size_t)n * F + f] = (T)acc;
    }
  // F_n backward (each input cell collects from every window that contains it) and the
  // aux ReLU mask
  std::vector<T> dU((size_t)B * A * Hu * Wu);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int q = 0; q < A; ++q)
      for (int h = 0; h < Hu; ++h)
        for (int w = 0; w < Wu; ++w) {
          double acc = 0.0;
          for (int i = 0; i < oh; ++i)
            for (int j = 0; j < ow; ++j) {
              int h0, h1, w0, w1;
              adaptive_window(i, Hu, oh, h0, h1);
              adaptive_window(j, Wu, ow, w0, w1);
              if (h < h0 || h >= h1 || w < w0 || w >= w1) continue;
              const size_t f = (size_t)n * F + (q * oh + i) * ow + j;
              if (a.head_pool == 1) {  // max pooling hands the gradient to the selected element
                if (parg[f] == h * Wu + w) acc += (double)dPq[f];
                continue;
              }
              acc += (double)dPq[f] / (double)((h1 - h0) * (w1 - w0));
            }
          const int64_t e = ((int64_t)(n * A + q) * Hu + h) * Wu + w;
          const bool on = mask_u ? mask_u[e] != 0 : U[e] > (T)0;
          if (a.relu && !on) acc = 0.0;
          dU[(size_t)e] = (T)acc;
        }
  // beta_n: weight and bias gradient
#pragma omp parallel for collapse(2) schedule(static)
  for (int q = 0; q < A; ++q)
    for (int k = 0; k < K; ++k)
      for (int r = 0; r < Ra; ++r)
        for (int s = 0; s < Sa; ++s) {
          double acc = 0.0;
          for (int n = 0; n < B; ++n)
            for (int i = 0; i < Hu; ++i)
              for (int j = 0; j < Wu; ++j) {
                const int h = i + r - pa, w = j + s - pa;
                if (h < 0 || h >= Hp || w < 0 || w >= Wp_) continue;
                acc += (double)dU[((size_t)(n * A + q) * Hu + i) * Wu + j] *
                       (double)Y[((int64_t)(n * K + k) * Hp + h) * Wp_ + w];
              }
          dWa[((int64_t)(q * K + k) * Ra + r) * Sa + s] = (T)acc;
        }
#pragma omp parallel for schedule(static)
  for (int q = 0; q < A; ++q) {
    double acc = 0.0;
    for (int n = 0; n < B; ++n)
      for (int e = 0; e < Hu * Wu; ++e) acc += (double)dU[(size_t)(n * A + q) * Hu * Wu + e];
    dba[q] = (T)acc;
  }
  // data gradient of the aux conv w.r.t. the emitted activation Y (the only data gradient
  // the method needs: it links theta_n to the head's loss)
  std::vector<T> dY((size_t)B * K * Hp * Wp_);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int k = 0; k < K; ++k)
      for (int h = 0; h < Hp; ++h)
        for (int w = 0; w < Wp_; ++w) {
          double acc = 0.0;
          for (int q = 0; q < A; ++q)
            for (int r = 0; r < Ra; ++r)
              for (int s = 0; s < Sa; ++s) {
                const int i = h - r + pa, j = w - s + pa;  // output cell that read (h,w) via tap (r,s)
                if (i < 0 || i >= Hu || j < 0 || j >= Wu) continue;
                acc += (double)dU[((size_t)(n * A + q) * Hu + i) * Wu + j] *
                       (double)Wa[((int64_t)(q * K + k) * Ra + r) * Sa + s];
              }
          dY[((size_t)(n * K + k) * Hp + h) * Wp_ + w] = (T)acc;
        }
  // P_n backward (route to the recorded arg-max) and the layer's ReLU mask
  std::vector<T> dZ((size_t)B * K * Ho * Wo, (T)0);
#pragma omp parallel for collapse(2) schedule(static)
  for (int n = 0; n < B; ++n)
    for (int k = 0; k < K; ++k) {
      const int64_t zb = (int64_t)(n * K + k) * Ho * Wo, yb = (int64_t)(n * K + k) * Hp * Wp_;
      if (d.pool_kind == 0) {
        for (int e = 0; e < Ho * Wo; ++e) {
          const bool on = mask_z ? mask_z[zb + e] != 0 : Z[zb + e] > (T)0;
          dZ[(size_t)(zb + e)] = on ? dY[(size_t)(yb + e)] : (T)0;
        }
      } else {
        // overlapping windows may elect the same cell more than once: sum in double
        std::vector<double> plane((size_t)Ho * Wo, 0.0);
        for (int e = 0; e < Hp * Wp_; ++e) {
          const int32_t t = arg[yb + e];
          if (t < 0) continue;
          const bool on = mask_z ? mask_z[zb + t] != 0 : Z[zb + t] > (T)0;
          if (on) plane[(size_t)t] += (double)dY[(size_t)(yb + e)];
        }
        for (int e = 0; e < Ho * Wo; ++e) dZ[(size_t)(zb + e)] = (T)plane[(size_t)e];
      }
    }
  // theta_n: weight, bias and projection gradients.  Nothing for x or x_skip.
#pragma omp parallel for collapse(2) schedule(static)
  for (int k = 0; k < K; ++k)
    for (int c = 0; c < C; ++c)
      for (int r = 0; r < R; ++r)
        for (int s = 0; s < S; ++s) {
          double acc = 0.0;
          for (int n = 0; n < B; ++n)
            for (int i = 0; i < Ho; ++i)
              for (int j = 0; j < Wo; ++j) {
                const int h = i * st + r - p, w = j * st + s - p;
                if (h < 0 || h >= H || w < 0 || w >= Wd) continue;
                acc += (double)dZ[((size_t)(n * K + k) * Ho + i) * Wo + j] *
                       (double)x[((int64_t)(n * C + c) * H + h) * Wd + w];
              }
          dW[((int64_t)(k * C + c) * R + r) * S + s] = (T)acc;
        }
#pragma omp parallel for schedule(static)
  for (int k = 0; k < K; ++k) {
    double acc = 0.0;
    for (int n = 0; n < B; ++n)
      for (int e = 0; e < Ho * Wo; ++e) acc += (double)dZ[(size_t)(n * K + k) * Ho * Wo + e];
    db[k] = (T)acc;
  }
  if (d.skip_kind == 2 && dWp) {
    const int ss = d.skip_stride;
#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < K; ++k)
      for (int c = 0; c < d.skip_C; ++c) {
        double acc = 0.0;
        for (int n = 0; n < B; ++n)
          for (int i = 0; i < Ho; ++i)
            for (int j = 0; j < Wo; ++j)
              acc += (double)dZ[((size_t)(n * K + k) * Ho + i) * Wo + j] *
                     (double)xs[((int64_t)(n * d.skip_C + c) * d.skip_H + i * ss) * d.skip_W + j * ss];
        dWp[(int64_t)k * d.skip_C + c] = (T)acc;
      }
  }
  if (dY_out) std::memcpy(dY_out, dY.data(), dY.size() * sizeof(T));
  if (dZ_out) std::memcpy(dZ_out, dZ.data(), dZ.size() * sizeof(T));
}

template <typename T>
void sgd_update(int64_t numel, T *w, const T *g, T *v, double lr, double mu) {
  for (int64_t e = 0; e < numel; ++e) {
    double step = (double)g[e];
    if (v && mu != 0.0) {
      step = mu * (double)v[e] + (double)g[e];
      v[e] = (T)step;
      step = (double)v[e];  // the stored (rounded) momentum is what moves the weight
    }
    w[e] = (T)((double)w[e] - lr * step);
  }
}

template <typename T>
void cache_write(T *cache, int32_t *cl, int64_t se, int64_t first, int B, const T *y, const int32_t *labels) {
  for (int n = 0; n < B; ++n) {
    for (int64_t e = 0; e < se; ++e) cache[(first + n) * se + e] = y[(int64_t)n * se + e];
    if (cl && labels) cl[first + n] = labels[n];
  }
}

template <typename T>
void cache_read(const T *cache, const int32_t *cl, int64_t se, int64_t first, const int64_t *idx, int B,
                T *xo, int32_t *lo) {
  for (int n = 0; n < B; ++n) {
    const int64_t row = idx ? idx[n] : first + n;
    for (int64_t e = 0; e < se; ++e) xo[(int64_t)n * se + e] = cache[row * se + e];
    if (cl && lo) lo[n] = cl[row];
  }
}

template <typename T>
void local_step(const nfo_layer_desc &d, const nfo_aux_desc &a, int B, const T *x, const T *xs,
                const int32_t *labels, T *W, T *b, T *Wp, T *Wa, T *ba, T *Wf, T *bf, T *gW, T *gb,
                T *gWp, T *gWa, T *gba, T *gWf, T *gbf, T *vW, T *vb, T *vWp, T *vWa, T *vba, T *vWf,
                T *vbf, double lr, double mu, T *Y, double *loss) {
  Dims o;
  if (!layer_dims(d, o)) return;
  const int K = d.C_out, A = a.A, F = A * a.pool_oh * a.pool_ow, Cls = a.n_classes;
  const int Hu = o.Hp + 2 * a.pad - a.R + 1, Wu = o.Wp + 2 * a.pad - a.S + 1;
  const int64_t nW = (int64_t)K * d.C_in * d.R * d.S, nWp = d.skip_kind == 2 ? (int64_t)K * d.skip_C : 0,
                nWa = (int64_t)A * K * a.R * a.S, nWf = (int64_t)Cls * F;
  std::vector<T> Z((size_t)B * K * o.Ho * o.Wo), U((size_t)B * A * Hu * Wu), Pq((size_t)B * F),
      z((size_t)B * Cls), dz((size_t)B * Cls);
  std::vector<int32_t> arg(d.pool_kind ? (size_t)B * K * o.Hp * o.Wp : 0), parg((size_t)B * F);
  std::vector<T> tW(nW), tb(K), tWp(nWp), tWa(nWa), tba(A), tWf(nWf), tbf(Cls);
  // lines 3-5 of Algorithm 2
  layer_fwd<T>(d, B, x, xs, W, b, Wp, Z.data(), Y, arg.empty() ? nullptr : arg.data());
  aux_fwd_loss<T>(a, B, Y, labels, Wa, ba, Wf, bf, U.data(), Pq.data(), z.data(), loss, dz.data(), nullptr,
                  parg.data());
  // line 6
  local_bwd<T>(d, a, B, x, xs, Z.data(), Y, arg.empty() ? nullptr : arg.data(), U.data(), Pq.data(),
               dz.data(), Wa, Wf, tW.data(), tb.data(), nWp ? tWp.data() : nullptr, tWa.data(), tba.data(),
               tWf.data(), tbf.data(), nullptr, nullptr, nullptr, nullptr, parg.data());
  // line 7
  sgd_update<T>(nW, W, tW.data(), vW, lr, mu);
  sgd_update<T>(K, b, tb.data(), vb, lr, mu);
  if (nWp) sgd_update<T>(nWp, Wp, tWp.data(), vWp, lr, mu);
  sgd_update<T>(nWa, Wa, tWa.data(), vWa, lr, mu);
  sgd_update<T>(A, ba, tba.data(), vba, lr, mu);
  sgd_update<T>(nWf, Wf, tWf.data(), vWf, lr, mu);
  sgd_update<T>(Cls, bf, tbf.data(), vbf, lr, mu);
  auto out = [](T *dst, const std::vector<T> &src) {
    if (dst && !src.empty()) std::memcpy(dst, src.data(), src.size() * sizeof(T));
  };
  out(gW, tW), out(gb, tb), out(gWp, tWp), out(gWa, tWa), out(gba, tba), out(gWf, tWf), out(gbf, tbf);
}

}  // namespace

extern "C" {

int32_t nfo_layer_dims(const nfo_layer_desc *d, int32_t *Ho, int32_t *Wo, int32_t *Hp, int32_t *Wp) {
  Dims o;
  if (!d || !layer_dims(*d, o)) return -1;
  if (Ho) *Ho = o.Ho;
  if (Wo) *Wo = o.Wo;
  if (Hp) *Hp = o.Hp;
  if (Wp) *Wp = o.Wp;
  return 0;
}

int32_t nfo_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void nfo_set_num_threads(int32_t n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

#define NFO_DEFINE(T, SUF)                                                                         \
  void nfo_layer_fwd_##SUF(const nfo_layer_desc *d, int32_t B, const T *x, const T *x_skip,        \
                           const T *W, const T *b, const T *Wp, T *Z, T *Y, int32_t *arg) {        \
    layer_fwd<T>(*d, B, x, x_skip, W, b, Wp, Z, Y, arg);                                           \
  }                                                                                                \
  void nfo_aux_fwd_loss_##SUF(const nfo_aux_desc *a, int32_t B, const T *y, const int32_t *labels, \
                              const T *Wa, const T *ba, const T *Wf, const T *bf, T *U, T *Pq,     \
                              T *z, double *loss, T *dz, T *Upre, int32_t *parg) {                 \
    aux_fwd_loss<T>(*a, B, y, labels, Wa, ba, Wf, bf, U, Pq, z, loss, dz, Upre, parg);             \
  }                                                                                                \
  void nfo_local_bwd_##SUF(const nfo_layer_desc *d, const nfo_aux_desc *a, int32_t B, const T *x,  \
                           const T *x_skip, const T *Z, const T *Y, const int32_t *arg,            \
                           const T *U, const T *Pq, const T *dz, const T *Wa, const T *Wf, T *dW,  \
                           T *db, T *dWp, T *dWa, T *dba, T *dWf, T *dbf, T *dY, T *dZ,            \
                           const uint8_t *mask_u, const uint8_t *mask_z, const int32_t *parg) {    \
    local_bwd<T>(*d, *a, B, x, x_skip, Z, Y, arg, U, Pq, dz, Wa, Wf, dW, db, dWp, dWa, dba, dWf,   \
                 dbf, dY, dZ, mask_u, mask_z, parg);                                               \
  }                                                                                                \
  void nfo_sgd_update_##SUF(int64_t numel, T *w, const T *g, T *v, double lr, double mu) {         \
    sgd_update<T>(numel, w, g, v, lr, mu);                                                         \
  }                                                                                                \
  void nfo_cache_write_##SUF(T *cache, int32_t *cl, int64_t se, int64_t first, int32_t B,          \
                             const T *y, const int32_t *labels) {                                  \
    cache_write<T>(cache, cl, se, first, B, y, labels);                                            \
  }                                                                                                \
  void nfo_cache_read_##SUF(const T *cache, const int32_t *cl, int64_t se, int64_t first,          \
                            const int64_t *idx, int32_t B, T *x_out, int32_t *labels_out) {        \
    cache_read<T>(cache, cl, se, first, idx, B, x_out, labels_out);                                \
  }                                                                                                \
  void nfo_local_step_##SUF(const nfo_layer_desc *d, const nfo_aux_desc *a, int32_t B, const T *x, \
                            const T *x_skip, const int32_t *labels, T *W, T *b, T *Wp, T *Wa,      \
                            T *ba, T *Wf, T *bf, T *gW, T *gb, T *gWp, T *gWa, T *gba, T *gWf,     \
                            T *gbf, T *vW, T *vb, T *vWp, T *vWa, T *vba, T *vWf, T *vbf,          \
                            double lr, double mu, T *Y, double *loss) {                            \
    local_step<T>(*d, *a, B, x, x_skip, labels, W, b, Wp, Wa, ba, Wf, bf, gW, gb, gWp, gWa, gba,   \
                  gWf, gbf, vW, vb, vWp, vWa, vba, vWf, vbf, lr, mu, Y, loss);                     \
  }

NFO_DEFINE(float, f32)
NFO_DEFINE(double, f64)

}  // extern "C"
