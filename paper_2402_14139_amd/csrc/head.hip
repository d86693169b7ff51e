// The auxiliary head after its convolution (NeuroFlux, arXiv 2402.14139, Eq. 2 and Eq. 3):
// adaptive average pooling F_n, the linear layer gamma_n, softmax cross-entropy with the
// batch mean, and the backward of those three (gradient line of Algorithm 2).
// These steps are tiny next to the convolutions; they are written as fused wavefront /
// workgroup reductions with a fixed summation order (deterministic).
#include "nf_internal.h"

namespace nf {
namespace {

constexpr int HT = 256;  // threads per workgroup in this file

__device__ inline void adaptive_window(int i, int L, int O, int &lo, int &hi) {
  lo = (i * L) / O;
  hi = ((i + 1) * L + O - 1) / O;
}

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// One workgroup per sample: pool U[n] -> Pq[n], logits, log-sum-exp, per-sample loss, dL/dz.
// Dynamic LDS: Pq (F floats) + z (Cls floats) + partial pool sums (G*F floats) + 8 scratch.
__global__ __launch_bounds__(HT) void head_fwd_kernel(HeadShape s, const float *__restrict__ U,
                                                      const int32_t *__restrict__ labels,
                                                      const float *__restrict__ Wf, const float *__restrict__ bf,
                                                      float *__restrict__ Pq, float *__restrict__ dz,
                                                      float *__restrict__ loss_n, int G) {
  extern __shared__ float sm[];
  float *pq = sm;               // [F]
  float *z = pq + s.F;          // [Cls]
  float *part = z + s.Cls;      // [G][F]
  float *red = part + G * s.F;  // [8]
  const int n = blockIdx.x, t = threadIdx.x;
  const float *Un = U + (long long)n * s.Hu * s.Wu * s.A;

  // ---- F_n: adaptive average pool; group g of G sums every G-th row of each window ----
  for (int idx = t; idx < G * s.F; idx += HT) {
    const int g = idx / s.F, f = idx - g * s.F;
    const int cell = f / s.A, a = f - cell * s.A;
    const int i = cell / s.ow, jj = cell - i * s.ow;
    int h0, h1, w0, w1;
    adaptive_window(i, s.Hu, s.oh, h0, h1);
    adaptive_window(jj, s.Wu, s.ow, w0, w1);
    float acc = 0.f;
    for (int hh = h0 + g; hh < h1; hh += G)
      for (int ww = w0; ww < w1; ++ww) acc += Un[((long long)hh * s.Wu + ww) * s.A + a];
    part[idx] = acc;
  }
  __syncthreads();
  for (int f = t; f < s.F; f += HT) {
    const int cell = f / s.A;
    const int i = cell / s.ow, jj = cell - i * s.ow;
    int h0, h1, w0, w1;
    adaptive_window(i, s.Hu, s.oh, h0, h1);
    adaptive_window(jj, s.Wu, s.ow, w0, w1);
    float acc = 0.f;
    for (int g = 0; g < G; ++g) acc += part[g * s.F + f];
    const float v = acc / (float)((h1 - h0) * (w1 - w0));
    pq[f] = v;
    Pq[(long long)n * s.F + f] = v;
  }
  __syncthreads();

  // ---- gamma_n: one wavefront per class, lanes over features ----
  const int lane = t & 63, wave = t >> 6;
  for (int q = wave; q < s.Cls; q += HT / 64) {
    const float *wr = Wf + (long long)q * s.F;
    float acc = 0.f;
    for (int f = lane; f < s.F; f += 64) acc += wr[f] * pq[f];
    acc = wave_sum(acc);
    if (lane == 0) z[q] = acc + (bf ? bf[q] : 0.f);
  }
  __syncthreads();

  // ---- softmax cross-entropy ----
  float m = -INFINITY;
  for (int q = t; q < s.Cls; q += HT) m = fmaxf(m, z[q]);
  m = wave_max(m);
  if (lane == 0) red[wave] = m;
  __syncthreads();
  m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float se = 0.f;
  for (int q = t; q < s.Cls; q += HT) se += expf(z[q] - m);
  se = wave_sum(se);
  if (lane == 0) red[4 + wave] = se;
  __syncthreads();
  se = (red[4] + red[5]) + (red[6] + red[7]);
  const float lse = m + logf(se);
  const int y = labels[n];
  const float invB = 1.f / (float)s.B;
  for (int q = t; q < s.Cls; q += HT) dz[(long long)n * s.Cls + q] = (expf(z[q] - lse) - (q == y ? 1.f : 0.f)) * invB;
  if (t == 0) loss_n[n] = lse - ((y >= 0 && y < s.Cls) ? z[y] : 0.f);
}

// batch mean of the per-sample losses, fixed order
__global__ __launch_bounds__(HT) void loss_mean_kernel(const float *__restrict__ loss_n, int B,
                                                       float *__restrict__ out) {
  __shared__ float red[HT];
  float acc = 0.f;
  for (int i = threadIdx.x; i < B; i += HT) acc += loss_n[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = HT / 2; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = red[0] / (float)B;
}

// gamma_n backward in one launch:
//   blocks [0, nb_w)          one class q and one chunk of `fch` features: the 256 threads are
//                             fch feature lanes x (256/fch) batch slices; slice sums are added in
//                             order through LDS.  dWf[q][f] = sum_n dz[n][q] * Pq[n][f];
//                             chunk 0 also forms dbf[q] = sum_n dz[n][q].
//   blocks [nb_w, nb_w+nb_p)  dPq[n][f] = sum_q dz[n][q] * Wf[q][f], one thread per element
__global__ __launch_bounds__(HT) void fc_bwd_kernel(HeadShape s, const float *__restrict__ Pq,
                                                    const float *__restrict__ dz, const float *__restrict__ Wf,
                                                    float *__restrict__ dWf, float *__restrict__ dbf,
                                                    float *__restrict__ dPq, int nb_w, int fch, int nchunks) {
  __shared__ float red[HT];
  __shared__ float redb[HT];
  const int b = blockIdx.x, t = threadIdx.x;
  if (b < nb_w) {
    const int q = b / nchunks, chunk = b - q * nchunks;
    const int fl = t % fch, ns = t / fch, NS = HT / fch;
    const int f = chunk * fch + fl;
    float acc = 0.f, bsum = 0.f;
    if (f < s.F) {
      for (int n = ns; n < s.B; n += NS) {
        const float d = dz[(long long)n * s.Cls + q];
        bsum += d;
        acc += d * Pq[(long long)n * s.F + f];
      }
    }
    red[t] = acc;
    redb[t] = bsum;
    __syncthreads();
    if (ns == 0 && f < s.F) {
      for (int k = 1; k < NS; ++k) acc += red[k * fch + fl];
      dWf[(long long)q * s.F + f] = acc;
    }
    if (t == 0 && chunk == 0) {
      for (int k = 1; k < NS; ++k) bsum += redb[k * fch];
      dbf[q] = bsum;
    }
  } else {
    const long long i = (long long)(b - nb_w) * HT + t;
    if (i >= (long long)s.B * s.F) return;
    const int n = (int)(i / s.F), f = (int)(i - (long long)n * s.F);
    float acc = 0.f;
    for (int q = 0; q < s.Cls; ++q) acc += dz[(long long)n * s.Cls + q] * Wf[(long long)q * s.F + f];
    dPq[i] = acc;
  }
}

// F_n backward + the aux ReLU mask: dU = [U > 0] * sum over windows containing (h,w) of dPq / |window|
__global__ __launch_bounds__(HT) void pool_relu_bwd_kernel(HeadShape s, const float *__restrict__ U,
                                                           const float *__restrict__ dPq, float *__restrict__ dU) {
  const long long total = (long long)s.B * s.Hu * s.Wu * s.A;
  const long long i = (long long)blockIdx.x * HT + threadIdx.x;
  if (i >= total) return;
  const int a = (int)(i % s.A);
  long long r = i / s.A;
  const int w = (int)(r % s.Wu);
  r /= s.Wu;
  const int hh = (int)(r % s.Hu);
  const int n = (int)(r / s.Hu);
  float acc = 0.f;
  if (!s.relu || U[i] > 0.f) {
    for (int ci = 0; ci < s.oh; ++ci) {
      int h0, h1;
      adaptive_window(ci, s.Hu, s.oh, h0, h1);
      if (hh < h0 || hh >= h1) continue;
      for (int cj = 0; cj < s.ow; ++cj) {
        int w0, w1;
        adaptive_window(cj, s.Wu, s.ow, w0, w1);
        if (w < w0 || w >= w1) continue;
        acc += dPq[(long long)n * s.F + (ci * s.ow + cj) * s.A + a] / (float)((h1 - h0) * (w1 - w0));
      }
    }
  }
  dU[i] = acc;
}

}  // namespace

hipError_t launch_head_fwd(const HeadShape &h, const float *U, const int32_t *labels, const float *Wf,
                           const float *bf, float *Pq, float *dz, float *loss_n, hipStream_t st) {
  int G = 1;
  const int rows = (h.Hu + h.oh - 1) / h.oh;
  while (G * 2 * h.F <= 2 * HT && G * 2 <= rows) G *= 2;
  const size_t lds = (size_t)(h.F + h.Cls + G * h.F + 8) * sizeof(float);
  hipLaunchKernelGGL(head_fwd_kernel, dim3(h.B), dim3(HT), lds, st, h, U, labels, Wf, bf, Pq, dz, loss_n, G);
  return hipGetLastError();
}

hipError_t launch_loss_mean(const float *loss_n, int B, float *loss_out, hipStream_t st) {
  hipLaunchKernelGGL(loss_mean_kernel, dim3(1), dim3(HT), 0, st, loss_n, B, loss_out);
  return hipGetLastError();
}

hipError_t launch_fc_bwd(const HeadShape &h, const float *Pq, const float *dz, const float *Wf, float *dWf,
                         float *dbf, float *dPq, hipStream_t st) {
  int fch = 16;
  while (fch < 64 && fch < h.F) fch *= 2;
  const int nchunks = (h.F + fch - 1) / fch;
  const int nb_w = h.Cls * nchunks;
  const int nb_p = (int)(((long long)h.B * h.F + HT - 1) / HT);
  hipLaunchKernelGGL(fc_bwd_kernel, dim3(nb_w + nb_p), dim3(HT), 0, st, h, Pq, dz, Wf, dWf, dbf, dPq, nb_w, fch,
                     nchunks);
  return hipGetLastError();
}

hipError_t launch_pool_relu_bwd(const HeadShape &h, const float *U, const float *dPq, float *dU, hipStream_t st) {
  const long long total = (long long)h.B * h.Hu * h.Wu * h.A;
  hipLaunchKernelGGL(pool_relu_bwd_kernel, dim3((unsigned)((total + HT - 1) / HT)), dim3(HT), 0, st, h, U, dPq, dU);
  return hipGetLastError();
}

}  // namespace nf
