// Workgroup jobs of the head's backward that reduce over the batch (NeuroFlux, arXiv 2402.14139,
// gradient line of Algorithm 2 for the linear layer gamma_n of Eq. 2, batch mean of Eq. 3).
// They are device functions so that either the head's own backward launch (head_bwd_kernel) or
// the launch that finishes the convolution weight gradients (wgrad_reduce_kernel) can carry them
// as extra workgroups.
#pragma once
#include "nf_internal.h"

namespace nf {

constexpr int GJ_T = 256;  // threads of a workgroup running these jobs

__device__ inline void gamma_sgd(float g, float *w, float *v, long long i, float lr, float mu) {
  if (v && mu != 0.f) {
    g = mu * v[i] + g;
    v[i] = g;
  }
  w[i] -= lr * g;
}

// Workgroup b of the gamma_n job: one class q and one chunk of `fch` features; the 256 threads are
// fch feature lanes x (256/fch) batch slices, slice sums added in order through LDS.
//   dWf[q][f] = sum_n dz[n][q] * Pq[n][f];  chunk 0 also forms dbf[q] = sum_n dz[n][q].
// With g.Wf given the update line of Algorithm 2 follows at once (nothing reads the linear layer's
// parameters after the forward).  red, redb: 256 floats of LDS each.
__device__ inline void gamma_block(const GammaJob &g, int b, float *red, float *redb) {
  const int t = threadIdx.x;
  const int fch = g.fch, nchunks = g.nchunks;
  const int q = b / nchunks, chunk = b - q * nchunks;
  const int fl = t % fch, ns = t / fch, NS = GJ_T / fch;
  const int f = chunk * fch + fl;
  float acc = 0.f, bsum = 0.f;
  if (f < g.F) {
#pragma unroll 4
    for (int n = ns; n < g.B; n += NS) {
      const float d = g.dz[(long long)n * g.Cls + q];
      bsum += d;
      acc += d * g.Pq[(long long)n * g.F + f];
    }
  }
  red[t] = acc;
  redb[t] = bsum;
  __syncthreads();
  if (ns == 0 && f < g.F) {
    for (int k = 1; k < NS; ++k) acc += red[k * fch + fl];
    g.dWf[(long long)q * g.F + f] = acc;
    if (g.Wf) gamma_sgd(acc, g.Wf, g.vWf, (long long)q * g.F + f, g.lr, g.mu);
  }
  if (t == 0 && chunk == 0) {
    for (int k = 1; k < NS; ++k) bsum += redb[k * fch];
    g.dbf[q] = bsum;
    if (g.bf) gamma_sgd(bsum, g.bf, g.vbf, q, g.lr, g.mu);
  }
}

// batch mean of the per-sample losses, fixed order (one workgroup); red: 256 floats of LDS
__device__ inline void loss_mean_block(const float *__restrict__ loss_n, int B, float *__restrict__ out, float *red) {
  float acc = 0.f;
  for (int i = threadIdx.x; i < B; i += GJ_T) acc += loss_n[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = GJ_T / 2; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = red[0] / (float)B;
}

}  // namespace nf
