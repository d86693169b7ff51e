// The auxiliary head after its convolution (NeuroFlux, arXiv 2402.14139, Eq. 2 and Eq. 3):
// adaptive average (or max) pooling F_n, the linear layer gamma_n, softmax cross-entropy (or
// mean squared error against the one-hot label) with the batch mean, and the backward of those
// three (gradient line of Algorithm 2).
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

// F_n: adaptive average pool (PMAX: adaptive max pool, which also records the flat position
// h*Wu+w of the first maximal element in row-major window order).  A workgroup serves G (sample,
// output cell) pairs; each pair has CA channel lanes (V channels each, 16-byte accesses when
// V == 4) x NS window-position slices, CA * NS * G = HT.  Slice results are combined in order
// through LDS.
// With splits > 0 the aux activation does not exist yet: it is formed here from the raw partial
// sums of the split aux convolution, U = act(sum_z part[z] + ba), and written out on the way.
template <int V, bool PMAX>
__global__ __launch_bounds__(HT) void head_pool_kernel(HeadShape s, float *__restrict__ U,
                                                       const float *__restrict__ part, int splits,
                                                       const float *__restrict__ ba, float *__restrict__ Pq,
                                                       int32_t *__restrict__ parg, int CA, int NS) {
  __shared__ float red[HT * V];
  __shared__ int redi[PMAX ? HT * V : 1];
  const int t = threadIdx.x;
  const int per = CA * NS, G = HT / per;
  const int grp = t / per, tg = t - grp * per;
  const int lane = tg % CA, slice = tg / CA;
  const int cells = s.oh * s.ow;
  const long long pair = (long long)blockIdx.x * G + grp;
  const bool live = grp < G && pair < (long long)s.B * cells;
  const int n = live ? (int)(pair / cells) : 0, cell = live ? (int)(pair - (long long)n * cells) : 0;
  const int ci = cell / s.ow, cj = cell - ci * s.ow;
  int h0, h1, w0, w1;
  adaptive_window(ci, s.Hu, s.oh, h0, h1);
  adaptive_window(cj, s.Wu, s.ow, w0, w1);
  const int ww = w1 - w0, npos = (h1 - h0) * ww;
  const int AV = s.A / V;
  const float inv = 1.f / (float)npos;
  const long long total = (long long)s.B * s.Hu * s.Wu * s.A;
  for (int c0 = 0; c0 < AV; c0 += CA) {
    const int col = c0 + lane;
    float acc[V];
    int bpos[V];
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = PMAX ? -INFINITY : 0.f, bpos[e] = 0x7fffffff;
    if (live && col < AV) {
      float bias[V];
#pragma unroll
      for (int e = 0; e < V; ++e) bias[e] = (splits > 0 && ba) ? ba[col * V + e] : 0.f;
#pragma unroll 4
      for (int pos = slice; pos < npos; pos += NS) {
        const int hh = h0 + pos / ww, wx = w0 + pos % ww;
        const long long at = (((long long)n * s.Hu + hh) * s.Wu + wx) * s.A + col * V;
        float v[V];
        if (splits > 0) {
#pragma unroll
          for (int e = 0; e < V; ++e) v[e] = 0.f;
          for (int z = 0; z < splits; ++z) {
            const float *src = part + (long long)z * total + at;
            if constexpr (V == 4) {
              const float4 x = *reinterpret_cast<const float4 *>(src);
              v[0] += x.x, v[1] += x.y, v[2] += x.z, v[3] += x.w;
            } else {
              v[0] += src[0];
            }
          }
#pragma unroll
          for (int e = 0; e < V; ++e) {
            v[e] += bias[e];
            if (s.relu) v[e] = v[e] > 0.f ? v[e] : 0.f;
          }
          if constexpr (V == 4) {
            *reinterpret_cast<float4 *>(U + at) = make_float4(v[0], v[1], v[2], v[3]);
          } else {
            U[at] = v[0];
          }
        } else {
          if constexpr (V == 4) {
            const float4 x = *reinterpret_cast<const float4 *>(U + at);
            v[0] = x.x, v[1] = x.y, v[2] = x.z, v[3] = x.w;
          } else {
            v[0] = U[at];
          }
        }
#pragma unroll
        for (int e = 0; e < V; ++e) {
          if constexpr (PMAX) {
            if (v[e] > acc[e]) acc[e] = v[e], bpos[e] = hh * s.Wu + wx;  // strict: first maximum of the slice
          } else {
            acc[e] += v[e];
          }
        }
      }
    }
    __syncthreads();  // previous round's reads of red are done
#pragma unroll
    for (int e = 0; e < V; ++e) {
      red[t * V + e] = acc[e];
      if constexpr (PMAX) redi[t * V + e] = bpos[e];
    }
    __syncthreads();
    if (live && slice == 0 && col < AV) {
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const long long o = (long long)n * s.F + cell * s.A + col * V + e;
        if constexpr (PMAX) {
          float best = acc[e];
          int bp = bpos[e];
          for (int k = 1; k < NS; ++k) {
            const int at = (grp * per + k * CA + lane) * V + e;
            const float cv = red[at];
            const int cp = redi[at];
            if (cv > best || (cv == best && cp < bp)) best = cv, bp = cp;  // ties: earliest position
          }
          Pq[o] = best;
          parg[o] = bp;
        } else {
          float sum = acc[e];
          for (int k = 1; k < NS; ++k) sum += red[(grp * per + k * CA + lane) * V + e];
          Pq[o] = sum * inv;
        }
      }
    }
  }
}

// gamma_n and Eq. 3 for one sample per workgroup: logits (one thread per class, the pooled
// features staged in LDS), log-sum-exp, per-sample loss, dL/dz, and -- the sample's dz being at
// hand -- the gradient w.r.t. the pooled features dPq[n][f] = sum_q dz[n][q] * Wf[q][f].
// Dynamic LDS: F + Cls + 8 floats.
__global__ __launch_bounds__(HT) void head_fc_kernel(HeadShape s, const float *__restrict__ Pq,
                                                     const int32_t *__restrict__ labels,
                                                     const float *__restrict__ Wf, const float *__restrict__ bf,
                                                     float *__restrict__ dz, float *__restrict__ loss_n,
                                                     float *__restrict__ dPq) {
  extern __shared__ float sm[];
  float *pq = sm;           // [F]
  float *z = pq + s.F;      // [Cls]
  float *red = z + s.Cls;   // [8]
  const int n = blockIdx.x, t = threadIdx.x;
  for (int f = t; f < s.F; f += HT) pq[f] = Pq[(long long)n * s.F + f];
  __syncthreads();
  for (int q = t; q < s.Cls; q += HT) {
    const float *wr = Wf + (long long)q * s.F;
    float acc = 0.f;
    if ((s.F & 3) == 0) {
#pragma unroll 8
      for (int f = 0; f < s.F; f += 4) {
        const float4 w = *reinterpret_cast<const float4 *>(wr + f);
        acc += w.x * pq[f] + w.y * pq[f + 1] + w.z * pq[f + 2] + w.w * pq[f + 3];
      }
    } else {
      for (int f = 0; f < s.F; ++f) acc += wr[f] * pq[f];
    }
    z[q] = acc + (bf ? bf[q] : 0.f);
  }
  __syncthreads();

  const int lane = t & 63, wave = t >> 6;
  if (s.mse) {
    // squared error against the one-hot label, mean over the classes (the batch mean follows)
    const int y = labels[n];
    const float sc = 2.f / ((float)s.B * (float)s.Cls);
    float se = 0.f;
    for (int q = t; q < s.Cls; q += HT) {
      const float e = z[q] - (q == y ? 1.f : 0.f);
      se += e * e;
      dz[(long long)n * s.Cls + q] = e * sc;
    }
    se = wave_sum(se);
    if (lane == 0) red[wave] = se;
    __syncthreads();
    if (t == 0) loss_n[n] = ((red[0] + red[1]) + (red[2] + red[3])) / (float)s.Cls;
    for (int q = t; q < s.Cls; q += HT) z[q] = (z[q] - (q == y ? 1.f : 0.f)) * sc;
    __syncthreads();
    for (int f = t; f < s.F; f += HT) {
      float acc = 0.f;
#pragma unroll 4
      for (int q = 0; q < s.Cls; ++q) acc += z[q] * Wf[(long long)q * s.F + f];
      dPq[(long long)n * s.F + f] = acc;
    }
    return;
  }
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
  const float zy = (y >= 0 && y < s.Cls) ? z[y] : 0.f;
  __syncthreads();  // every read of the logits is done: z[] becomes dz[]
  for (int q = t; q < s.Cls; q += HT) {
    const float d = (expf(z[q] - lse) - (q == y ? 1.f : 0.f)) * invB;
    dz[(long long)n * s.Cls + q] = d;
    z[q] = d;
  }
  if (t == 0) loss_n[n] = lse - zy;
  __syncthreads();
  for (int f = t; f < s.F; f += HT) {
    float acc = 0.f;
#pragma unroll 10
    for (int q = 0; q < s.Cls; ++q) acc += z[q] * Wf[(long long)q * s.F + f];
    dPq[(long long)n * s.F + f] = acc;
  }
}

// The same step for wide heads (many pooled features): G samples per workgroup share every load
// of Wf, and the workgroup has WT = 1024 threads so that the chip still holds as many wavefronts
// as with one sample per 256 threads.  Logits: one wavefront per class, its lanes striding the
// features (coalesced float4 reads of the class's row), wavefront sum; softmax: one wavefront per
// sample; dPq: one thread per feature, the loop over classes unrolled so that many independent
// loads are in flight.  Needs F % 4 == 0.  Dynamic LDS: G * (F + Cls) floats.
constexpr int WT = 1024;
template <int G>
__global__ __launch_bounds__(WT) void head_fc_wide_kernel(HeadShape s, const float *__restrict__ Pq,
                                                          const int32_t *__restrict__ labels,
                                                          const float *__restrict__ Wf,
                                                          const float *__restrict__ bf, float *__restrict__ dz,
                                                          float *__restrict__ loss_n, float *__restrict__ dPq) {
  extern __shared__ float sm[];
  float *pq = sm;               // [G][F]
  float *z = pq + G * s.F;      // [G][Cls]
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int n0 = blockIdx.x * G;
  const int ng = min(G, s.B - n0);
  for (int i = t * 4; i < G * s.F; i += WT * 4) {
    const int g = i / s.F;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (g < ng) v = *reinterpret_cast<const float4 *>(Pq + (long long)n0 * s.F + i);
    *reinterpret_cast<float4 *>(pq + i) = v;
  }
  __syncthreads();
  for (int q = wave; q < s.Cls; q += WT / 64) {
    const float *wr = Wf + (long long)q * s.F;
    float acc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] = 0.f;
#pragma unroll 4
    for (int f = lane * 4; f < s.F; f += 256) {
      const float4 w = *reinterpret_cast<const float4 *>(wr + f);
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float4 x = *reinterpret_cast<const float4 *>(pq + g * s.F + f);
        acc[g] += w.x * x.x + w.y * x.y + w.z * x.z + w.w * x.w;
      }
    }
    const float bias = bf ? bf[q] : 0.f;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float v = wave_sum(acc[g]);
      if (lane == 0) z[g * s.Cls + q] = v + bias;
    }
  }
  __syncthreads();
  const float invB = 1.f / (float)s.B;
  if (wave < ng && s.mse) {
    const int g = wave;
    float *zg = z + g * s.Cls;
    const int y = labels[n0 + g];
    const float sc = 2.f / ((float)s.B * (float)s.Cls);
    float se = 0.f;
    for (int q = lane; q < s.Cls; q += 64) {
      const float e = zg[q] - (q == y ? 1.f : 0.f);
      se += e * e;
      dz[(long long)(n0 + g) * s.Cls + q] = e * sc;
      zg[q] = e * sc;
    }
    se = wave_sum(se);
    if (lane == 0) loss_n[n0 + g] = se / (float)s.Cls;
  } else if (wave < ng) {
    const int g = wave;
    float *zg = z + g * s.Cls;
    float m = -INFINITY;
    for (int q = lane; q < s.Cls; q += 64) m = fmaxf(m, zg[q]);
    m = wave_max(m);
    float se = 0.f;
    for (int q = lane; q < s.Cls; q += 64) se += expf(zg[q] - m);
    se = wave_sum(se);
    const float lse = m + logf(se);
    const int y = labels[n0 + g];
    const float zy = (y >= 0 && y < s.Cls) ? zg[y] : 0.f;
    // (one wavefront owns zg: its read of zg[y] above is issued before the stores below)
    for (int q = lane; q < s.Cls; q += 64) {
      const float d = (expf(zg[q] - lse) - (q == y ? 1.f : 0.f)) * invB;
      dz[(long long)(n0 + g) * s.Cls + q] = d;
      zg[q] = d;
    }
    if (lane == 0) loss_n[n0 + g] = lse - zy;
  }
  __syncthreads();
  for (int f = t; f < s.F; f += WT) {
    float acc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] = 0.f;
#pragma unroll 20
    for (int q = 0; q < s.Cls; ++q) {
      const float w = Wf[(long long)q * s.F + f];
#pragma unroll
      for (int g = 0; g < G; ++g) acc[g] += z[g * s.Cls + q] * w;
    }
#pragma unroll
    for (int g = 0; g < G; ++g)
      if (g < ng) dPq[(long long)(n0 + g) * s.F + f] = acc[g];
  }
}

// Forward-only head for early-exit evaluation: one sample per workgroup; logits with one
// wavefront per class (lanes stride the features), then the arg-max over the classes with the
// lowest index winning among equal maxima.  Dynamic LDS: F + Cls floats.
__global__ __launch_bounds__(HT) void head_predict_kernel(HeadShape s, const float *__restrict__ Pq,
                                                          const int32_t *__restrict__ labels,
                                                          const float *__restrict__ Wf,
                                                          const float *__restrict__ bf,
                                                          float *__restrict__ logits_out, int32_t *__restrict__ pred,
                                                          int32_t *__restrict__ hit) {
  extern __shared__ float sm[];
  __shared__ float rv[HT];
  __shared__ int ri[HT];
  float *pq = sm;          // [F]
  float *z = pq + s.F;     // [Cls]
  const int n = blockIdx.x, t = threadIdx.x, lane = t & 63, wave = t >> 6;
  for (int f = t; f < s.F; f += HT) pq[f] = Pq[(long long)n * s.F + f];
  __syncthreads();
  for (int q = wave; q < s.Cls; q += HT / 64) {
    const float *wr = Wf + (long long)q * s.F;
    float acc = 0.f;
    for (int f = lane; f < s.F; f += 64) acc += wr[f] * pq[f];
    acc = wave_sum(acc);
    if (lane == 0) {
      const float v = acc + (bf ? bf[q] : 0.f);
      z[q] = v;
      if (logits_out) logits_out[(long long)n * s.Cls + q] = v;
    }
  }
  __syncthreads();
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int q = t; q < s.Cls; q += HT)
    if (z[q] > best) best = z[q], bi = q;  // ascending q, strict: lowest index of this thread's maxima
  rv[t] = best, ri[t] = bi;
  __syncthreads();
  for (int o = HT / 2; o > 0; o >>= 1) {
    if (t < o) {
      const float cv = rv[t + o];
      const int ci = ri[t + o];
      if (cv > rv[t] || (cv == rv[t] && ci < ri[t])) rv[t] = cv, ri[t] = ci;
    }
    __syncthreads();
  }
  if (t == 0) {
    const int p = ri[0] == 0x7fffffff ? 0 : ri[0];  // no logit compared greater than -inf (all NaN): class 0
    pred[n] = p;
    if (labels) hit[n] = p == labels[n] ? 1 : 0;
  }
}

__global__ __launch_bounds__(HT) void count_hits_kernel(const int32_t *__restrict__ hit, int B,
                                                        int32_t *__restrict__ out, int accumulate) {
  __shared__ int red[HT];
  int acc = 0;
  for (int i = threadIdx.x; i < B; i += HT) acc += hit[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int o = HT / 2; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = (accumulate ? *out : 0) + red[0];
}

// batch mean of the per-sample losses, fixed order (one workgroup)
__device__ inline void loss_mean_block(const float *__restrict__ loss_n, int B, float *__restrict__ out, float *red) {
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
__global__ __launch_bounds__(HT) void loss_mean_kernel(const float *__restrict__ loss_n, int B,
                                                       float *__restrict__ out) {
  __shared__ float red[HT];
  loss_mean_block(loss_n, B, out, red);
}

// Backward of the head after the softmax in one launch (gradient line of Algorithm 2); the
// workgroup index selects the job:
//   [0, nb_w)   gamma_n: one class q and one chunk of `fch` features; the 256 threads are fch
//               feature lanes x (256/fch) batch slices, slice sums added in order through LDS.
//               dWf[q][f] = sum_n dz[n][q] * Pq[n][f]; chunk 0 also forms dbf[q] = sum_n dz[n][q].
//   then nb_u   F_n backward + aux ReLU mask: dU = [U > 0] * sum over windows containing (h,w)
//               of dPq / |window| (max pooling: of dPq where the window selected (h,w)), V
//               channels per thread;
//   then nb_t   re-lay of the aux filter for the data gradient: WaT[k][r][s][a] = Wa[a][R-1-r][S-1-s][k];
//   then 0/1    batch mean of the per-sample losses (when loss_out is given).
struct HeadBwdJobs {
  int nb_w, nb_u, nb_t, fch, nchunks;
};
template <int V>
__global__ __launch_bounds__(HT) void head_bwd_kernel(HeadShape s, HeadBwdJobs jb, const float *__restrict__ Pq,
                                                      const float *__restrict__ dz, float *__restrict__ dWf,
                                                      float *__restrict__ dbf, const float *__restrict__ U,
                                                      const float *__restrict__ dPq, float *__restrict__ dU,
                                                      const float *__restrict__ Wa, float *__restrict__ WaT, int R,
                                                      int S, int K, const float *__restrict__ loss_n,
                                                      float *__restrict__ loss_out,
                                                      const int32_t *__restrict__ parg) {
  __shared__ float red[HT];
  __shared__ float redb[HT];
  int b = blockIdx.x;
  const int t = threadIdx.x;
  if (b < jb.nb_w) {
    const int fch = jb.fch, nchunks = jb.nchunks;
    const int q = b / nchunks, chunk = b - q * nchunks;
    const int fl = t % fch, ns = t / fch, NS = HT / fch;
    const int f = chunk * fch + fl;
    float acc = 0.f, bsum = 0.f;
    if (f < s.F) {
#pragma unroll 4
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
    return;
  }
  b -= jb.nb_w;
  if (b < jb.nb_u) {
    const int AV = s.A / V;
    const long long total = (long long)s.B * s.Hu * s.Wu * AV;
    const long long i = (long long)b * HT + t;
    if (i >= total) return;
    const int av = (int)(i % AV);
    long long r = i / AV;
    const int w = (int)(r % s.Wu);
    r /= s.Wu;
    const int hh = (int)(r % s.Hu);
    const int n = (int)(r / s.Hu);
    const long long e0 = i * V;
    float u[V], acc[V];
    if constexpr (V == 4) {
      const float4 t4 = *reinterpret_cast<const float4 *>(U + e0);
      u[0] = t4.x, u[1] = t4.y, u[2] = t4.z, u[3] = t4.w;
    } else {
      u[0] = U[e0];
    }
#pragma unroll
    for (int e = 0; e < V; ++e) acc[e] = 0.f;
    for (int ci = 0; ci < s.oh; ++ci) {
      int h0, h1;
      adaptive_window(ci, s.Hu, s.oh, h0, h1);
      if (hh < h0 || hh >= h1) continue;
      for (int cj = 0; cj < s.ow; ++cj) {
        int w0, w1;
        adaptive_window(cj, s.Wu, s.ow, w0, w1);
        if (w < w0 || w >= w1) continue;
        const long long fo = (long long)n * s.F + (ci * s.ow + cj) * s.A + av * V;
        const float *src = dPq + fo;
        if (s.pmax) {  // max pooling hands the gradient to the element it selected
#pragma unroll
          for (int e = 0; e < V; ++e)
            if (parg[fo + e] == hh * s.Wu + w) acc[e] += src[e];
        } else {
          const float inv = 1.f / (float)((h1 - h0) * (w1 - w0));
#pragma unroll
          for (int e = 0; e < V; ++e) acc[e] += src[e] * inv;
        }
      }
    }
#pragma unroll
    for (int e = 0; e < V; ++e)
      if (s.relu && !(u[e] > 0.f)) acc[e] = 0.f;
    if constexpr (V == 4) {
      *reinterpret_cast<float4 *>(dU + e0) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    } else {
      dU[e0] = acc[0];
    }
    return;
  }
  b -= jb.nb_u;
  if (b < jb.nb_t) {
    const long long total = (long long)s.A * R * S * K;
    const long long i = (long long)b * HT + t;
    if (i >= total) return;
    const int a = (int)(i % s.A);
    long long r = i / s.A;
    const int sx = (int)(r % S);
    r /= S;
    const int rr = (int)(r % R);
    const int k = (int)(r / R);
    WaT[i] = Wa[(((long long)a * R + (R - 1 - rr)) * S + (S - 1 - sx)) * K + k];
    return;
  }
  loss_mean_block(loss_n, s.B, loss_out, red);
}

}  // namespace

hipError_t launch_head_pool(const HeadShape &h, float *U, const float *part, int splits, const float *ba, float *Pq,
                            int32_t *parg, hipStream_t st) {
  const int V = h.A % 4 == 0 ? 4 : 1;
  const int AV = h.A / V;
  int CA = 1;
  while (CA < AV && CA < HT) CA *= 2;  // channel lanes: power of two covering A / V (or all threads)
  // largest pooling window -> position slices (power of two, at most what the workgroup has left)
  const int wh = (h.Hu + h.oh - 1) / h.oh + (h.Hu % h.oh ? 1 : 0), wwid = (h.Wu + h.ow - 1) / h.ow + (h.Wu % h.ow ? 1 : 0);
  int NS = 1;
  while (NS * 2 <= wh * wwid && CA * NS * 2 <= HT) NS *= 2;
  const int G = HT / (CA * NS);
  const long long pairs = (long long)h.B * h.oh * h.ow;
  const dim3 grid((unsigned)((pairs + G - 1) / G));
  if (h.pmax) {
    if (V == 4)
      hipLaunchKernelGGL((head_pool_kernel<4, true>), grid, dim3(HT), 0, st, h, U, part, splits, ba, Pq, parg, CA, NS);
    else
      hipLaunchKernelGGL((head_pool_kernel<1, true>), grid, dim3(HT), 0, st, h, U, part, splits, ba, Pq, parg, CA, NS);
  } else if (V == 4) {
    hipLaunchKernelGGL((head_pool_kernel<4, false>), grid, dim3(HT), 0, st, h, U, part, splits, ba, Pq, parg, CA, NS);
  } else {
    hipLaunchKernelGGL((head_pool_kernel<1, false>), grid, dim3(HT), 0, st, h, U, part, splits, ba, Pq, parg, CA, NS);
  }
  return hipGetLastError();
}

hipError_t launch_head_fc(const HeadShape &h, const float *Pq, const int32_t *labels, const float *Wf,
                          const float *bf, float *dz, float *loss_n, float *dPq, hipStream_t st) {
  constexpr int G = 4;
  const size_t lds_wide = (size_t)G * (h.F + h.Cls) * sizeof(float);
  if (h.F >= 256 && h.F % 4 == 0 && lds_wide <= 48 * 1024) {
    hipLaunchKernelGGL(head_fc_wide_kernel<G>, dim3((h.B + G - 1) / G), dim3(WT), lds_wide, st, h, Pq, labels, Wf, bf,
                       dz, loss_n, dPq);
    return hipGetLastError();
  }
  const size_t lds = (size_t)(h.F + h.Cls + 8) * sizeof(float);
  hipLaunchKernelGGL(head_fc_kernel, dim3(h.B), dim3(HT), lds, st, h, Pq, labels, Wf, bf, dz, loss_n, dPq);
  return hipGetLastError();
}

hipError_t launch_head_predict(const HeadShape &h, const float *Pq, const int32_t *labels, const float *Wf,
                               const float *bf, float *logits_out, int32_t *pred, int32_t *hit, hipStream_t st) {
  const size_t lds = (size_t)(h.F + h.Cls) * sizeof(float);
  hipLaunchKernelGGL(head_predict_kernel, dim3(h.B), dim3(HT), lds, st, h, Pq, labels, Wf, bf, logits_out, pred, hit);
  return hipGetLastError();
}

hipError_t launch_count_hits(const int32_t *hit, int B, int32_t *out, bool accumulate, hipStream_t st) {
  hipLaunchKernelGGL(count_hits_kernel, dim3(1), dim3(HT), 0, st, hit, B, out, accumulate ? 1 : 0);
  return hipGetLastError();
}

hipError_t launch_loss_mean(const float *loss_n, int B, float *loss_out, hipStream_t st) {
  hipLaunchKernelGGL(loss_mean_kernel, dim3(1), dim3(HT), 0, st, loss_n, B, loss_out);
  return hipGetLastError();
}

hipError_t launch_head_bwd(const HeadShape &h, const float *Pq, const float *dz, float *dWf, float *dbf,
                           const float *U, const float *dPq, float *dU, const float *Wa, float *WaT, int R, int S,
                           int K, const float *loss_n, float *loss_out, const int32_t *parg, hipStream_t st) {
  HeadBwdJobs jb;
  // feature lanes per workgroup: few, so that many batch slices share the reduction over n
  jb.fch = 8;
  while (jb.fch < 32 && jb.fch * 2 <= h.F) jb.fch *= 2;
  jb.nchunks = (h.F + jb.fch - 1) / jb.fch;
  jb.nb_w = h.Cls * jb.nchunks;
  const int V = h.A % 4 == 0 ? 4 : 1;
  const long long total = (long long)h.B * h.Hu * h.Wu * (h.A / V);
  jb.nb_u = (int)((total + HT - 1) / HT);
  jb.nb_t = Wa ? (int)(((long long)h.A * R * S * K + HT - 1) / HT) : 0;
  const dim3 grid((unsigned)(jb.nb_w + jb.nb_u + jb.nb_t + (loss_out ? 1 : 0)));
  if (V == 4)
    hipLaunchKernelGGL(head_bwd_kernel<4>, grid, dim3(HT), 0, st, h, jb, Pq, dz, dWf, dbf, U, dPq, dU, Wa, WaT, R, S, K,
                       loss_n, loss_out, parg);
  else
    hipLaunchKernelGGL(head_bwd_kernel<1>, grid, dim3(HT), 0, st, h, jb, Pq, dz, dWf, dbf, U, dPq, dU, Wa, WaT, R, S, K,
                       loss_n, loss_out, parg);
  return hipGetLastError();
}

}  // namespace nf
