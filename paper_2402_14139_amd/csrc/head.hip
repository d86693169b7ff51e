// The auxiliary head after its convolution (NeuroFlux, arXiv 2402.14139, Eq. 2 and Eq. 3):
// adaptive average (or max) pooling F_n, the linear layer gamma_n, softmax cross-entropy (or
// mean squared error against the one-hot label) with the batch mean, and the backward of those
// three (gradient line of Algorithm 2).
// These steps are tiny next to the convolutions; they are written as fused wavefront /
// workgroup reductions with a fixed summation order (deterministic).
#include "head_gamma.h"
#include "nf_internal.h"

namespace nf {
namespace {

constexpr int HT = 256;  // threads per workgroup in this file
static_assert(HT == GJ_T, "the batch-reducing jobs assume this workgroup size");

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
// (all threads of a workgroup; pairs [pair0, pair0 + G) below pair_end; red / redi: HT*V entries of
// LDS; pq_lds / parg_lds, when given, also receive the results at index (pair - lds_pair0) * A + channel)
template <int V, bool PMAX>
__device__ inline void pool_pairs(const HeadShape &s, long long pair0, long long pair_end, float *__restrict__ U,
                                  const float *__restrict__ part, int splits, const float *__restrict__ ba,
                                  float *__restrict__ Pq, int32_t *__restrict__ parg, int CA, int NS, float *red,
                                  int *redi, float *pq_lds, int *parg_lds, long long lds_pair0) {
  const int t = threadIdx.x;
  const int per = CA * NS, G = HT / per;
  const int grp = t / per, tg = t - grp * per;
  const int lane = tg % CA, slice = tg / CA;
  const int cells = s.oh * s.ow;
  const long long pair = pair0 + grp;
  const bool live = grp < G && pair < pair_end;
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
          if (pq_lds) {
            const int li = (int)(pair - lds_pair0) * s.A + col * V + e;
            pq_lds[li] = best, parg_lds[li] = bp;
          }
        } else {
          float sum = acc[e];
          for (int k = 1; k < NS; ++k) sum += red[(grp * per + k * CA + lane) * V + e];
          Pq[o] = sum * inv;
          if (pq_lds) pq_lds[(int)(pair - lds_pair0) * s.A + col * V + e] = sum * inv;
        }
      }
    }
  }
}

template <int V, bool PMAX>
__global__ __launch_bounds__(HT) void head_pool_kernel(HeadShape s, float *__restrict__ U,
                                                       const float *__restrict__ part, int splits,
                                                       const float *__restrict__ ba, float *__restrict__ Pq,
                                                       int32_t *__restrict__ parg, int CA, int NS) {
  __shared__ float red[HT * V];
  __shared__ int redi[PMAX ? HT * V : 1];
  const int G = HT / (CA * NS);
  pool_pairs<V, PMAX>(s, (long long)blockIdx.x * G, (long long)s.B * s.oh * s.ow, U, part, splits, ba, Pq, parg, CA, NS,
                      red, redi, nullptr, nullptr, 0);
}

// gamma_n and Eq. 3 for one sample (all threads of a workgroup): logits (one thread per class, the
// pooled features pq[F] already staged in LDS), log-sum-exp, per-sample loss, dL/dz, and -- the
// sample's dz being at hand -- the gradient w.r.t. the pooled features
// dPq[f] = sum_q dz[q] * Wf[q][f], stored to dPq_out (global row of the sample, or an LDS array).
// z: Cls floats of LDS, red: 8 floats of LDS.  write = false: dz and the loss are formed but not
// stored (a workgroup that only needs dPq of a sample another workgroup reports).
__device__ inline void fc_loss_sample(const HeadShape &s, int n, const float *pq, float *z, float *red,
                                      const int32_t *__restrict__ labels, const float *__restrict__ Wf,
                                      const float *__restrict__ bf, float *__restrict__ dz,
                                      float *__restrict__ loss_n, float *dPq_out, bool write = true) {
  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  // logits: P threads per class, each over a contiguous 1/P of the features (P a power of two with
  // P * Cls <= 256 and whole 16-byte groups per part), so that one batch of independent loads per
  // thread covers the row; the P partial sums are added in order through LDS
  __shared__ float zp[HT];
  int P = 1;
  if ((s.F & 3) == 0)
    while (P < 8 && 2 * P * s.Cls <= HT && ((s.F >> 2) % (2 * P)) == 0) P *= 2;
  if (s.Cls <= HT) {
    const int part = t / s.Cls, q = t - part * s.Cls;
    if (part < P) {
      const int fn = s.F / P, f0 = part * fn;
      const float *wr = Wf + (long long)q * s.F + f0;
      float acc = 0.f;
      if ((s.F & 3) == 0) {
#pragma unroll 8
        for (int f = 0; f < fn; f += 4) {
          const float4 w = *reinterpret_cast<const float4 *>(wr + f);
          acc += w.x * pq[f0 + f] + w.y * pq[f0 + f + 1] + w.z * pq[f0 + f + 2] + w.w * pq[f0 + f + 3];
        }
      } else {
        for (int f = 0; f < fn; ++f) acc += wr[f] * pq[f0 + f];
      }
      zp[t] = acc;
    }
    __syncthreads();
    if (t < s.Cls) {
      float acc = zp[t];
      for (int k = 1; k < P; ++k) acc += zp[k * s.Cls + t];
      z[t] = acc + (bf ? bf[t] : 0.f);
    }
  } else {
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
  }
  __syncthreads();

  if (s.mse) {
    // squared error against the one-hot label, mean over the classes (the batch mean follows)
    const int y = labels[n];
    const float sc = 2.f / ((float)s.B * (float)s.Cls);
    float se = 0.f;
    for (int q = t; q < s.Cls; q += HT) {
      const float e = z[q] - (q == y ? 1.f : 0.f);
      se += e * e;
      if (write) dz[(long long)n * s.Cls + q] = e * sc;
    }
    se = wave_sum(se);
    if (lane == 0) red[wave] = se;
    __syncthreads();
    if (t == 0 && write) loss_n[n] = ((red[0] + red[1]) + (red[2] + red[3])) / (float)s.Cls;
    for (int q = t; q < s.Cls; q += HT) z[q] = (z[q] - (q == y ? 1.f : 0.f)) * sc;
    __syncthreads();
    for (int f = t; f < s.F; f += HT) {
      float acc = 0.f;
#pragma unroll 4
      for (int q = 0; q < s.Cls; ++q) acc += z[q] * Wf[(long long)q * s.F + f];
      dPq_out[f] = acc;
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
    if (write) dz[(long long)n * s.Cls + q] = d;
    z[q] = d;
  }
  if (t == 0 && write) loss_n[n] = lse - zy;
  __syncthreads();
  for (int f = t; f < s.F; f += HT) {
    float acc = 0.f;
#pragma unroll 10
    for (int q = 0; q < s.Cls; ++q) acc += z[q] * Wf[(long long)q * s.F + f];
    dPq_out[f] = acc;
  }
}

// One sample per workgroup.  Dynamic LDS: F + Cls + 8 floats.
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
  fc_loss_sample(s, n, pq, z, red, labels, Wf, bf, dz, loss_n, dPq + (long long)n * s.F);
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

__global__ __launch_bounds__(HT) void loss_mean_kernel(const float *__restrict__ loss_n, int B,
                                                       float *__restrict__ out) {
  __shared__ float red[HT];
  loss_mean_block(loss_n, B, out, red);
}

// dU for V consecutive channels of one element (n, hh, w, av): F_n backward + aux ReLU mask.
// dpq points at the sample's dPq[F] (global or LDS), pargn at its selection record (max pooling).
template <int V>
__device__ inline void du_element(const HeadShape &s, int hh, int w, int av, const float *__restrict__ u_at,
                                  const float *dpq, const int32_t *pargn, float *__restrict__ du_at) {
  float u[V], acc[V];
  if constexpr (V == 4) {
    const float4 t4 = *reinterpret_cast<const float4 *>(u_at);
    u[0] = t4.x, u[1] = t4.y, u[2] = t4.z, u[3] = t4.w;
  } else {
    u[0] = u_at[0];
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
      const int fo = (ci * s.ow + cj) * s.A + av * V;
      const float *src = dpq + fo;
      if (s.pmax) {  // max pooling hands the gradient to the element it selected
#pragma unroll
        for (int e = 0; e < V; ++e)
          if (pargn[fo + e] == hh * s.Wu + w) acc[e] += src[e];
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
    *reinterpret_cast<float4 *>(du_at) = make_float4(acc[0], acc[1], acc[2], acc[3]);
  } else {
    du_at[0] = acc[0];
  }
}

// element i of the re-laid aux filter: WaT[k][r][s][a] = Wa[a][R-1-r][S-1-s][k]
__device__ inline void wat_element(long long i, int A, int R, int S, int K, const float *__restrict__ Wa,
                                   float *__restrict__ WaT) {
  const int a = (int)(i % A);
  long long r = i / A;
  const int sx = (int)(r % S);
  r /= S;
  const int rr = (int)(r % R);
  const int k = (int)(r / R);
  WaT[i] = Wa[(((long long)a * R + (R - 1 - rr)) * S + (S - 1 - sx)) * K + k];
}

// The whole per-sample chain of a head with a small activation map in one launch: workgroup n
// (n < B) runs F_n, gamma_n, the loss and dL/dz, dPq and the backward through F_n and the aux ReLU
// for sample n; the pooled features, dPq and the max-pooling selection stay in LDS between the
// stages.  With splits > 0 the aux activation is first formed from the raw partial sums of the
// split aux convolution (see pool_pairs).  Workgroups from B on re-lay the aux filter for the
// data gradient.
// Dynamic LDS: 2*F + Cls + 8 floats, + F ints for max pooling.
template <int V, bool PMAX>
__global__ __launch_bounds__(HT) void head_sample_kernel(HeadShape s, float *__restrict__ U,
                                                         const float *__restrict__ part, int splits,
                                                         const float *__restrict__ ba,
                                                         const int32_t *__restrict__ labels,
                                                         const float *__restrict__ Wf, const float *__restrict__ bf,
                                                         float *__restrict__ Pq, int32_t *__restrict__ parg,
                                                         float *__restrict__ dz, float *__restrict__ loss_n,
                                                         float *__restrict__ dU, const float *__restrict__ Wa,
                                                         float *__restrict__ WaT, int R, int S, int K, int CA, int NS) {
  extern __shared__ float sm[];
  __shared__ float red[HT * V];
  __shared__ int redi[PMAX ? HT * V : 1];
  const int t = threadIdx.x;
  if ((int)blockIdx.x >= s.B) {
    const long long i = (long long)(blockIdx.x - s.B) * HT + t;
    if (i < (long long)s.A * R * S * K) wat_element(i, s.A, R, S, K, Wa, WaT);
    return;
  }
  float *pq = sm;            // [F]
  float *dpq = pq + s.F;     // [F]
  float *z = dpq + s.F;      // [Cls]
  float *red8 = z + s.Cls;   // [8]
  int *pargl = reinterpret_cast<int *>(red8 + 8);  // [F] (max pooling)
  const int n = blockIdx.x;
  const int cells = s.oh * s.ow, G = HT / (CA * NS);
  for (int c0 = 0; c0 < cells; c0 += G)
    pool_pairs<V, PMAX>(s, (long long)n * cells + c0, (long long)(n + 1) * cells, U, part, splits, ba, Pq, parg, CA,
                        NS, red, redi, pq, PMAX ? pargl : nullptr, (long long)n * cells);
  __syncthreads();  // (with splits > 0 the sample's U was formed and written on the way: visible to the workgroup)
  fc_loss_sample(s, n, pq, z, red8, labels, Wf, bf, dz, loss_n, dpq);
  __syncthreads();
  const int AV = s.A / V, per_n = s.Hu * s.Wu * AV;
  const long long base = (long long)n * per_n;
  for (int i = t; i < per_n; i += HT) {
    const int av = i % AV, r = i / AV;
    const int w = r % s.Wu, hh = r / s.Wu;
    du_element<V>(s, hh, w, av, U + (base + i) * V, dpq, PMAX ? pargl : nullptr, dU + (base + i) * V);
  }
}

// Everything of the head after F_n for a LARGE activation map in one launch: gamma_n, the loss and
// dL/dz, dPq, and the backward through F_n and the aux ReLU (dU).  A sample's map is cut into NS
// slices, one workgroup each, so that the launch has enough workgroups to stream dU; every one of
// them recomputes the sample's tiny linear layer (F * Cls products, Wf from L2) instead of reading
// dPq from an earlier launch, and slice 0 stores dz and the per-sample loss.  Workgroups from
// B * NS on re-lay the aux filter for the data gradient.  With `ppart` given, F_n itself is formed
// here too (and Pq stored by slice 0) from the column sums the aux convolution's epilogue left.
// Dynamic LDS: 2*F + Cls + 8 floats.
template <int V>
__global__ __launch_bounds__(HT) void head_wide_kernel(HeadShape s, int NS, const float *__restrict__ U,
                                                       float *__restrict__ Pq, const float *__restrict__ ppart,
                                                       const int32_t *__restrict__ labels,
                                                       const float *__restrict__ Wf, const float *__restrict__ bf,
                                                       float *__restrict__ dz, float *__restrict__ loss_n,
                                                       const int32_t *__restrict__ parg, float *__restrict__ dU,
                                                       const float *__restrict__ Wa, float *__restrict__ WaT, int R,
                                                       int S, int K) {
  extern __shared__ float sm[];
  const int t = threadIdx.x;
  if ((int)blockIdx.x >= s.B * NS) {
    const long long i = (long long)(blockIdx.x - s.B * NS) * HT + t;
    if (i < (long long)s.A * R * S * K) wat_element(i, s.A, R, S, K, Wa, WaT);
    return;
  }
  float *pq = sm;            // [F]
  float *dpq = pq + s.F;     // [F]
  float *z = dpq + s.F;      // [Cls]
  float *red8 = z + s.Cls;   // [8]
  const int n = blockIdx.x / NS, sl = blockIdx.x - n * NS;
  if (ppart) {
    // F_n (2x2 average pooling of an even-sized map) from the column sums the aux convolution left
    // per 16 consecutive pixels: image rows of 16 pixels carry both halves in two slots, wider rows
    // are whole 16-pixel groups per half.  Rows ascending, groups ascending: a fixed order.
    const bool split = s.Wu == 16;
    const int gpr = s.Wu >> 4;                // 16-pixel groups per image row
    const int gph = split ? 1 : (gpr >> 1);   // ... per half row
    const float inv = 1.f / (float)((s.Hu >> 1) * (s.Wu >> 1));
    for (int f = t; f < s.F; f += HT) {
      const int cell = f / s.A, a = f - cell * s.A;
      const int ci = cell >> 1, cj = cell & 1;
      // partial i of the cell: image row ci*Hu/2 + i / gph, group i % gph of the half row; loaded
      // eight at a time (independent loads), added in order
      const int np = (s.Hu >> 1) * gph;
      const float *src = ppart + (split ? cj : 0) * s.A + a;
      float acc = 0.f;
      for (int i0 = 0; i0 < np; i0 += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int i = i0 + u, hr = i / gph;
          const long long r16 = ((long long)n * s.Hu + ci * (s.Hu >> 1) + hr) * gpr + (split ? 0 : cj * gph + (i - hr * gph));
          v[u] = i < np ? src[r16 * 2 * s.A] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
      }
      pq[f] = acc * inv;
      if (sl == 0) Pq[(long long)n * s.F + f] = acc * inv;
    }
  } else {
    for (int f = t; f < s.F; f += HT) pq[f] = Pq[(long long)n * s.F + f];
  }
  __syncthreads();
  fc_loss_sample(s, n, pq, z, red8, labels, Wf, bf, dz, loss_n, dpq, sl == 0);
  __syncthreads();
  const int AV = s.A / V, per_n = s.Hu * s.Wu * AV;
  const int per_sl = (per_n + NS - 1) / NS;
  const int i1 = min(per_n, (sl + 1) * per_sl);
  const long long base = (long long)n * per_n;
  for (int i = sl * per_sl + t; i < i1; i += HT) {
    const int av = i % AV, r = i / AV;
    const int w = r % s.Wu, hh = r / s.Wu;
    du_element<V>(s, hh, w, av, U + (base + i) * V, dpq, s.pmax ? parg + (long long)n * s.F : nullptr,
                  dU + (base + i) * V);
  }
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
    GammaJob g;
    g.B = s.B, g.F = s.F, g.Cls = s.Cls, g.Pq = Pq, g.dz = dz, g.dWf = dWf, g.dbf = dbf;
    g.Wf = g.bf = g.vWf = g.vbf = nullptr, g.lr = g.mu = 0.f;
    g.fch = jb.fch, g.nchunks = jb.nchunks;
    gamma_block(g, b, red, redb);
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
    du_element<V>(s, hh, w, av, U + i * V, dPq + (long long)n * s.F, s.pmax ? parg + (long long)n * s.F : nullptr,
                  dU + i * V);
    return;
  }
  b -= jb.nb_u;
  if (b < jb.nb_t) {
    const long long total = (long long)s.A * R * S * K;
    const long long i = (long long)b * HT + t;
    if (i >= total) return;
    wat_element(i, s.A, R, S, K, Wa, WaT);
    return;
  }
  loss_mean_block(loss_n, s.B, loss_out, red);
}

}  // namespace

// pooling decomposition of a workgroup (see pool_pairs): channel lanes CA, position slices NS
static void pool_lanes(const HeadShape &h, int V, int *CA_out, int *NS_out) {
  const int AV = h.A / V;
  int CA = 1;
  while (CA < AV && CA < HT) CA *= 2;  // channel lanes: power of two covering A / V (or all threads)
  // largest pooling window -> position slices (power of two, at most what the workgroup has left)
  const int wh = (h.Hu + h.oh - 1) / h.oh + (h.Hu % h.oh ? 1 : 0), wwid = (h.Wu + h.ow - 1) / h.ow + (h.Wu % h.ow ? 1 : 0);
  int NS = 1;
  while (NS * 2 <= wh * wwid && CA * NS * 2 <= HT) NS *= 2;
  *CA_out = CA, *NS_out = NS;
}

hipError_t launch_head_pool(const HeadShape &h, float *U, const float *part, int splits, const float *ba, float *Pq,
                            int32_t *parg, hipStream_t st) {
  const int V = h.A % 4 == 0 ? 4 : 1;
  int CA, NS;
  pool_lanes(h, V, &CA, &NS);
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

bool head_sample_applicable(const HeadShape &h) {
  // a sample's activation map of at most 4 KiB (measured: at 16 KiB per sample and 128 samples the
  // three chip-wide launches are faster than 128 workgroups doing a sample each), the linear layer
  // narrow enough that sharing its weights between samples (head_fc_wide_kernel) does not pay
  return (long long)h.Hu * h.Wu * h.A <= 1024 && h.F <= 256 && h.Cls <= 1024;
}

hipError_t launch_head_sample(const HeadShape &h, float *U, const float *part, int splits, const float *ba,
                              const int32_t *labels, const float *Wf, const float *bf, float *Pq, int32_t *parg, float *dz, float *loss_n, float *dU, const float *Wa,
                              float *WaT, int R, int S, int K, hipStream_t st) {
  const int V = h.A % 4 == 0 ? 4 : 1;
  int CA, NS;
  pool_lanes(h, V, &CA, &NS);
  const unsigned nb_t = Wa ? (unsigned)(((long long)h.A * R * S * K + HT - 1) / HT) : 0;
  const dim3 grid((unsigned)h.B + nb_t);
  const size_t lds = (size_t)(2 * h.F + h.Cls + 8) * sizeof(float) + (h.pmax ? (size_t)h.F * sizeof(int) : 0);
#define NF_HS(V_, P_)                                                                                              \
  hipLaunchKernelGGL((head_sample_kernel<V_, P_>), grid, dim3(HT), lds, st, h, U, part, splits, ba, labels, Wf, bf, Pq, \
                     parg, dz, loss_n, dU, Wa, WaT, R, S, K, CA, NS)
  if (h.pmax) {
    if (V == 4) NF_HS(4, true);
    else NF_HS(1, true);
  } else {
    if (V == 4) NF_HS(4, false);
    else NF_HS(1, false);
  }
#undef NF_HS
  return hipGetLastError();
}

bool head_wide_applicable(const HeadShape &h) {
  // the linear layer small enough to be recomputed by every slice of a sample (its weights read
  // from L2 by every workgroup); wider ones share the weights between samples (head_fc_wide_kernel)
  return !head_sample_applicable(h) && (long long)h.F * h.Cls <= 16384 && h.F <= 1024 && h.Cls <= 1024;
}

bool head_pool_partials_applicable(const HeadShape &h) {
  // 2x2 average pooling of an even-sized map whose rows are whole groups of 16 pixels per half (or
  // exactly 16 pixels: the two halves are the two 8-pixel sums of a group)
  return !h.pmax && h.oh == 2 && h.ow == 2 && h.Hu % 2 == 0 && (h.Wu == 16 || h.Wu % 32 == 0);
}

hipError_t launch_head_wide(const HeadShape &h, const float *U, float *Pq, const float *ppart, const int32_t *labels,
                            const float *Wf, const float *bf, float *dz, float *loss_n, const int32_t *parg,
                            float *dU, const float *Wa, float *WaT, int R, int S, int K, hipStream_t st) {
  const int V = h.A % 4 == 0 ? 4 : 1;
  // slices per sample: about 768 workgroups in all, at least 1024 values of dU each
  const long long per_sample = (long long)h.Hu * h.Wu * h.A;
  int NS = (768 + h.B - 1) / h.B;
  if (NS > per_sample / 1024) NS = (int)(per_sample / 1024);
  if (NS < 1) NS = 1;
  const unsigned nb_t = Wa ? (unsigned)(((long long)h.A * R * S * K + HT - 1) / HT) : 0;
  const dim3 grid((unsigned)(h.B * NS) + nb_t);
  const size_t lds = (size_t)(2 * h.F + h.Cls + 8) * sizeof(float);
  if (V == 4)
    hipLaunchKernelGGL(head_wide_kernel<4>, grid, dim3(HT), lds, st, h, NS, U, Pq, ppart, labels, Wf, bf, dz, loss_n, parg, dU,
                       Wa, WaT, R, S, K);
  else
    hipLaunchKernelGGL(head_wide_kernel<1>, grid, dim3(HT), lds, st, h, NS, U, Pq, ppart, labels, Wf, bf, dz, loss_n, parg, dU,
                       Wa, WaT, R, S, K);
  return hipGetLastError();
}

int gamma_job_plan(GammaJob &g) {
  // feature lanes per workgroup: few, so that many batch slices share the reduction over n
  g.fch = 8;
  while (g.fch < 32 && g.fch * 2 <= g.F) g.fch *= 2;
  g.nchunks = (g.F + g.fch - 1) / g.fch;
  g.nb_w = g.Cls * g.nchunks;
  g.nb_l = g.loss_out ? 1 : 0;
  return g.nb_w + g.nb_l;
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
  GammaJob gj;
  gj.F = h.F, gj.Cls = h.Cls, gj.loss_out = nullptr;
  gamma_job_plan(gj);
  jb.fch = gj.fch, jb.nchunks = gj.nchunks, jb.nb_w = gj.nb_w;
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
