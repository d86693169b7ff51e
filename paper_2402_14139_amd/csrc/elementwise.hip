// Memory-bound kernels of the local training step (NeuroFlux, arXiv 2402.14139):
// the max-pool P_n of Eq. 1 and its backward, the filter flip/transpose used by the data
// gradient of beta_n, the update line of Algorithm 2 (SGD with momentum, all tensors of a
// layer in one launch), and the activation-cache row copies (write, and read with
// re-batching / gather).  All are 16-byte vectorised where shapes allow and bounded by HBM.
#include "nf_internal.h"

namespace nf {
namespace {

constexpr int ET = 256;

// ---- P_n: max-pool over NHWC, records the window-local index of the first maximum ----
template <int V>
__global__ __launch_bounds__(ET) void maxpool_fwd_kernel(const float *__restrict__ T, float *__restrict__ Y,
                                                         uint8_t *__restrict__ arg, int B, int Ho, int Wo, int K,
                                                         int Hp, int Wp, int pk, int ps, int pp) {
  const int KV = K / V;
  const long long total = (long long)B * Hp * Wp * KV;
  const long long i = (long long)blockIdx.x * ET + threadIdx.x;
  if (i >= total) return;
  const int kv = (int)(i % KV);
  long long r = i / KV;
  const int jw = (int)(r % Wp);
  r /= Wp;
  const int ih = (int)(r % Hp);
  const int n = (int)(r / Hp);
  float best[V];
  int bi[V];
#pragma unroll
  for (int e = 0; e < V; ++e) best[e] = -INFINITY, bi[e] = 0;
  for (int u = 0; u < pk; ++u) {
    const int hh = ih * ps + u - pp;
    if ((unsigned)hh >= (unsigned)Ho) continue;
    for (int v = 0; v < pk; ++v) {
      const int ww = jw * ps + v - pp;
      if ((unsigned)ww >= (unsigned)Wo) continue;
      const float *src = T + (((long long)n * Ho + hh) * Wo + ww) * K + kv * V;
      float tv[V];
      if constexpr (V == 4) {
        const float4 q = *reinterpret_cast<const float4 *>(src);
        tv[0] = q.x, tv[1] = q.y, tv[2] = q.z, tv[3] = q.w;
      } else {
        tv[0] = src[0];
      }
#pragma unroll
      for (int e = 0; e < V; ++e)
        if (tv[e] > best[e]) best[e] = tv[e], bi[e] = u * pk + v;
    }
  }
  const long long o = (((long long)n * Hp + ih) * Wp + jw) * K + kv * V;
  if constexpr (V == 4) {
    *reinterpret_cast<float4 *>(Y + o) = make_float4(best[0], best[1], best[2], best[3]);
    *reinterpret_cast<uchar4 *>(arg + o) = make_uchar4((uint8_t)bi[0], (uint8_t)bi[1], (uint8_t)bi[2], (uint8_t)bi[3]);
  } else {
    Y[o] = best[0];
    arg[o] = (uint8_t)bi[0];
  }
}

// ---- P_n backward fused with the layer's ReLU mask (gather form, no atomics):
// dZ[pos] = sum over pooled cells whose recorded arg-max is pos and whose value is > 0 ----
template <int V>
__global__ __launch_bounds__(ET) void maxpool_bwd_kernel(const float *__restrict__ dY, const float *__restrict__ Y,
                                                         const uint8_t *__restrict__ arg, float *__restrict__ dZ,
                                                         int B, int Ho, int Wo, int K, int Hp, int Wp, int pk,
                                                         int ps, int pp) {
  const int KV = K / V;
  const long long total = (long long)B * Ho * Wo * KV;
  const long long i = (long long)blockIdx.x * ET + threadIdx.x;
  if (i >= total) return;
  const int kv = (int)(i % KV);
  long long r = i / KV;
  const int ww = (int)(r % Wo);
  r /= Wo;
  const int hh = (int)(r % Ho);
  const int n = (int)(r / Ho);
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = 0.f;
  // pooled rows ih with ih*ps - pp <= hh < ih*ps - pp + pk
  const int ih_hi = min(Hp - 1, (hh + pp) / ps);
  const int jw_hi = min(Wp - 1, (ww + pp) / ps);
  for (int ih = ih_hi; ih >= 0 && ih * ps - pp + pk > hh; --ih) {
    const int u = hh - (ih * ps - pp);
    for (int jw = jw_hi; jw >= 0 && jw * ps - pp + pk > ww; --jw) {
      const int v = ww - (jw * ps - pp);
      const int local = u * pk + v;
      const long long o = (((long long)n * Hp + ih) * Wp + jw) * K + kv * V;
      if constexpr (V == 4) {
        // one 4-byte and two 16-byte loads, then selects (no per-element branches)
        const uint32_t a4 = *reinterpret_cast<const uint32_t *>(arg + o);
        const float4 y4 = *reinterpret_cast<const float4 *>(Y + o);
        const float4 d4 = *reinterpret_cast<const float4 *>(dY + o);
        const float yv[4] = {y4.x, y4.y, y4.z, y4.w}, dv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e)
          acc[e] += (((int)((a4 >> (8 * e)) & 0xffu) == local) & (yv[e] > 0.f)) ? dv[e] : 0.f;
      } else {
#pragma unroll
        for (int e = 0; e < V; ++e)
          if (arg[o + e] == local && Y[o + e] > 0.f) acc[e] += dY[o + e];
      }
    }
  }
  const long long oz = (((long long)n * Ho + hh) * Wo + ww) * K + kv * V;
  if constexpr (V == 4) {
    *reinterpret_cast<float4 *>(dZ + oz) = make_float4(acc[0], acc[1], acc[2], acc[3]);
  } else {
    dZ[oz] = acc[0];
  }
}

// ---- epilogue of a split forward-type contraction: sum of the parts in order, bias, identity
// shortcut, ReLU, mask (Eq. 1 after the convolution; data gradient of beta_n) ----
template <int V>
__global__ __launch_bounds__(ET) void fwd_finish_kernel(const float *__restrict__ part, int splits, long long total,
                                                        int N, const float *__restrict__ bias,
                                                        const float *__restrict__ addsrc,
                                                        const float *__restrict__ mask, int relu,
                                                        float *__restrict__ out) {
  const long long i = ((long long)blockIdx.x * ET + threadIdx.x) * V;
  if (i >= total) return;
  float v[V];
#pragma unroll
  for (int e = 0; e < V; ++e) v[e] = 0.f;
  for (int z = 0; z < splits; ++z) {
    const float *src = part + (long long)z * total + i;
    if constexpr (V == 4) {
      const float4 t = *reinterpret_cast<const float4 *>(src);
      v[0] += t.x, v[1] += t.y, v[2] += t.z, v[3] += t.w;
    } else {
      v[0] += src[0];
    }
  }
  const int n = (int)(i % N);
#pragma unroll
  for (int e = 0; e < V; ++e) {
    if (bias) v[e] += bias[n + e];
    if (addsrc) v[e] += addsrc[i + e];
    if (relu) v[e] = v[e] > 0.f ? v[e] : 0.f;
    if (mask) v[e] = mask[i + e] > 0.f ? v[e] : 0.f;
  }
  if constexpr (V == 4) {
    *reinterpret_cast<float4 *>(out + i) = make_float4(v[0], v[1], v[2], v[3]);
  } else {
    out[i] = v[0];
  }
}

// ---- update line of Algorithm 2: blockIdx.y = tensor, grid-stride over its elements ----
__global__ __launch_bounds__(ET) void sgd_kernel(SgdTensors t) {
  const int ti = blockIdx.y;
  float *__restrict__ w = t.w[ti];
  const float *__restrict__ g = t.g[ti];
  float *__restrict__ v = t.v[ti];
  const long long n = t.numel[ti];
  const bool use_v = (v != nullptr) && (t.mu != 0.f);
  const long long n4 = n >> 2;
  const long long stride = (long long)gridDim.x * ET;
  for (long long i = (long long)blockIdx.x * ET + threadIdx.x; i < n4; i += stride) {
    float4 wv = reinterpret_cast<float4 *>(w)[i];
    float4 gv = reinterpret_cast<const float4 *>(g)[i];
    if (use_v) {
      float4 vv = reinterpret_cast<float4 *>(v)[i];
      vv.x = t.mu * vv.x + gv.x, vv.y = t.mu * vv.y + gv.y, vv.z = t.mu * vv.z + gv.z, vv.w = t.mu * vv.w + gv.w;
      reinterpret_cast<float4 *>(v)[i] = vv;
      gv = vv;
    }
    wv.x -= t.lr * gv.x, wv.y -= t.lr * gv.y, wv.z -= t.lr * gv.z, wv.w -= t.lr * gv.w;
    reinterpret_cast<float4 *>(w)[i] = wv;
  }
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {  // tail of up to 3 elements
    const long long i = (n4 << 2) + threadIdx.x;
    float gv = g[i];
    if (use_v) {
      gv = t.mu * v[i] + gv;
      v[i] = gv;
    }
    w[i] -= t.lr * gv;
  }
}

// ---- activation cache rows: dst row (dst_first + n) <- src row (idx ? idx[n] : src_first + n) ----
__global__ __launch_bounds__(ET) void cache_copy_kernel(const float *__restrict__ src, float *__restrict__ dst,
                                                        const int32_t *__restrict__ src_lab,
                                                        int32_t *__restrict__ dst_lab, long long se,
                                                        long long src_first, long long dst_first,
                                                        const long long *__restrict__ idx, long long capacity) {
  const int n = blockIdx.y;
  long long srow = idx ? idx[n] : src_first + n;
  if (idx) srow = srow < 0 ? 0 : (srow >= capacity ? capacity - 1 : srow);
  const float *s = src + srow * se;
  float *d = dst + (dst_first + n) * se;
  const long long stride = (long long)gridDim.x * ET;
  if ((se & 3) == 0) {
    const long long n4 = se >> 2;
    for (long long i = (long long)blockIdx.x * ET + threadIdx.x; i < n4; i += stride)
      reinterpret_cast<float4 *>(d)[i] = reinterpret_cast<const float4 *>(s)[i];
  } else {
    for (long long i = (long long)blockIdx.x * ET + threadIdx.x; i < se; i += stride) d[i] = s[i];
  }
  if (src_lab && dst_lab && blockIdx.x == 0 && threadIdx.x == 0) dst_lab[dst_first + n] = src_lab[srow];
}

inline unsigned nblocks(long long total) { return (unsigned)((total + ET - 1) / ET); }

}  // namespace

hipError_t launch_maxpool_fwd(const float *T, float *Y, uint8_t *arg, int B, int Ho, int Wo, int K, int Hp, int Wp,
                              int pk, int ps, int pp, hipStream_t st) {
  if (K % 4 == 0)
    hipLaunchKernelGGL(maxpool_fwd_kernel<4>, dim3(nblocks((long long)B * Hp * Wp * (K / 4))), dim3(ET), 0, st, T, Y,
                       arg, B, Ho, Wo, K, Hp, Wp, pk, ps, pp);
  else
    hipLaunchKernelGGL(maxpool_fwd_kernel<1>, dim3(nblocks((long long)B * Hp * Wp * K)), dim3(ET), 0, st, T, Y, arg,
                       B, Ho, Wo, K, Hp, Wp, pk, ps, pp);
  return hipGetLastError();
}

hipError_t launch_maxpool_bwd(const float *dY, const float *Y, const uint8_t *arg, float *dZ, int B, int Ho, int Wo,
                              int K, int Hp, int Wp, int pk, int ps, int pp, hipStream_t st) {
  if (K % 4 == 0)
    hipLaunchKernelGGL(maxpool_bwd_kernel<4>, dim3(nblocks((long long)B * Ho * Wo * (K / 4))), dim3(ET), 0, st, dY, Y,
                       arg, dZ, B, Ho, Wo, K, Hp, Wp, pk, ps, pp);
  else
    hipLaunchKernelGGL(maxpool_bwd_kernel<1>, dim3(nblocks((long long)B * Ho * Wo * K)), dim3(ET), 0, st, dY, Y, arg,
                       dZ, B, Ho, Wo, K, Hp, Wp, pk, ps, pp);
  return hipGetLastError();
}

hipError_t launch_fwd_finish(const float *part, int splits, long long M, int N, const float *bias,
                             const float *addsrc, const float *mask, int relu, float *out, hipStream_t st) {
  const long long total = M * N;
  if (N % 4 == 0)
    hipLaunchKernelGGL(fwd_finish_kernel<4>, dim3(nblocks(total / 4)), dim3(ET), 0, st, part, splits, total, N, bias,
                       addsrc, mask, relu, out);
  else
    hipLaunchKernelGGL(fwd_finish_kernel<1>, dim3(nblocks(total)), dim3(ET), 0, st, part, splits, total, N, bias,
                       addsrc, mask, relu, out);
  return hipGetLastError();
}

hipError_t launch_sgd(const SgdTensors &t, hipStream_t st) {
  long long mx = 0;
  for (int i = 0; i < t.n; ++i) mx = t.numel[i] > mx ? t.numel[i] : mx;
  long long bx = (mx / 4 + ET - 1) / ET;
  if (bx < 1) bx = 1;
  if (bx > 2048) bx = 2048;
  hipLaunchKernelGGL(sgd_kernel, dim3((unsigned)bx, t.n), dim3(ET), 0, st, t);
  return hipGetLastError();
}

hipError_t launch_cache_copy(const float *src, float *dst, const int32_t *src_lab, int32_t *dst_lab,
                             long long sample_elems, long long src_first, long long dst_first,
                             const long long *idx, long long capacity, int B, hipStream_t st) {
  long long bx = (sample_elems / 4 + ET - 1) / ET;
  if (bx < 1) bx = 1;
  if (bx > 64) bx = 64;
  hipLaunchKernelGGL(cache_copy_kernel, dim3((unsigned)bx, B), dim3(ET), 0, st, src, dst, src_lab, dst_lab,
                     sample_elems, src_first, dst_first, idx, capacity);
  return hipGetLastError();
}

}  // namespace nf
