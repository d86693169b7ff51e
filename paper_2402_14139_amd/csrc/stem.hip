// First-layer ("stem") convolutions: few input channels, so the whole reduction R*S*C fits one
// 32-wide staging step (3x3x3 = 27 for RGB inputs).  NeuroFlux, arXiv 2402.14139: Eq. 1 for the
// first local layer (forward) and the gradient line of Algorithm 2 for its filter (weight gradient).
//
// These layers are bound by HBM, not by the MFMA pipe: the forward writes 64 output channels for 27
// multiply-adds each (arithmetic intensity ~13 flop/byte), the weight gradient reads them back.  The
// general-shape kernels spend their time in a pipelined reduction loop that here has one step;
// the kernels below stage the im2col rows once (scalar gathers: a channel count of 3 has no
// 16-byte groups), run the few MFMAs and stream the output / the dZ rows with 16-byte accesses.
#include "nf_internal.h"

namespace nf {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int NT = 256;   // threads per workgroup
constexpr int KS = 32;    // staged reduction length (R*S*C <= KS, zero padded)
constexpr int LDK = KS + 4;

// element kg = (r, s, c) of the im2col row of output pixel (img, ho, wo); zero outside the image.
// Branch-free (the address is clamped into the tensor, the value selected afterwards) so that a
// thread's gathers are all in flight together instead of one behind each branch.
__device__ inline float col_elem(const float *__restrict__ x, int H, int W, int C, int S, int RSC, int stride, int pad,
                                 int img, int ho, int wo, int kg, bool live) {
  const int k = min(kg, RSC - 1);
  const int tap = k / C, c = k - tap * C;
  const int r = tap / S, s = tap - r * S;
  const int hi = ho * stride - pad + r, wi = wo * stride - pad + s;
  const bool ok = live & (kg < RSC) & ((unsigned)hi < (unsigned)H) & ((unsigned)wi < (unsigned)W);
  const int hc = min(max(hi, 0), H - 1), wc = min(max(wi, 0), W - 1);
  const float v = x[((long long)(img * H + hc) * W + wc) * C + c];
  return ok ? v : 0.f;
}

// out[m][n] = act(bias[n] + sum_kg col[m][kg] * w[n][kg] (+ addsrc[m][n])), zeroed where mask <= 0.
// Tile: 128 output pixels x 64 output channels, 4 waves as 2 x 2, each 64 x 32 on 32x32x2 MFMAs.
__global__ __launch_bounds__(NT) void stem_fwd_kernel(FwdProblem p) {
  constexpr int BM = 128, BN = 64;
  __shared__ __attribute__((aligned(16))) float As[BM][LDK];
  __shared__ __attribute__((aligned(16))) float Bs[BN][LDK];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int j = lane & 31, g = lane >> 5;
  const int tiles_n = (p.N + BN - 1) / BN;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  {  // im2col rows: thread -> (row, half of the reduction axis)
    const int row = t & (BM - 1), kh = t >> 7;
    const int m = m0 + row;
    int img = 0, ho = 0, wo = 0;
    const bool live = m < p.M;
    if (live) {
      img = (int)p.div_howo.div((uint32_t)m);
      const int rem = m - img * p.Ho * p.Wo;
      ho = (int)p.div_wo.div((uint32_t)rem);
      wo = rem - ho * p.Wo;
    }
    float v[KS / 2];
#pragma unroll
    for (int i = 0; i < KS / 2; ++i)
      v[i] = col_elem(p.x, p.H, p.W, p.C, p.S, p.RSC, p.stride, p.pad, img, ho, wo, kh * (KS / 2) + i, live);
#pragma unroll
    for (int i = 0; i < KS / 2; i += 4)
      *reinterpret_cast<float4 *>(&As[row][kh * (KS / 2) + i]) = make_float4(v[i], v[i + 1], v[i + 2], v[i + 3]);
  }
  {  // filter rows: thread -> (n, quarter of the reduction axis)
    const int nl = t & (BN - 1), kq = t >> 6;
    const int n = n0 + nl;
#pragma unroll
    for (int k = kq * (KS / 4); k < (kq + 1) * (KS / 4); ++k)
      Bs[nl][k] = (n < p.N && k < p.RSC) ? p.w[(long long)n * p.RSC + k] : 0.f;
  }
  __syncthreads();

  floatx16 acc[2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[a][e] = 0.f;
#pragma unroll
  for (int ks = 0; ks < KS / 8; ++ks) {
    const float4 b4 = *reinterpret_cast<const float4 *>(&Bs[wn * 32 + j][ks * 8 + g * 4]);
    const float bv[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
    for (int a = 0; a < 2; ++a) {
      const float4 a4 = *reinterpret_cast<const float4 *>(&As[wm * 64 + a * 32 + j][ks * 8 + g * 4]);
      const float av[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) acc[a] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[kk], bv[kk], acc[a], 0, 0, 0);
    }
  }

  const int n = n0 + wn * 32 + j;
  if (n >= p.N) return;
  const float bias = p.bias ? p.bias[n] : 0.f;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int m = m0 + wm * 64 + a * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
      if (m >= p.M) continue;
      const long long o = (long long)m * p.N + n;
      float v = acc[a][e] + bias;
      if (p.addsrc) v += p.addsrc[o];
      if (p.relu) v = v > 0.f ? v : 0.f;
      if (p.mask) v = p.mask[o] > 0.f ? v : 0.f;
      p.out[o] = v;
    }
}

// part[z][pr][q] = sum over the rows m of split z of d[m][pr] * col[m][q]  (q < RSC <= 32), and
// part_b[z][pr] = sum of d[m][pr]: a 64 x 32 output tile per workgroup (blockIdx.y picks the 64
// output channels, blockIdx.z the split).  Steps of 32 rows: d rows and im2col rows staged in LDS,
// each wave takes 8 of them (4 MFMA k-pairs x 2 tiles); the four waves' tiles are added in a
// fixed order at the end.
template <bool VEC>
__global__ __launch_bounds__(NT) void stem_wgrad_kernel(WgradProblem p) {
  constexpr int BP = 64, BR = 32;  // output-channel tile, rows per step
  constexpr int LDP = BP + 4;
  __shared__ __attribute__((aligned(16))) float Ds[BR][LDP];
  __shared__ __attribute__((aligned(16))) float Xs[BR][LDK];
  __shared__ __attribute__((aligned(16))) float red[4][2][32][33];
  __shared__ float redb[16][BP];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int j = lane & 31, g = lane >> 5;
  const int p0 = blockIdx.y * BP, z = blockIdx.z;
  const int m_begin = z * p.m_per_split, m_end = min(p.M, m_begin + p.m_per_split);

  floatx16 acc[2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[a][e] = 0.f;
  // d staging: thread -> (row = t / 16 (+16), 4 consecutive output channels); its column sums feed the bias gradient
  const int drow = t >> 4, dc = (t & 15) * 4;
  float4 bsum = make_float4(0.f, 0.f, 0.f, 0.f);
  // im2col staging: thread -> (row = t % 32, 4 consecutive kg)
  const int xrow = t & 31, xk = (t >> 5) * 4;

  for (int mb = m_begin; mb < m_end; mb += BR) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int r = drow + 16 * i, m = mb + r;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (m < m_end) {
        const float *src = p.d + (long long)m * p.P + p0 + dc;
        if constexpr (VEC) {
          if (p0 + dc < p.P) v = *reinterpret_cast<const float4 *>(src);  // P % 4 == 0: whole group inside
        } else {
          if (p0 + dc + 0 < p.P) v.x = src[0];
          if (p0 + dc + 1 < p.P) v.y = src[1];
          if (p0 + dc + 2 < p.P) v.z = src[2];
          if (p0 + dc + 3 < p.P) v.w = src[3];
        }
      }
      *reinterpret_cast<float4 *>(&Ds[r][dc]) = v;
      bsum.x += v.x, bsum.y += v.y, bsum.z += v.z, bsum.w += v.w;
    }
    {
      const int m = mb + xrow;
      const bool live = m < m_end;
      const int mc = min(m, p.M - 1);
      const int img = (int)p.div_howo.div((uint32_t)mc);
      const int rem = mc - img * p.Ho * p.Wo;
      const int ho = (int)p.div_wo.div((uint32_t)rem);
      const int wo = rem - ho * p.Wo;
      float4 v;
      v.x = col_elem(p.x, p.H, p.W, p.C, p.S, p.RSC, p.stride, p.pad, img, ho, wo, xk + 0, live);
      v.y = col_elem(p.x, p.H, p.W, p.C, p.S, p.RSC, p.stride, p.pad, img, ho, wo, xk + 1, live);
      v.z = col_elem(p.x, p.H, p.W, p.C, p.S, p.RSC, p.stride, p.pad, img, ho, wo, xk + 2, live);
      v.w = col_elem(p.x, p.H, p.W, p.C, p.S, p.RSC, p.stride, p.pad, img, ho, wo, xk + 3, live);
      *reinterpret_cast<float4 *>(&Xs[xrow][xk]) = v;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = wave * 8 + 2 * i + g;
      const float xv = Xs[r][j];
#pragma unroll
      for (int a = 0; a < 2; ++a) acc[a] = __builtin_amdgcn_mfma_f32_32x32x2f32(Ds[r][a * 32 + j], xv, acc[a], 0, 0, 0);
    }
    __syncthreads();
  }

  // ---- the four waves' tiles, added in a fixed order: (w0 + w1) + (w2 + w3) ----
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int e = 0; e < 16; ++e) red[wave][a][8 * (e >> 2) + 4 * g + (e & 3)][j] = acc[a][e];
  *reinterpret_cast<float4 *>(&redb[drow][dc]) = bsum;
  __syncthreads();
  float *part = p.part + (long long)z * p.P * p.Qld;
  for (int i = t; i < BP * 32; i += NT) {
    const int pl = i >> 5, q = i & 31, a = pl >> 5, r = pl & 31;
    const int pr = p0 + pl;
    if (pr < p.P && q < p.Q) part[(long long)pr * p.Qld + q] = (red[0][a][r][q] + red[1][a][r][q]) + (red[2][a][r][q] + red[3][a][r][q]);
  }
  if (p.part_b && t < BP && p0 + t < p.P) {
    float s = 0.f;
    for (int r = 0; r < 16; ++r) s += redb[r][t];
    p.part_b[(long long)z * p.P + p0 + t] = s;
  }
}

}  // namespace

bool stem_fwd_applicable(const FwdProblem &p) {
  // one staging step, no projection columns, no split; layers the 16-byte fast path can serve keep it
  if (p.RSC > KS || p.Cs != 0 || p.ksplits > 1 || p.Kg != p.RSC) return false;
  if (p.C % 4 == 0) return false;
  const long long B = p.M / ((long long)p.Ho * p.Wo);
  return B * p.H * p.W * p.C < (1ll << 31) && (long long)p.M * p.N < (1ll << 40);
}

hipError_t launch_stem_fwd(const FwdProblem &p, hipStream_t st, const char **kernel) {
  const int tiles = ((p.M + 127) / 128) * ((p.N + 63) / 64);
  *kernel = "stem_fwd";
  hipLaunchKernelGGL(stem_fwd_kernel, dim3((unsigned)tiles), dim3(NT), 0, st, p);
  return hipGetLastError();
}

bool stem_wgrad_applicable(const WgradProblem &p) {
  if (p.RSC > KS || p.Cs != 0 || p.Q != p.RSC) return false;
  if (p.C % 4 == 0) return false;
  const long long B = p.M / ((long long)p.Ho * p.Wo);
  return B * p.H * p.W * p.C < (1ll << 31);
}

hipError_t launch_stem_wgrad(const WgradProblem &p, hipStream_t st, const char **kernel) {
  const dim3 grid(1, (unsigned)((p.P + 63) / 64), (unsigned)p.splits);
  *kernel = "stem_wgrad";
  if (p.P % 4 == 0)
    hipLaunchKernelGGL(stem_wgrad_kernel<true>, grid, dim3(NT), 0, st, p);
  else
    hipLaunchKernelGGL(stem_wgrad_kernel<false>, grid, dim3(NT), 0, st, p);
  return hipGetLastError();
}

}  // namespace nf
