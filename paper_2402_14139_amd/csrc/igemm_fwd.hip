// Implicit-GEMM convolution on fp32 MFMA (v_mfma_f32_32x32x2_f32) for gfx950.
//
// Serves three steps of the local training step (NeuroFlux, arXiv 2402.14139):
//   - the layer's convolution theta_n of Eq. 1, with bias, shortcut and ReLU fused,
//   - the auxiliary convolution beta_n of Eq. 2 (bias + ReLU fused),
//   - the data gradient of beta_n w.r.t. the emitted activation (a convolution of dU with
//     the flipped, transposed filter), with the layer's ReLU mask fused.
//
// GEMM view: out[m][n] = sum_kg A[m][kg] * Bw[n][kg];  m = (img,ho,wo), n = output channel,
// kg = (r,s,c) with c fastest (NHWC activations, KRSC weights), so both operands are
// contiguous along kg.  A workgroup of 4 wavefronts owns a BM x BN tile; per step of
// BK = 32 it stages the im2col gather of A and the rows of Bw in LDS ([row][BK+4] floats,
// the +4 keeps 16-byte row reads of 16 consecutive lanes on distinct banks), each lane
// reads four consecutive kg of its row with one ds_read_b128 and feeds four MFMAs.
// Global loads for step kb+1 are issued before the MFMAs of step kb (register prefetch,
// two LDS buffers, one barrier per step).
#include "nf_internal.h"

namespace nf {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 32;
constexpr int LDK = BK + 4;
constexpr int NTHREADS = 256;

template <int BM, int BN, int WM, int WN, int VEC>
__global__ __launch_bounds__(NTHREADS) void igemm_fwd_kernel(FwdProblem p) {
  constexpr int TM = BM / WM, TN = BN / WN;   // wave tile
  constexpr int MT = TM / 32, NT = TN / 32;   // 32x32 MFMA tiles per wave
  constexpr int PA = BM / 32, PB = BN / 32;   // 16-byte chunks per thread per step
  static_assert(WM * WN == 4 && MT >= 1 && NT >= 1, "4 waves per workgroup");

  __shared__ __attribute__((aligned(16))) float As[2][BM][LDK];
  __shared__ __attribute__((aligned(16))) float Bs[2][BN][LDK];

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int j = lane & 31, h = lane >> 5;

  // tile rasterisation: consecutive workgroups walk N first (they share the A rows)
  const int tiles_n = (p.N + BN - 1) / BN;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  // ---- per-thread gather state: this thread always loads chunk `ch` of rows row0+32*i ----
  const int ch = t & 7, row0 = t >> 3;
  int pix[PA], hi0[PA], wi0[PA], spix[PA];
#pragma unroll
  for (int i = 0; i < PA; ++i) {
    const int m = m0 + row0 + 32 * i;
    if (m < p.M) {
      const int img = (int)p.div_howo.div((uint32_t)m);
      const int rem = m - img * p.Ho * p.Wo;
      const int ho = (int)p.div_wo.div((uint32_t)rem);
      const int wo = rem - ho * p.Wo;
      pix[i] = img * p.H * p.W;
      hi0[i] = ho * p.stride - p.pad;
      wi0[i] = wo * p.stride - p.pad;
      spix[i] = p.Cs ? (img * p.Hs + ho * p.ss) * p.Ws + wo * p.ss : 0;
    } else {
      pix[i] = 0;
      hi0[i] = -(1 << 20);  // every tap out of range -> zeros
      wi0[i] = -(1 << 20);
      spix[i] = -1;
    }
  }

  float4 ra[PA], rb[PB];
  const int nkb = (p.Kg + BK - 1) / BK;

  auto gload = [&](int kb) {
    const int kg = kb * BK + ch * 4;
    if constexpr (VEC == 4) {
      // one (tap, channel) decode per thread per step; a 16-byte chunk never straddles a tap
      int r = 0, s = 0, c = 0;
      const bool in_conv = kg < p.RSC, in_proj = !in_conv && kg < p.Kg;
      if (in_conv) {
        const int tap = kg / p.C;
        c = kg - tap * p.C;
        r = tap / p.S;
        s = tap - r * p.S;
      } else {
        c = kg - p.RSC;
      }
#pragma unroll
      for (int i = 0; i < PA; ++i) {
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (in_conv) {
          const int hi = hi0[i] + r, wi = wi0[i] + s;
          if ((unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W)
            v = *reinterpret_cast<const float4 *>(p.x + ((long long)(pix[i] + hi * p.W + wi) * p.C + c));
        } else if (in_proj && spix[i] >= 0) {
          v = *reinterpret_cast<const float4 *>(p.xs + ((long long)spix[i] * p.Cs + c));
        }
        ra[i] = v;
      }
#pragma unroll
      for (int i = 0; i < PB; ++i) {
        const int n = n0 + row0 + 32 * i;
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (n < p.N) {
          if (in_conv)
            v = *reinterpret_cast<const float4 *>(p.w + ((long long)n * p.RSC + kg));
          else if (in_proj)
            v = *reinterpret_cast<const float4 *>(p.wp + ((long long)n * p.Cs + c));
        }
        rb[i] = v;
      }
    } else {
      // scalar gather (channel counts that are not multiples of 4, e.g. RGB stems)
      int r[4], s[4], c[4], kind[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int k = kg + e;
        kind[e] = k < p.RSC ? 0 : (k < p.Kg ? 1 : 2);
        r[e] = s[e] = 0;
        if (kind[e] == 0) {
          const int tap = k / p.C;
          c[e] = k - tap * p.C;
          r[e] = tap / p.S;
          s[e] = tap - r[e] * p.S;
        } else {
          c[e] = k - p.RSC;
        }
      }
#pragma unroll
      for (int i = 0; i < PA; ++i) {
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = 0.f;
          if (kind[e] == 0) {
            const int hi = hi0[i] + r[e], wi = wi0[i] + s[e];
            if ((unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W)
              v[e] = p.x[(long long)(pix[i] + hi * p.W + wi) * p.C + c[e]];
          } else if (kind[e] == 1 && spix[i] >= 0) {
            v[e] = p.xs[(long long)spix[i] * p.Cs + c[e]];
          }
        }
        ra[i] = make_float4(v[0], v[1], v[2], v[3]);
      }
#pragma unroll
      for (int i = 0; i < PB; ++i) {
        const int n = n0 + row0 + 32 * i;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = 0.f;
          if (n < p.N) {
            if (kind[e] == 0)
              v[e] = p.w[(long long)n * p.RSC + kg + e];
            else if (kind[e] == 1)
              v[e] = p.wp[(long long)n * p.Cs + c[e]];
          }
        }
        rb[i] = make_float4(v[0], v[1], v[2], v[3]);
      }
    }
  };

  auto lstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < PA; ++i) *reinterpret_cast<float4 *>(&As[buf][row0 + 32 * i][ch * 4]) = ra[i];
#pragma unroll
    for (int i = 0; i < PB; ++i) *reinterpret_cast<float4 *>(&Bs[buf][row0 + 32 * i][ch * 4]) = rb[i];
  };

  floatx16 acc[MT][NT];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < NT; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  gload(0);
  lstore(0);
  __syncthreads();

  for (int kb = 0; kb < nkb; ++kb) {
    const int cur = kb & 1;
    const bool more = kb + 1 < nkb;
    if (more) gload(kb + 1);
#pragma unroll
    for (int ks = 0; ks < BK / 8; ++ks) {
      float4 af[MT], bf[NT];
#pragma unroll
      for (int a = 0; a < MT; ++a)
        af[a] = *reinterpret_cast<const float4 *>(&As[cur][wm * TM + a * 32 + j][ks * 8 + h * 4]);
#pragma unroll
      for (int b = 0; b < NT; ++b)
        bf[b] = *reinterpret_cast<const float4 *>(&Bs[cur][wn * TN + b * 32 + j][ks * 8 + h * 4]);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
        for (int a = 0; a < MT; ++a)
#pragma unroll
          for (int b = 0; b < NT; ++b) {
            const float av = kk == 0 ? af[a].x : kk == 1 ? af[a].y : kk == 2 ? af[a].z : af[a].w;
            const float bv = kk == 0 ? bf[b].x : kk == 1 ? bf[b].y : kk == 2 ? bf[b].z : bf[b].w;
            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[a][b], 0, 0, 0);
          }
      }
    }
    if (more) lstore(cur ^ 1);
    __syncthreads();
  }

  // ---- epilogue: bias, identity shortcut, ReLU, mask; lanes 0..31 store 32 consecutive n ----
#pragma unroll
  for (int b = 0; b < NT; ++b) {
    const int n = n0 + wn * TN + b * 32 + j;
    if (n >= p.N) continue;
    const float bias = p.bias ? p.bias[n] : 0.f;
#pragma unroll
    for (int a = 0; a < MT; ++a) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm * TM + a * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
        if (m >= p.M) continue;
        const long long o = (long long)m * p.N + n;
        float v = acc[a][b][e] + bias;
        if (p.addsrc) v += p.addsrc[o];
        if (p.relu) v = v > 0.f ? v : 0.f;
        if (p.mask) v = p.mask[o] > 0.f ? v : 0.f;
        p.out[o] = v;
      }
    }
  }
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_cfg(const FwdProblem &p, bool vec, hipStream_t st) {
  const int tiles = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
  if (vec)
    hipLaunchKernelGGL((igemm_fwd_kernel<BM, BN, WM, WN, 4>), dim3(tiles), dim3(NTHREADS), 0, st, p);
  else
    hipLaunchKernelGGL((igemm_fwd_kernel<BM, BN, WM, WN, 1>), dim3(tiles), dim3(NTHREADS), 0, st, p);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_igemm_fwd(const FwdProblem &p, hipStream_t st, const char **kernel) {
  if (igemm_fwd_fast_applicable(p)) return launch_igemm_fwd_fast(p, st, kernel);
  if (stem_fwd_applicable(p)) return launch_stem_fwd(p, st, kernel);
  const bool vec = (p.C % 4 == 0) && (p.Cs % 4 == 0);
  if (p.N > 64) {
    *kernel = vec ? "igemm_fwd_128x128_v4" : "igemm_fwd_128x128_v1";
    return launch_cfg<128, 128, 2, 2>(p, vec, st);
  }
  if (p.N > 32) {
    *kernel = vec ? "igemm_fwd_128x64_v4" : "igemm_fwd_128x64_v1";
    return launch_cfg<128, 64, 2, 2>(p, vec, st);
  }
  *kernel = vec ? "igemm_fwd_128x32_v4" : "igemm_fwd_128x32_v1";
  return launch_cfg<128, 32, 4, 1>(p, vec, st);
}

}  // namespace nf
