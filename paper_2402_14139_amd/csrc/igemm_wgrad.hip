// Implicit-GEMM weight gradient on fp32 MFMA (v_mfma_f32_32x32x2_f32) for gfx950.
//
// Serves the gradient line of Algorithm 2 (NeuroFlux, arXiv 2402.14139) for the two
// convolutions of a local layer: theta_n (with its 1x1 projection shortcut) and beta_n.
//
// GEMM view: G[p][q] = sum_m D[m][p] * X[m][q];  m = (img,ho,wo) is the REDUCTION index,
// p = output channel of the convolution (D = dL/d(conv output), NHWC so p is contiguous),
// q = (r,s,c) (+ projection channels), X = im2col gather of the convolution's input.
// Both operands are contiguous along the non-reduced index, so LDS tiles are [m][p] and
// [m][q]; a lane reads PT (QT) consecutive p (q) of one m with a single ds_read and uses
// them as the operands of PT x QT MFMAs whose 32 rows (columns) are the strided sets
// {PT*r + t}.  The reduction over m is split across blockIdx.z; partial tiles go to a
// workspace and are summed in a fixed order by wgrad_reduce_kernel (deterministic).
// Column sums of D (the bias gradient) are accumulated by the q-tile-0 workgroups from
// the values they stage anyway.
#include "nf_internal.h"

namespace nf {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BKM = 32;  // reduction rows staged per step
constexpr int NTHREADS = 256;

template <int N>
struct VecLoad;
template <>
struct VecLoad<1> {
  static __device__ inline void ld(const float *s, float *v) { v[0] = s[0]; }
};
template <>
struct VecLoad<2> {
  static __device__ inline void ld(const float *s, float *v) {
    const float2 t = *reinterpret_cast<const float2 *>(s);
    v[0] = t.x, v[1] = t.y;
  }
};
template <>
struct VecLoad<4> {
  static __device__ inline void ld(const float *s, float *v) {
    const float4 t = *reinterpret_cast<const float4 *>(s);
    v[0] = t.x, v[1] = t.y, v[2] = t.z, v[3] = t.w;
  }
};

// BP x BQ output tile, WP x WQ waves, each wave (32*PT) x (32*QT).
template <int BP, int BQ, int WP, int WQ, int VEC>
__global__ __launch_bounds__(NTHREADS) void igemm_wgrad_kernel(WgradProblem p) {
  constexpr int TP = BP / WP, TQ = BQ / WQ;
  constexpr int PT = TP / 32, QT = TQ / 32;
  static_assert(WP * WQ == 4 && (PT == 1 || PT == 2 || PT == 4) && (QT == 1 || QT == 2 || QT == 4), "tile");
  constexpr int LDP = BP + 4, LDQ = BQ + 4;
  constexpr int CP = BP / 4, CQ = BQ / 4;             // 16-byte chunks per staged row
  constexpr int RP = NTHREADS / CP, RQ = NTHREADS / CQ;  // rows covered per pass
  constexpr int NP = BKM / RP, NQ = BKM / RQ;         // passes per step
  static_assert(NP >= 1 && NQ >= 1 && RP * NP == BKM && RQ * NQ == BKM, "staging");

  __shared__ __attribute__((aligned(16))) float Ds[2][BKM][LDP];
  __shared__ __attribute__((aligned(16))) float Xs[2][BKM][LDQ];

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wp = wave / WQ, wq = wave % WQ;
  const int j = lane & 31, h = lane >> 5;
  const int p0 = blockIdx.y * BP, q0 = blockIdx.x * BQ;
  const int m_begin = blockIdx.z * p.m_per_split;
  const int m_end = min(p.M, m_begin + p.m_per_split);

  // D staging: this thread always loads columns p0 + chp*4 .. +3
  const int chp = t % CP, rowp = t / CP;
  const int pcol = p0 + chp * 4;
  // X staging: this thread always loads columns q0 + chq*4 .. +3, i.e. fixed (r,s,c)
  const int chq = t % CQ, rowq = t / CQ;
  const int qcol = q0 + chq * 4;
  int qr[4], qs[4], qc[4], qkind[4];  // VEC==4 uses entry 0 only
#pragma unroll
  for (int e = 0; e < (VEC == 4 ? 1 : 4); ++e) {
    const int q = qcol + e;
    qkind[e] = q < p.RSC ? 0 : (q < p.Q ? 1 : 2);
    qr[e] = qs[e] = qc[e] = 0;
    if (qkind[e] == 0) {
      const int tap = q / p.C;
      qc[e] = q - tap * p.C;
      qr[e] = tap / p.S;
      qs[e] = tap - qr[e] * p.S;
    } else {
      qc[e] = q - p.RSC;
    }
  }

  float4 rd[NP], rx[NQ];
  float4 bsum = make_float4(0.f, 0.f, 0.f, 0.f);
  const bool do_bias = (blockIdx.x == 0) && (p.part_b != nullptr);

  auto gload = [&](int mb) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      const int m = mb + rowp + RP * i;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (m < m_end) {
        const float *src = p.d + (long long)m * p.P + pcol;
        if constexpr (VEC == 4) {
          if (pcol < p.P) v = *reinterpret_cast<const float4 *>(src);
        } else {
          if (pcol + 0 < p.P) v.x = src[0];
          if (pcol + 1 < p.P) v.y = src[1];
          if (pcol + 2 < p.P) v.z = src[2];
          if (pcol + 3 < p.P) v.w = src[3];
        }
      }
      rd[i] = v;
    }
#pragma unroll
    for (int i = 0; i < NQ; ++i) {
      const int m = mb + rowq + RQ * i;
      float v[4] = {0.f, 0.f, 0.f, 0.f};
      if (m < m_end) {
        const int img = (int)p.div_howo.div((uint32_t)m);
        const int rem = m - img * p.Ho * p.Wo;
        const int ho = (int)p.div_wo.div((uint32_t)rem);
        const int wo = rem - ho * p.Wo;
        if constexpr (VEC == 4) {
          if (qkind[0] == 0) {
            const int hi = ho * p.stride - p.pad + qr[0], wi = wo * p.stride - p.pad + qs[0];
            if ((unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W)
              VecLoad<4>::ld(p.x + ((long long)((img * p.H + hi) * p.W + wi) * p.C + qc[0]), v);
          } else if (qkind[0] == 1) {
            VecLoad<4>::ld(p.xs + ((long long)((img * p.Hs + ho * p.ss) * p.Ws + wo * p.ss) * p.Cs + qc[0]), v);
          }
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (qkind[e] == 0) {
              const int hi = ho * p.stride - p.pad + qr[e], wi = wo * p.stride - p.pad + qs[e];
              if ((unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W)
                v[e] = p.x[(long long)((img * p.H + hi) * p.W + wi) * p.C + qc[e]];
            } else if (qkind[e] == 1) {
              v[e] = p.xs[(long long)((img * p.Hs + ho * p.ss) * p.Ws + wo * p.ss) * p.Cs + qc[e]];
            }
          }
        }
      }
      rx[i] = make_float4(v[0], v[1], v[2], v[3]);
    }
  };

  auto lstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < NP; ++i) {
      *reinterpret_cast<float4 *>(&Ds[buf][rowp + RP * i][chp * 4]) = rd[i];
      if (do_bias) {
        bsum.x += rd[i].x, bsum.y += rd[i].y, bsum.z += rd[i].z, bsum.w += rd[i].w;
      }
    }
#pragma unroll
    for (int i = 0; i < NQ; ++i) *reinterpret_cast<float4 *>(&Xs[buf][rowq + RQ * i][chq * 4]) = rx[i];
  };

  floatx16 acc[PT][QT];
#pragma unroll
  for (int a = 0; a < PT; ++a)
#pragma unroll
    for (int b = 0; b < QT; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  const int nsteps = (m_end - m_begin + BKM - 1) / BKM;
  if (nsteps > 0) {
    gload(m_begin);
    lstore(0);
  }
  __syncthreads();
  for (int sidx = 0; sidx < nsteps; ++sidx) {
    const int cur = sidx & 1;
    const bool more = sidx + 1 < nsteps;
    if (more) gload(m_begin + (sidx + 1) * BKM);
#pragma unroll
    for (int kk = 0; kk < BKM / 2; ++kk) {
      float av[PT], bv[QT];
      VecLoad<PT>::ld(&Ds[cur][2 * kk + h][wp * TP + PT * j], av);
      VecLoad<QT>::ld(&Xs[cur][2 * kk + h][wq * TQ + QT * j], bv);
#pragma unroll
      for (int a = 0; a < PT; ++a)
#pragma unroll
        for (int b = 0; b < QT; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[a], bv[b], acc[a][b], 0, 0, 0);
    }
    if (more) lstore(cur ^ 1);
    __syncthreads();
  }

  // ---- store the partial tile: lane holds, per (a, e), QT consecutive q ----
  float *part = p.part + (long long)blockIdx.z * p.P * p.Qld;
#pragma unroll
  for (int a = 0; a < PT; ++a) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int r = 8 * (e >> 2) + 4 * h + (e & 3);
      const int pr = p0 + wp * TP + PT * r + a;
      if (pr >= p.P) continue;
#pragma unroll
      for (int b = 0; b < QT; ++b) {
        const int q = q0 + wq * TQ + QT * j + b;
        if (q < p.Q) part[(long long)pr * p.Qld + q] = acc[a][b][e];
      }
    }
  }

  // ---- bias-gradient partials: sum the per-thread column sums over the RP staging rows ----
  if (do_bias) {  // uniform per workgroup
    __syncthreads();
    float *red = &Ds[0][0][0];  // reuse: [RP][BP]
    *reinterpret_cast<float4 *>(&red[rowp * BP + chp * 4]) = bsum;
    __syncthreads();
    if (t < BP && p0 + t < p.P) {
      float s = 0.f;
      for (int r = 0; r < RP; ++r) s += red[r * BP + t];
      p.part_b[(long long)blockIdx.z * p.P + p0 + t] = s;
    }
  }
}

__global__ void wgrad_reduce_kernel(const float *__restrict__ part, const float *__restrict__ part_b, int splits,
                                    int P, int Q, int Qld, int Q0, float *__restrict__ out0,
                                    float *__restrict__ out1, float *__restrict__ ob) {
  const long long total = (long long)P * Q;
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < total) {
    const int pr = (int)(i / Q), q = (int)(i - (long long)pr * Q);
    const float *src = part + (long long)pr * Qld + q;
    float s = 0.f;
    for (int z = 0; z < splits; ++z) s += src[(long long)z * P * Qld];
    if (q < Q0)
      out0[(long long)pr * Q0 + q] = s;
    else
      out1[(long long)pr * (Q - Q0) + (q - Q0)] = s;
  } else if (ob && i < total + P) {
    const int pr = (int)(i - total);
    float s = 0.f;
    for (int z = 0; z < splits; ++z) s += part_b[(long long)z * P + pr];
    ob[pr] = s;
  }
}

struct TileChoice {
  int BP, BQ;
};
inline TileChoice pick_tile(int P) {
  if (P > 64) return {128, 128};
  if (P > 32) return {64, 128};
  return {32, 256};
}

template <int BP, int BQ, int WP, int WQ>
hipError_t launch_cfg(const WgradProblem &p, bool vec, hipStream_t st) {
  dim3 grid((p.Q + BQ - 1) / BQ, (p.P + BP - 1) / BP, p.splits);
  if (vec)
    hipLaunchKernelGGL((igemm_wgrad_kernel<BP, BQ, WP, WQ, 4>), grid, dim3(NTHREADS), 0, st, p);
  else
    hipLaunchKernelGGL((igemm_wgrad_kernel<BP, BQ, WP, WQ, 1>), grid, dim3(NTHREADS), 0, st, p);
  return hipGetLastError();
}

}  // namespace

int wgrad_pick_splits(int P, int Q, int M) {
  const TileChoice tc = pick_tile(P);
  const long long tiles = (long long)((P + tc.BP - 1) / tc.BP) * ((Q + tc.BQ - 1) / tc.BQ);
  // aim at ~4 workgroups per compute unit (256 CUs), keep at least 4 staging steps per split
  long long want = (1024 + tiles - 1) / tiles;
  const long long max_by_m = (M + 4 * BKM - 1) / (4 * BKM);
  if (want > max_by_m) want = max_by_m;
  if (want < 1) want = 1;
  if (want > 512) want = 512;
  return (int)want;
}

hipError_t launch_igemm_wgrad(const WgradProblem &p, hipStream_t st, const char **kernel) {
  const bool vec = (p.C % 4 == 0) && (p.Cs % 4 == 0) && (p.P % 4 == 0);
  if (p.P > 64) {
    *kernel = vec ? "igemm_wgrad_128x128_v4" : "igemm_wgrad_128x128_v1";
    return launch_cfg<128, 128, 2, 2>(p, vec, st);
  }
  if (p.P > 32) {
    *kernel = vec ? "igemm_wgrad_64x128_v4" : "igemm_wgrad_64x128_v1";
    return launch_cfg<64, 128, 2, 2>(p, vec, st);
  }
  *kernel = vec ? "igemm_wgrad_32x256_v4" : "igemm_wgrad_32x256_v1";
  return launch_cfg<32, 256, 1, 4>(p, vec, st);
}

hipError_t launch_wgrad_reduce(const float *part, const float *part_b, int splits, int P, int Q, int Qld,
                               int Q0, float *out0, float *out1, float *ob, hipStream_t st) {
  const long long total = (long long)P * Q + (ob ? P : 0);
  const int threads = 256;
  const long long blocks = (total + threads - 1) / threads;
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)blocks), dim3(threads), 0, st, part, part_b, splits, P, Q,
                     Qld, Q0, out0, out1, ob);
  return hipGetLastError();
}

}  // namespace nf
