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
#include "head_gamma.h"
#include "nf_internal.h"

namespace nf {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BKM = 32;  // reduction rows staged per step
constexpr int NTHREADS = 256;
constexpr int OOB = (int)0x80000000;    // offset no buffer of < 2 GiB contains
constexpr int RSRC_FLAGS = 0x00020000;  // raw buffer, 32-bit data format
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ inline float4 bload(__amdgpu_buffer_rsrc_t r, int voff) {
  const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, 0, 0));
  return make_float4(v.x, v.y, v.z, v.w);
}

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
// BUF (needs VEC == 4 and operands < 2 GiB): global reads are raw buffer loads and every
// "no data here" case (row past the split, tap outside the image, column past P or Q) is an
// out-of-range offset that the hardware answers with zeros -- no branches in the gather.
template <int BP, int BQ, int WP, int WQ, int VEC, bool BUF>
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

  const __amdgpu_buffer_rsrc_t rsd = __builtin_amdgcn_make_buffer_rsrc((void *)p.d, 0, p.d_bytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rsx = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, p.x_bytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rsxs = __builtin_amdgcn_make_buffer_rsrc((void *)p.xs, 0, p.xs_bytes, RSRC_FLAGS);
  const int dcol_off = pcol < p.P ? pcol * 4 : OOB;  // byte offset of this thread's D columns
  const int xtap_off = ((qr[0] * p.W + qs[0]) * p.C + qc[0]) * 4;

  auto gload = [&](int mb) {
    if constexpr (BUF) {
#pragma unroll
      for (int i = 0; i < NP; ++i) {
        const int m = mb + rowp + RP * i;
        const bool ok = m < m_end && dcol_off != OOB;
        rd[i] = bload(rsd, ok ? m * p.P * 4 + dcol_off : OOB);
      }
#pragma unroll
      for (int i = 0; i < NQ; ++i) {
        const int m = mb + rowq + RQ * i;
        const int img = (int)p.div_howo.div((uint32_t)m);
        const int rem = m - img * p.Ho * p.Wo;
        const int ho = (int)p.div_wo.div((uint32_t)rem);
        const int wo = rem - ho * p.Wo;
        if (qkind[0] == 0) {  // fixed per thread
          const int hi0 = ho * p.stride - p.pad, wi0 = wo * p.stride - p.pad;
          const bool ok = m < m_end && (unsigned)(hi0 + qr[0]) < (unsigned)p.H && (unsigned)(wi0 + qs[0]) < (unsigned)p.W;
          rx[i] = bload(rsx, ok ? ((img * p.H + hi0) * p.W + wi0) * p.C * 4 + xtap_off : OOB);
        } else {
          const bool ok = m < m_end && qkind[0] == 1;
          rx[i] = bload(rsxs, ok ? (((img * p.Hs + ho * p.ss) * p.Ws + wo * p.ss) * p.Cs + qc[0]) * 4 : OOB);
        }
      }
      return;
    }
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

// Sum of the split partials in a fixed order, for up to two weight gradients in one launch,
// optionally followed in place by the update line of Algorithm 2 (momentum SGD) for the tensors
// just reduced and for up to two more whose gradient is already final.
// Per gradient: a workgroup owns 256/ZS groups of four consecutive elements of the flattened
// [P][Qld] tile array; its ZS thread rows each add every ZS-th split with 16-byte loads, then the
// ZS row sums are added in order through LDS.  Further workgroups do the same for the bias
// partials (16 columns x 16 thread rows each).
__device__ inline void sgd_elem(float g, float *w, float *v, long long i, float lr, float mu) {
  if (!w) return;
  if (v && mu != 0.f) {
    g = mu * v[i] + g;
    v[i] = g;
  }
  w[i] -= lr * g;
}

__global__ __launch_bounds__(256) void wgrad_reduce_kernel(ReduceSgd r) {
  __shared__ float4 red[256];
  const int t = threadIdx.x;
  int b = blockIdx.x;
#pragma unroll
  for (int ji = 0; ji < 2; ++ji) {
    if (ji >= r.njobs) break;
    const WgradReduce &jb = r.job[ji];
    if (b < jb.main_blocks && jb.direct) {
      // up to eight splits, 16-byte aligned tensors: one thread per group of four, every load
      // (partials, weight, momentum) issued before the first add, no LDS; partials are added in
      // split order
      const long long n4 = ((long long)jb.P * jb.Qld) >> 2;
      const long long i4 = (long long)b * 256 + t;
      if (i4 >= n4) return;
      const float4 *src = reinterpret_cast<const float4 *>(jb.part) + i4;
      const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
      constexpr int DMAX = 8;  // the launcher takes this path for at most DMAX splits
      float4 a[DMAX];
#pragma unroll
      for (int z = 0; z < DMAX; ++z) a[z] = z < jb.splits ? src[(long long)z * n4] : zero;
      const long long e = i4 << 2;
      const int pr = (int)(e / jb.Qld), q = (int)(e - (long long)pr * jb.Qld);
      const bool first = q < jb.Q0;
      const long long o = first ? (long long)pr * jb.Q0 + q : (long long)pr * (jb.Q - jb.Q0) + (q - jb.Q0);
      float *out = first ? jb.out0 : jb.out1, *w = first ? jb.w0 : jb.w1, *v = first ? jb.v0 : jb.v1;
      const bool mom = v && r.mu != 0.f;
      const float4 vv = (w && mom) ? *reinterpret_cast<const float4 *>(v + o) : zero;
      float4 wv = w ? *reinterpret_cast<const float4 *>(w + o) : zero;
      float4 g = a[0];
#pragma unroll
      for (int z = 1; z < DMAX; ++z)
        if (z < jb.splits) g.x += a[z].x, g.y += a[z].y, g.z += a[z].z, g.w += a[z].w;
      *reinterpret_cast<float4 *>(out + o) = g;
      if (w) {
        if (mom) {
          g.x = r.mu * vv.x + g.x, g.y = r.mu * vv.y + g.y, g.z = r.mu * vv.z + g.z, g.w = r.mu * vv.w + g.w;
          *reinterpret_cast<float4 *>(v + o) = g;
        }
        wv.x -= r.lr * g.x, wv.y -= r.lr * g.y, wv.z -= r.lr * g.z, wv.w -= r.lr * g.w;
        *reinterpret_cast<float4 *>(w + o) = wv;
      }
      return;
    }
    if (b < jb.main_blocks) {
      const int ZS = jb.ZS, cols = 256 / ZS;
      const int col = t % cols, zs = t / cols;
      const long long n4 = ((long long)jb.P * jb.Qld) >> 2;  // Qld is a multiple of 4
      const long long i4 = (long long)b * cols + col;
      float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i4 < n4) {
        const float4 *src = reinterpret_cast<const float4 *>(jb.part) + i4;
        for (int z = zs; z < jb.splits; z += ZS) {
          const float4 v = src[(long long)z * n4];
          s.x += v.x, s.y += v.y, s.z += v.z, s.w += v.w;
        }
      }
      red[t] = s;
      __syncthreads();
      if (zs == 0 && i4 < n4) {
        for (int k = 1; k < ZS; ++k) {
          const float4 v = red[k * cols + col];
          s.x += v.x, s.y += v.y, s.z += v.z, s.w += v.w;
        }
        const long long e = i4 << 2;
        const int pr = (int)(e / jb.Qld), q = (int)(e - (long long)pr * jb.Qld);
        if (jb.vec4) {  // no group of four straddles a row end or the out0/out1 boundary
          const bool first = q < jb.Q0;
          const long long o = first ? (long long)pr * jb.Q0 + q : (long long)pr * (jb.Q - jb.Q0) + (q - jb.Q0);
          float *out = first ? jb.out0 : jb.out1, *w = first ? jb.w0 : jb.w1, *v = first ? jb.v0 : jb.v1;
          *reinterpret_cast<float4 *>(out + o) = s;
          if (w) {
            float4 g = s;
            if (v && r.mu != 0.f) {
              const float4 vv = *reinterpret_cast<const float4 *>(v + o);
              g.x = r.mu * vv.x + g.x, g.y = r.mu * vv.y + g.y, g.z = r.mu * vv.z + g.z, g.w = r.mu * vv.w + g.w;
              *reinterpret_cast<float4 *>(v + o) = g;
            }
            float4 wv = *reinterpret_cast<const float4 *>(w + o);
            wv.x -= r.lr * g.x, wv.y -= r.lr * g.y, wv.z -= r.lr * g.z, wv.w -= r.lr * g.w;
            *reinterpret_cast<float4 *>(w + o) = wv;
          }
          return;
        }
        const float vals[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int qq = q + k;
          if (qq < jb.Q0) {
            const long long o = (long long)pr * jb.Q0 + qq;
            jb.out0[o] = vals[k];
            sgd_elem(vals[k], jb.w0, jb.v0, o, r.lr, r.mu);
          } else if (qq < jb.Q) {
            const long long o = (long long)pr * (jb.Q - jb.Q0) + (qq - jb.Q0);
            jb.out1[o] = vals[k];
            sgd_elem(vals[k], jb.w1, jb.v1, o, r.lr, r.mu);
          }
        }
      }
      return;
    }
    b -= jb.main_blocks;
    if (b < jb.bias_blocks) {
      const int pr = b * 16 + (t & 15), zb = t >> 4;
      float sb = 0.f;
      if (pr < jb.P)
        for (int z = zb; z < jb.splits; z += 16) sb += jb.part_b[(long long)z * jb.P + pr];
      float *redb = reinterpret_cast<float *>(red);
      redb[t] = sb;
      __syncthreads();
      if (zb == 0 && pr < jb.P) {
        for (int k = 1; k < 16; ++k) sb += redb[k * 16 + (t & 15)];
        jb.ob[pr] = sb;
        sgd_elem(sb, jb.wb, jb.vb, pr, r.lr, r.mu);
      }
      return;
    }
    b -= jb.bias_blocks;
  }
#pragma unroll
  for (int xi = 0; xi < 2; ++xi) {
    if (xi >= r.nx) break;
    if (b < r.xblocks[xi]) {
      const long long i = (long long)b * 256 + t;
      if (i < r.xn[xi]) sgd_elem(r.xg[xi][i], r.xw[xi], r.xv[xi], i, r.lr, r.mu);
      return;
    }
    b -= r.xblocks[xi];
  }
  // the linear layer's gradient (+ update) and the batch-mean loss, when this launch carries them
  if (r.gamma.dWf) {
    float *redf = reinterpret_cast<float *>(red);
    if (b < r.gamma.nb_w) {
      gamma_block(r.gamma, b, redf, redf + 256);
      return;
    }
    b -= r.gamma.nb_w;
    if (b < r.gamma.nb_l) loss_mean_block(r.gamma.loss_n, r.gamma.B, r.gamma.loss_out, redf);
  }
}

struct TileChoice {
  int BP, BQ;
};
inline TileChoice pick_tile(int P) {
  if (P > 64) return {128, 128};
  if (P > 32) return {64, 64};
  return {32, 128};
}

template <int BP, int BQ, int WP, int WQ>
hipError_t launch_cfg(const WgradProblem &p0, bool vec, hipStream_t st) {
  WgradProblem p = p0;
  dim3 grid((p.Q + BQ - 1) / BQ, (p.P + BP - 1) / BP, p.splits);
  const long long lim = 0x7FFFFFF0ll, B = p.M / ((long long)p.Ho * p.Wo);
  const long long db = (long long)p.M * p.P * 4, xb = B * p.H * p.W * p.C * 4, xsb = p.Cs ? B * p.Hs * p.Ws * p.Cs * 4 : 0;
  if (vec && db <= lim && xb <= lim && xsb <= lim) {
    p.d_bytes = (uint32_t)db, p.x_bytes = (uint32_t)xb, p.xs_bytes = (uint32_t)xsb;
    hipLaunchKernelGGL((igemm_wgrad_kernel<BP, BQ, WP, WQ, 4, true>), grid, dim3(NTHREADS), 0, st, p);
  } else if (vec) {
    hipLaunchKernelGGL((igemm_wgrad_kernel<BP, BQ, WP, WQ, 4, false>), grid, dim3(NTHREADS), 0, st, p);
  } else {
    hipLaunchKernelGGL((igemm_wgrad_kernel<BP, BQ, WP, WQ, 1, false>), grid, dim3(NTHREADS), 0, st, p);
  }
  return hipGetLastError();
}

}  // namespace

int wgrad_pick_splits(int P, int Q, int M) {
  const TileChoice tc = pick_tile(P);
  const long long tp = (P + tc.BP - 1) / tc.BP, tq = (Q + tc.BQ - 1) / tc.BQ, tiles = tp * tq;
  // Cost model in microseconds, minimised over the split count S (at least 4 staging steps per
  // split).  Two workgroups fit on a compute unit (LDS) and run best as a pair (measured: one
  // per CU is ~1.6x slower), the chip has 256 CUs: workgroups execute in rounds of 512, and a
  // partly filled round costs as much as a full one.  MFMA time = padded work at ~100 TFLOP/s
  // times rounds*512/workgroups.  Every workgroup writes its tile once and the reduction reads
  // it back: 8 bytes per partial element at ~3 TB/s.
  const double work_us = 2.0 * M * (double)(tp * tc.BP) * (double)(tq * tc.BQ) / 100e12 * 1e6;
  const long long max_by_m = (M + 4 * BKM - 1) / (4 * BKM);
  long long best = 1;
  double best_cost = 1e30;
  for (long long S = 1; S <= max_by_m && S <= 512; ++S) {
    const long long wgs = tiles * S, rounds = (wgs + 511) / 512;
    const double cost = work_us * (double)(rounds * 512) / (double)wgs + 8.0 * (double)S * P * Q / 3e12 * 1e6;
    if (cost < best_cost) best_cost = cost, best = S;
  }
  return (int)best;
}

hipError_t launch_igemm_wgrad(const WgradProblem &p, hipStream_t st, const char **kernel) {
  if (igemm_wgrad_small_applicable(p)) return launch_igemm_wgrad_small(p, st, kernel);
  if (igemm_wgrad_fast_applicable(p)) return launch_igemm_wgrad_fast(p, st, kernel);
  if (stem_wgrad_applicable(p)) return launch_stem_wgrad(p, st, kernel);
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

hipError_t launch_wgrad_reduce_sgd(const ReduceSgd &r0, hipStream_t st) {
  ReduceSgd r = r0;
  unsigned blocks = 0;
  for (int j = 0; j < r.njobs; ++j) {
    WgradReduce &jb = r.job[j];
    int ZS = 1;
    while (ZS < 16 && ZS < jb.splits) ZS *= 2;
    const int cols = 256 / ZS;
    const long long n4 = ((long long)jb.P * jb.Qld) / 4;
    jb.ZS = ZS;
    auto al16 = [](const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
    jb.vec4 = (jb.Q0 % 4 == 0 && jb.Q % 4 == 0 && jb.Qld == jb.Q && al16(jb.out0) && al16(jb.out1) && al16(jb.w0) &&
               al16(jb.w1) && al16(jb.v0) && al16(jb.v1))
                  ? 1
                  : 0;
    jb.direct = (jb.vec4 && jb.splits <= 8) ? 1 : 0;
    jb.main_blocks = jb.direct ? (int)((n4 + 255) / 256) : (int)((n4 + cols - 1) / cols);
    jb.bias_blocks = jb.ob ? (jb.P + 15) / 16 : 0;
    blocks += (unsigned)(jb.main_blocks + jb.bias_blocks);
  }
  for (int x = 0; x < r.nx; ++x) {
    r.xblocks[x] = (int)((r.xn[x] + 255) / 256);
    blocks += (unsigned)r.xblocks[x];
  }
  if (r.gamma.dWf) blocks += (unsigned)gamma_job_plan(r.gamma);
  if (!blocks) return hipSuccess;
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(blocks), dim3(256), 0, st, r);
  return hipGetLastError();
}

}  // namespace nf
