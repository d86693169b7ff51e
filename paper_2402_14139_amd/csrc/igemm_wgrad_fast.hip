// Fast path of the implicit-GEMM weight gradient (see igemm_wgrad.hip for the GEMM view and the
// gradient line of Algorithm 2 it serves; NeuroFlux, arXiv 2402.14139).
//
// Requirements (checked by the launcher): channel counts and P multiples of 4, every operand
// smaller than 2 GiB.  What differs from the general kernel:
//   - all global reads are raw buffer loads with "no data here" (row past the split, tap outside
//     the image, column past P or Q) expressed as an out-of-range offset that the hardware answers
//     with zeros: the gather has no branches;
//   - global loads run two staging steps ahead of the MFMAs (two register sets), LDS fragment
//     reads one sub-step ahead (two fragment slots), one barrier per step;
//   - steps run in unconditional pairs, so the accumulators never leave the MFMA register file;
//   - columns of the 1x1 projection shortcut are fetched by a second load whose result is added
//     (one of the two is always zero), instead of a per-lane branch.
#include <type_traits>

#include "nf_internal.h"

namespace nf {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int BKM = 32;  // reduction rows staged per step
constexpr int NTHREADS = 256;
constexpr int OOB = (int)0x80000000;    // offset no buffer of < 2 GiB contains
constexpr int RSRC_FLAGS = 0x00020000;  // raw buffer, 32-bit data format

__device__ inline float4 bload(__amdgpu_buffer_rsrc_t r, int voff) {
  const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, 0, 0));
  return make_float4(v.x, v.y, v.z, v.w);
}

template <int N>
struct Frag;
template <>
struct Frag<1> {
  static __device__ inline void ld(const float *s, float *v) { v[0] = s[0]; }
};
template <>
struct Frag<2> {
  static __device__ inline void ld(const float *s, float *v) {
    const float2 t = *reinterpret_cast<const float2 *>(s);
    v[0] = t.x, v[1] = t.y;
  }
};
template <>
struct Frag<4> {
  static __device__ inline void ld(const float *s, float *v) {
    const float4 t = *reinterpret_cast<const float4 *>(s);
    v[0] = t.x, v[1] = t.y, v[2] = t.z, v[3] = t.w;
  }
};

// BP x BQ output tile, WP x WQ waves, each wave (32*PT) x (32*QT); LDS tiles [m][p], [m][q].
// PROJ 0: no projection columns.  1: a tile may hold taps and projection channels (RSC not a
// multiple of BQ): two loads per row, one of them out of range.  2: RSC is a multiple of BQ, a
// tile is all taps or all projection channels: one load, its source picked per workgroup.
template <int BP, int BQ, int WP, int WQ, int PROJ>
__global__ __launch_bounds__(NTHREADS, 2) void igemm_wgrad_fast_kernel(WgradProblem p) {
  constexpr int TP = BP / WP, TQ = BQ / WQ;
  constexpr int PT = TP / 32, QT = TQ / 32;
  static_assert(WP * WQ == 4 && (PT == 1 || PT == 2 || PT == 4) && (QT == 1 || QT == 2 || QT == 4), "tile");
  constexpr int LDP = BP + 4, LDQ = BQ + 4;
  constexpr int CP = BP / 4, CQ = BQ / 4;                // 16-byte chunks per staged row
  constexpr int RP = NTHREADS / CP, RQ = NTHREADS / CQ;  // rows covered per pass
  constexpr int NP = BKM / RP, NQ = BKM / RQ;            // passes per step
  static_assert(NP >= 1 && NQ >= 1 && RP * NP == BKM && RQ * NQ == BKM, "staging");
  constexpr int NSS = BKM / 4;  // sub-steps per step: two MFMA k-slices (4 reduction rows) each

  __shared__ __attribute__((aligned(16))) float Ds[2][BKM][LDP];
  __shared__ __attribute__((aligned(16))) float Xs[2][BKM][LDQ];
  __shared__ int4 Rt[2][BKM];

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wp = wave / WQ, wq = wave % WQ;
  const int j = lane & 31, h = lane >> 5;
  // Workgroups are handed to the 8 XCDs (each with its own L2) round-robin by linear index.  The
  // index is re-mapped so that each XCD gets a contiguous run of (split, p-tile, q-tile) with the
  // tiles fastest: all tiles of one split read the same rows of D and X, which then come from that
  // XCD's L2 once instead of from every L2.
  const int gx = gridDim.x, gy = gridDim.y;
  const int nwg = gx * gy * (int)gridDim.z;
  const int lin = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
  const int per = nwg >> 3, rem = nwg & 7, xcd = lin & 7, slot = lin >> 3;
  const int log_id = xcd < rem ? xcd * (per + 1) + slot : rem * (per + 1) + (xcd - rem) * per + slot;
  const int bx = log_id % gx, byz = log_id / gx, by = byz % gy, bz = byz / gy;
  const int p0 = by * BP, q0 = bx * BQ;
  const int m_begin = bz * p.m_per_split;
  const int m_end = min(p.M, m_begin + p.m_per_split);

  // D staging: this thread always loads columns p0 + chp*4 .. +3
  const int chp = t % CP, rowp = t / CP;
  const int pcol = p0 + chp * 4;
  // X staging: this thread always loads columns q0 + chq*4 .. +3, i.e. one fixed (r,s,c) or one
  // fixed projection channel
  const int chq = t % CQ, rowq = t / CQ;
  const int qcol = q0 + chq * 4;
  const bool is_tap = qcol < p.RSC, is_proj = PROJ != 0 && !is_tap && qcol < p.Q;
  const bool tile_proj = PROJ == 2 && q0 >= p.RSC;  // uniform
  int qr = 0, qs = 0, qc = 0;
  if (is_tap) {
    const int tap = qcol / p.C;
    qc = qcol - tap * p.C;
    qr = tap / p.S;
    qs = tap - qr * p.S;
  } else {
    qc = qcol - p.RSC;
  }
  const int dcol_off = pcol < p.P ? pcol * 4 : OOB;  // byte offset of this thread's D columns
  const int xtap_off = ((qr * p.W + qs) * p.C + qc) * 4;

  const __amdgpu_buffer_rsrc_t rsd = __builtin_amdgcn_make_buffer_rsrc((void *)p.d, 0, p.d_bytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rsx = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, p.x_bytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rsxs = __builtin_amdgcn_make_buffer_rsrc((void *)p.xs, 0, p.xs_bytes, RSRC_FLAGS);
  // PROJ == 2: the one source of this workgroup's X columns
  const __amdgpu_buffer_rsrc_t rs_sel = __builtin_amdgcn_make_buffer_rsrc(
      (void *)(tile_proj ? p.xs : p.x), 0, tile_proj ? p.xs_bytes : p.x_bytes, RSRC_FLAGS);
  const int proj_mask = tile_proj ? -1 : 0;

  float4 rd[2][NP], rx[2][NQ];
  float4 bsum = make_float4(0.f, 0.f, 0.f, 0.f);
  const bool do_bias = (bx == 0) && (p.part_b != nullptr);
  const float bsel = do_bias ? 1.f : 0.f;

  // Row table: entry r of Rt[s & 1] describes reduction row m_begin + 32*s + r of staging step s:
  // {byte offset of its receptive field's corner in x, hi0, wi0, byte offset of its pixel in the
  // projection input}; hi0 is far negative for rows past the split.  Every thread decodes ONE row
  // per step (threads with equal t & 31 write the same entry) instead of its NQ rows.
  auto rt_make = [&](int s) {
    const int m = m_begin + s * BKM + (t & (BKM - 1));
    const int img = (int)p.div_howo.div((uint32_t)m);
    const int rem = m - img * p.Ho * p.Wo;
    const int ho = (int)p.div_wo.div((uint32_t)rem);
    const int wo = rem - ho * p.Wo;
    const int hi0 = ho * p.stride - p.pad, wi0 = wo * p.stride - p.pad;
    int4 e;
    e.x = ((img * p.H + hi0) * p.W + wi0) * p.C * 4;
    e.y = m < m_end ? hi0 : -(1 << 20);
    e.z = wi0;
    e.w = PROJ != 0 ? ((img * p.Hs + ho * p.ss) * p.Ws + wo * p.ss) * p.Cs * 4 : 0;
    Rt[s & 1][t & (BKM - 1)] = e;
  };

  // Branch-free gather of staging step `s` into register set `set` (the X rows go by the table entries
  // tread(s) fetched from Rt[s & 1]), one staged row per call so that the step can place the loads
  // between its MFMAs.
  auto gload_d = [&](int s, int set, int i) {
    const int m = m_begin + s * BKM + rowp + RP * i;
    const bool ok = (m < m_end) & (dcol_off != OOB);
    rd[set][i] = bload(rsd, (m * p.P * 4 + dcol_off) | (ok ? 0 : OOB));
  };
  int4 te[NQ];  // this thread's table entries of the step being loaded
  auto tread = [&](int s) {
#pragma unroll
    for (int i = 0; i < NQ; ++i) te[i] = Rt[s & 1][rowq + RQ * i];
  };
  auto gload_x = [&](int set, int i) {
    const int4 e = te[i];
    const bool ok = is_tap & ((unsigned)(e.y + qr) < (unsigned)p.H) & ((unsigned)(e.z + qs) < (unsigned)p.W);
    // the offset is formed unconditionally and pushed out of range by its top bit: a select would
    // let the compiler sink the table read into a branch
    float4 v;
    if constexpr (PROJ == 2) {
      // bit selects with the workgroup-uniform mask: a ?: here would be turned into branches
      const int okp = (is_proj & (e.y > -(1 << 19))) ? 0 : OOB, okt = ok ? 0 : OOB;
      const int off = (((e.w + qc * 4) | okp) & proj_mask) | (((e.x + xtap_off) | okt) & ~proj_mask);
      v = bload(rs_sel, off);
    } else {
      v = bload(rsx, (e.x + xtap_off) | (ok ? 0 : OOB));
      if constexpr (PROJ == 1) {
        const bool okp = is_proj & (e.y > -(1 << 19));
        const float4 u = bload(rsxs, (e.w + qc * 4) | (okp ? 0 : OOB));
        v.x += u.x, v.y += u.y, v.z += u.z, v.w += u.w;  // one of the two is all zeros
      }
    }
    rx[set][i] = v;
  };
  auto gload = [&](int s, int set) {
#pragma unroll
    for (int i = 0; i < NP; ++i) gload_d(s, set, i);
    tread(s);
#pragma unroll
    for (int i = 0; i < NQ; ++i) gload_x(set, i);
  };

  auto lstore_d = [&](int buf, int set, int i) {
    *reinterpret_cast<float4 *>(&Ds[buf][rowp + RP * i][chp * 4]) = rd[set][i];
    bsum.x += bsel * rd[set][i].x, bsum.y += bsel * rd[set][i].y, bsum.z += bsel * rd[set][i].z,
        bsum.w += bsel * rd[set][i].w;
  };
  auto lstore_x = [&](int buf, int set, int i) {
    *reinterpret_cast<float4 *>(&Xs[buf][rowq + RQ * i][chq * 4]) = rx[set][i];
  };
  auto lstore = [&](int buf, int set) {
#pragma unroll
    for (int i = 0; i < NP; ++i) lstore_d(buf, set, i);
#pragma unroll
    for (int i = 0; i < NQ; ++i) lstore_x(buf, set, i);
  };

  floatx16 acc[PT][QT];
#pragma unroll
  for (int a = 0; a < PT; ++a)
#pragma unroll
    for (int b = 0; b < QT; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  // fragments of one sub-step: two k-slices (rows 4*ss + 2*k2 + h), PT / QT consecutive columns
  float df[2][2][PT], xf[2][2][QT];
  auto lfrag = [&](int buf, int ss, int slot) {
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2) {
      Frag<PT>::ld(&Ds[buf][4 * ss + 2 * k2 + h][wp * TP + PT * j], df[slot][k2]);
      Frag<QT>::ld(&Xs[buf][4 * ss + 2 * k2 + h][wq * TQ + QT * j], xf[slot][k2]);
    }
  };
  auto mma = [&](int slot) {
#pragma unroll
    for (int k2 = 0; k2 < 2; ++k2)
#pragma unroll
      for (int a = 0; a < PT; ++a)
#pragma unroll
        for (int b = 0; b < QT; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(df[slot][k2][a], xf[slot][k2][b], acc[a][b], 0, 0, 0);
  };

  // ---- software pipeline: step s uses LDS buffer s&1 ----
  //   sub-steps 0..NSS-2: fragment reads of sub-step ss+1 ride on the MFMAs of sub-step ss; the
  //     address arithmetic and buffer loads of step s+2 are spread over the first four sub-steps,
  //     the LDS writes of step s+1 (loaded one step ago) over the next three;
  //   barrier; first fragments of step s+1; MFMAs of the last sub-step.
  // Every sub-step is closed by a scheduling fence: without it the compiler moves fragment reads
  // between sub-steps and some end up right in front of the MFMA that needs them.
  constexpr int NM = 2 * PT * QT;  // MFMAs per sub-step
  constexpr int NW = NP + NQ;      // staged rows per thread and step (buffer loads, LDS writes)
  constexpr int LPS = (NW + 3) / 4;  // rows loaded per sub-step over sub-steps 0..3
  constexpr int WPS = (NW + 2) / 3;  // rows written per sub-step over sub-steps 4..6
  static_assert(NSS == 8, "placement of loads and writes");
  auto step = [&](int s, auto par_tag) {
    constexpr int par = decltype(par_tag)::value;
#pragma unroll
    for (int ss = 0; ss + 1 < NSS; ++ss) {
      lfrag(par, ss + 1, (ss + 1) & 1);
      mma(ss & 1);
      if (ss == 0) {
        tread(s + 2);     // table entries a sub-step or more ahead of the loads that need them
        rt_make(s + 3);   // the other table buffer
      }
      if (ss < 4) {                 // step s + 2 into set `par`, which held step s, already in LDS
#pragma unroll
        for (int it = ss * LPS; it < (ss + 1) * LPS && it < NW; ++it) {
          if (it < NP) gload_d(s + 2, par, it);
          else gload_x(par, it - NP);
        }
      } else {                      // step s + 1
#pragma unroll
        for (int it = (ss - 4) * WPS; it < (ss - 3) * WPS && it < NW; ++it) {
          if (it < NP) lstore_d(par ^ 1, par ^ 1, it);
          else lstore_x(par ^ 1, par ^ 1, it - NP);
        }
      }
#pragma unroll
      for (int i = 0; i < NM; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                          // one MFMA
        if (i < 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);              // + fragment reads
        if (ss < 4) __builtin_amdgcn_sched_group_barrier(0x002, 6, 0);             // + address VALU
        if (ss < 4 && i < 2 * LPS) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // + a buffer load
        if (ss >= 4 && i < WPS) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0); // + an LDS write
        if (ss >= 4) __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
    lfrag(par ^ 1, 0, 0);
    mma((NSS - 1) & 1);
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
      if (i < 2) __builtin_amdgcn_sched_group_barrier(0x100, 2, 1);
    }
  };

  const int nsteps = (m_end - m_begin + BKM - 1) / BKM;
  rt_make(0);
  rt_make(1);
  __syncthreads();
  gload(0, 0);
  lstore(0, 0);
  gload(1, 1);
  __syncthreads();  // table reads done
  rt_make(2);
  __syncthreads();
  lfrag(0, 0, 0);
  // unconditional pairs inside the loop (a conditional second step there makes the compiler move the
  // accumulators out of and back into the MFMA register file around every iteration); an odd count
  // ends with one step after the loop
  int s = 0;
  for (; s + 1 < nsteps; s += 2) {
    step(s, std::integral_constant<int, 0>{});
    step(s + 1, std::integral_constant<int, 1>{});
  }
  if (nsteps & 1) step(s, std::integral_constant<int, 0>{});

  // ---- store the partial tile: lane holds, per (a, e), QT consecutive q ----
  float *part = p.part + (long long)bz * p.P * p.Qld;
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
      p.part_b[(long long)bz * p.P + p0 + t] = s;
    }
  }
}

template <int BP, int BQ, int WP, int WQ>
hipError_t launch_cfg(const WgradProblem &p, hipStream_t st) {
  dim3 grid((p.Q + BQ - 1) / BQ, (p.P + BP - 1) / BP, p.splits);
  if (p.Cs && p.RSC % BQ == 0)
    hipLaunchKernelGGL((igemm_wgrad_fast_kernel<BP, BQ, WP, WQ, 2>), grid, dim3(NTHREADS), 0, st, p);
  else if (p.Cs)
    hipLaunchKernelGGL((igemm_wgrad_fast_kernel<BP, BQ, WP, WQ, 1>), grid, dim3(NTHREADS), 0, st, p);
  else
    hipLaunchKernelGGL((igemm_wgrad_fast_kernel<BP, BQ, WP, WQ, 0>), grid, dim3(NTHREADS), 0, st, p);
  return hipGetLastError();
}

}  // namespace

bool igemm_wgrad_fast_applicable(const WgradProblem &p) {
  const long long lim = 0x7FFFFFF0ll, B = p.M / ((long long)p.Ho * p.Wo);
  if (p.C % 4 || p.Cs % 4 || p.P % 4) return false;
  if ((long long)p.M * p.P * 4 > lim || B * p.H * p.W * p.C * 4 > lim) return false;
  if (p.Cs && B * p.Hs * p.Ws * p.Cs * 4 > lim) return false;
  return true;
}

hipError_t launch_igemm_wgrad_fast(const WgradProblem &p0, hipStream_t st, const char **kernel) {
  if (contraction_mode() != NF_CONTRACT_F32 && igemm_wgrad_split_applicable(p0))
    return launch_igemm_wgrad_split(p0, contraction_mode() == NF_CONTRACT_BF16X9, st, kernel);
  WgradProblem p = p0;
  const long long B = p.M / ((long long)p.Ho * p.Wo);
  p.d_bytes = (uint32_t)((long long)p.M * p.P * 4);
  p.x_bytes = (uint32_t)(B * p.H * p.W * p.C * 4);
  p.xs_bytes = p.Cs ? (uint32_t)(B * p.Hs * p.Ws * p.Cs * 4) : 0;
  if (p.P > 64) {
    *kernel = "igemm_wgrad_fast_128x128";
    return launch_cfg<128, 128, 2, 2>(p, st);
  }
  if (p.P > 32) {
    *kernel = "igemm_wgrad_fast_64x64";
    return launch_cfg<64, 64, 2, 2>(p, st);
  }
  *kernel = "igemm_wgrad_fast_32x128";
  return launch_cfg<32, 128, 1, 4>(p, st);
}

}  // namespace nf
