// Fast path of the implicit-GEMM convolution (see igemm_fwd.hip for the GEMM view and the
// steps of the local training step it serves; NeuroFlux, arXiv 2402.14139, Eq. 1, Eq. 2 and
// the data gradient of beta_n).
//
// Requirements (checked by the launcher): channel counts multiples of 4, at most 32 filter
// taps, every operand smaller than 2 GiB.  What differs from the general kernel:
//   - all global reads are raw buffer loads; out-of-image taps, rows past M or N and the
//     padding of the reduction axis are expressed as an out-of-range offset, for which the
//     hardware returns zeros: the gather has no branches and no selects on data;
//   - per output row the validity of every filter tap is a bit mask computed once, and the
//     (tap, channel) decode of a thread's 16-byte chunk is two multiply-high divisions;
//   - the 1x1 projection shortcut is appended as whole reduction steps of its own;
//   - LDS fragment reads of sub-step ks+1 are issued before the MFMAs of sub-step ks;
//   - MFMA shape is a template parameter: 32x32x2 for the wide contractions, 16x16x4 for
//     the skinny ones (auxiliary heads with at most 16 filters).
#include <type_traits>

#include "nf_internal.h"

namespace nf {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));

constexpr int OOB = (int)0x80000000;      // offset no buffer of < 2 GiB contains
constexpr int RSRC_FLAGS = 0x00020000;    // raw buffer, 32-bit data format

struct FastAux {
  FastDiv div_c, div_s;
  uint32_t x_bytes, w_bytes, xs_bytes, wp_bytes;
  int nkb_conv, nkb_proj;
  FastDiv div_taps;
  int kb_per;  // reduction steps per split (gridDim.y splits; every split but the last gets this many)
};

__device__ inline float4 bload(__amdgpu_buffer_rsrc_t r, int voff) {
  const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, 0, 0));
  return make_float4(v.x, v.y, v.z, v.w);
}

template <int MF>
struct Mfma;
template <>
struct Mfma<32> {
  typedef floatx16 acc_t;
  static constexpr int NACC = 16, KSTEP = 8;  // k covered by one 16-byte fragment read
  static __device__ inline acc_t run(float a, float b, acc_t c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }
  // row of accumulator element e for lane group g (= lane / 32)
  static __device__ inline int row(int e, int g) { return 8 * (e >> 2) + 4 * g + (e & 3); }
};
template <>
struct Mfma<16> {
  typedef floatx4 acc_t;
  static constexpr int NACC = 4, KSTEP = 16;
  static __device__ inline acc_t run(float a, float b, acc_t c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }
  static __device__ inline int row(int e, int g) { return 4 * g + e; }  // g = lane / 16
};

// BK = reduction length staged per step (one barrier per step): 32 for the wide tiles, longer for
// the skinny ones, whose steps are dominated by the fixed cost of the barrier.
// MODE 0: plain; 1: projection shortcut appended to the reduction; 2: the epilogue operand (identity
// shortcut or ReLU mask, one value per output element) is fetched into registers before the main
// loop instead of at its end, where nothing would hide the latency.
// TI: order of the reduction axis.  false: kg = (tap, channel) as stored.  true (channels a multiple
// of BK): step kb = (channel chunk, tap) with the tap fastest, so that the shifted reads of one
// channel chunk by the R*S taps are neighbours in time and hit in L2 instead of re-streaming x from
// the fabric once per tap (measured: less than half of the fetched bytes).
template <int BM, int BN, int BK, int WM, int WN, int MF, int MODE, bool SCHED, bool TI>
__global__ __launch_bounds__(WM *WN * 64) void igemm_fwd_fast_kernel(FwdProblem p, FastAux q) {
  constexpr bool PROJ = MODE == 1, EPI = MODE == 2;
  using MM = Mfma<MF>;
  using acc_t = typename MM::acc_t;
  // Row padding that keeps the 16-byte fragment reads free of bank conflicts (counted with
  // SQ_LDS_BANK_CONFLICT on a read-only loop): a wave reading 32 consecutive rows (32x32x2 fragments)
  // needs a row stride of 4 mod 32 floats, one reading 16 consecutive rows in four k groups
  // (16x16x4 fragments) a stride of 8 mod 16; the other choice doubles the LDS time of every read.
  constexpr int LDK = BK + (MF == 16 ? 8 : 4);
  constexpr int NTHREADS = WM * WN * 64;
  constexpr int CPR = BK / 4;        // 16-byte chunks per staged row
  constexpr int RPP = NTHREADS / CPR;  // rows staged per pass
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int MT = TM / MF, NT = TN / MF;
  constexpr int PA = BM / RPP, PB = (BN + RPP - 1) / RPP;
  constexpr int NKS = BK / MM::KSTEP;
  static_assert(MT >= 1 && NT >= 1 && BM % RPP == 0, "tile");

  __shared__ __attribute__((aligned(16))) float As[2][BM][LDK];
  __shared__ __attribute__((aligned(16))) float Bs[2][BN][LDK];

  const int t = threadIdx.x;
  const int lane = t & 63, wave = t >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int j = lane % MF, g = lane / MF;  // row/column inside an MFMA tile, k group

  const int tiles_n = (p.N + BN - 1) / BN;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, q.x_bytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)p.w, 0, q.w_bytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rxs = __builtin_amdgcn_make_buffer_rsrc((void *)p.xs, 0, q.xs_bytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rwp = __builtin_amdgcn_make_buffer_rsrc((void *)p.wp, 0, q.wp_bytes, RSRC_FLAGS);

  // ---- per-thread gather state: chunk `ch` (4 consecutive kg) of rows row0 + RPP*i ----
  const int ch = t % CPR, row0 = t / CPR;
  int abase[PA], sbase[PA];
  uint32_t amask[PA];
#pragma unroll
  for (int i = 0; i < PA; ++i) {
    const int m = m0 + row0 + RPP * i;
    abase[i] = 0, sbase[i] = OOB, amask[i] = 0;
    if (m < p.M) {
      const int img = (int)p.div_howo.div((uint32_t)m);
      const int rem = m - img * p.Ho * p.Wo;
      const int ho = (int)p.div_wo.div((uint32_t)rem);
      const int wo = rem - ho * p.Wo;
      const int hi0 = ho * p.stride - p.pad, wi0 = wo * p.stride - p.pad;
      abase[i] = ((img * p.H + hi0) * p.W + wi0) * p.C * 4;  // may point before the image: used only with a valid tap
      uint32_t mask = 0;
      for (int r = 0; r < p.R; ++r)
        for (int s = 0; s < p.S; ++s)
          if ((unsigned)(hi0 + r) < (unsigned)p.H && (unsigned)(wi0 + s) < (unsigned)p.W) mask |= 1u << (r * p.S + s);
      amask[i] = mask;
      if (q.nkb_proj) sbase[i] = ((img * p.Hs + ho * p.ss) * p.Ws + wo * p.ss) * p.Cs * 4;
    }
  }
  int bbase[PB], pbase[PB];
#pragma unroll
  for (int i = 0; i < PB; ++i) {
    const int n = n0 + row0 + RPP * i;
    const bool ok = n < p.N && (row0 + RPP * i) < BN;
    bbase[i] = ok ? n * p.RSC * 4 : OOB;
    pbase[i] = ok ? n * p.Cs * 4 : OOB;
  }

  // Two register sets of staged chunks: global loads run two reduction steps ahead of the MFMAs.
  float4 ra[2][PA], rb[2][PB];
  // this workgroup's share of the reduction: steps [kb0, kb_end)
  const int kb0 = blockIdx.y * q.kb_per;
  const int kb_end = min(q.nkb_conv + q.nkb_proj, kb0 + q.kb_per);

  // Branch-free gather of step kb into register set `set`.  Steps past the end, the padding of the
  // reduction axis, taps outside the image and rows past M or N all become the out-of-range
  // offset.  The projection steps (kb >= nkb_conv) read the shortcut tensor and its 1x1 filter
  // through a uniform select of the buffer descriptor.
  auto gload = [&](int kb, int set) {
    int kg, tap, c;
    bool in;
    if constexpr (TI) {  // step kb = (channel chunk, tap): the tap is uniform over the step
      const int cc = (int)q.div_taps.div((uint32_t)kb);
      in = (kb < q.nkb_conv) & (kb < kb_end);
      tap = in ? kb - cc * (p.R * p.S) : 0;
      c = cc * BK + ch * 4;
      kg = tap * p.C + c;
    } else {
      kg = kb * BK + ch * 4;
      in = (kg < p.RSC) & (kb < kb_end);
      tap = in ? (int)q.div_c.div((uint32_t)kg) : 0;
      c = kg - tap * p.C;
    }
    const int r = (int)q.div_s.div((uint32_t)tap);
    const int sx = tap - r * p.S;
    const int toff = ((r * p.W + sx) * p.C + c) * 4;
    int offa[PA], offb[PB];
#pragma unroll
    for (int i = 0; i < PA; ++i) offa[i] = (in && ((amask[i] >> tap) & 1u)) ? abase[i] + toff : OOB;
#pragma unroll
    for (int i = 0; i < PB; ++i) offb[i] = (in && bbase[i] != OOB) ? bbase[i] + kg * 4 : OOB;
    if constexpr (PROJ) {
      const bool is_proj = kb >= q.nkb_conv;  // uniform
      const int cp = (kb - q.nkb_conv) * BK + ch * 4;
      const bool inp = is_proj && cp < p.Cs && kb < kb_end;
#pragma unroll
      for (int i = 0; i < PA; ++i) offa[i] = is_proj ? ((inp && sbase[i] != OOB) ? sbase[i] + cp * 4 : OOB) : offa[i];
#pragma unroll
      for (int i = 0; i < PB; ++i) offb[i] = is_proj ? ((inp && pbase[i] != OOB) ? pbase[i] + cp * 4 : OOB) : offb[i];
      if (is_proj) {
#pragma unroll
        for (int i = 0; i < PA; ++i) ra[set][i] = bload(rxs, offa[i]);
#pragma unroll
        for (int i = 0; i < PB; ++i) rb[set][i] = bload(rwp, offb[i]);
        return;
      }
    }
#pragma unroll
    for (int i = 0; i < PA; ++i) ra[set][i] = bload(rx, offa[i]);
#pragma unroll
    for (int i = 0; i < PB; ++i) rb[set][i] = bload(rw, offb[i]);
  };

  auto lstore = [&](int buf, int set) {
#pragma unroll
    for (int i = 0; i < PA; ++i) *reinterpret_cast<float4 *>(&As[buf][row0 + RPP * i][ch * 4]) = ra[set][i];
#pragma unroll
    for (int i = 0; i < PB; ++i)
      if (BN >= RPP * (i + 1) || row0 + RPP * i < BN)
        *reinterpret_cast<float4 *>(&Bs[buf][row0 + RPP * i][ch * 4]) = rb[set][i];
  };

  acc_t acc[MT][NT];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < NT; ++b)
#pragma unroll
      for (int e = 0; e < MM::NACC; ++e) acc[a][b][e] = 0.f;

  float4 af[2][MT], bf[2][NT];
  auto lfrag = [&](int buf, int ks, int slot) {
#pragma unroll
    for (int a = 0; a < MT; ++a)
      af[slot][a] = *reinterpret_cast<const float4 *>(&As[buf][wm * TM + a * MF + j][ks * MM::KSTEP + g * 4]);
#pragma unroll
    for (int b = 0; b < NT; ++b)
      bf[slot][b] = *reinterpret_cast<const float4 *>(&Bs[buf][wn * TN + b * MF + j][ks * MM::KSTEP + g * 4]);
  };
  auto mma = [&](int slot) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
#pragma unroll
      for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b) {
          const float av = kk == 0 ? af[slot][a].x : kk == 1 ? af[slot][a].y : kk == 2 ? af[slot][a].z : af[slot][a].w;
          const float bv = kk == 0 ? bf[slot][b].x : kk == 1 ? bf[slot][b].y : kk == 2 ? bf[slot][b].z : bf[slot][b].w;
          acc[a][b] = MM::run(av, bv, acc[a][b]);
        }
    }
  };
  static_assert(NKS % 2 == 0, "fragment slots alternate per sub-step");

  // ---- software pipeline ------------------------------------------------------------------
  // Step kb (LDS buffer kb&1):
  //   sub-steps 0..NKS-2: fragment reads of sub-step ks+1 ride on the first MFMAs of sub-step ks;
  //     the address arithmetic and the buffer loads of step kb+2 are spread between the MFMAs of
  //     the first sub-steps; the LDS writes of step kb+1 (loaded one step ago) ride on the MFMAs
  //     of sub-step NKS-2;
  //   barrier; first fragments of step kb+1; MFMAs of the last sub-step.
  // One barrier per step, and no instruction class waits for the MFMA pipe to drain.
  constexpr int NM = 4 * MT * NT;   // MFMAs per sub-step
  constexpr int NR = MT + NT;       // fragment reads per sub-step
  constexpr int NV = PA + PB;       // buffer loads (and LDS writes) per step
  auto step = [&](int kb, auto par_tag) {
    constexpr int par = decltype(par_tag)::value;
    gload(kb + 2, par);  // set `par` held step kb, already in LDS
    static_assert(!SCHED || NKS > 2, "placement of loads and writes");
#pragma unroll
    for (int ks = 0; ks + 1 < NKS; ++ks) {
      lfrag(par, ks + 1, (ks + 1) & 1);
      mma(ks & 1);
      if (ks + 2 == NKS) lstore(par ^ 1, par ^ 1);  // step kb+1
      if constexpr (SCHED) {
#pragma unroll
        for (int i = 0; i < NM; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                      // one MFMA
          if (i < NR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);          // + a fragment read
          if (ks == 0) __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);         // + address VALU
          if (ks == 1 && i >= NR && i < NR + NV) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);         // + a buffer load
          if (ks + 2 == NKS && i >= NR && i < NR + NV) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);  // + an LDS write
          if (ks != 0) __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);
        }
        // Fragment reads stay in the sub-step they were written in: without this fence the compiler
        // moved some of them right in front of the MFMA that needs them.
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __syncthreads();
    lfrag(par ^ 1, 0, 0);
    mma((NKS - 1) & 1);
    if constexpr (SCHED) {
#pragma unroll
      for (int i = 0; i < NM; ++i) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
        if (i < NR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 1);
      }
    }
  };

  gload(kb0, 0);
  float epi[EPI ? MT : 1][EPI ? NT : 1][EPI ? MM::NACC : 1];
  if constexpr (EPI) {
    const float *src = p.addsrc ? p.addsrc : p.mask;
#pragma unroll
    for (int b = 0; b < NT; ++b) {
      const int n = n0 + wn * TN + b * MF + j;
#pragma unroll
      for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int e = 0; e < MM::NACC; ++e) {
          const int m = m0 + wm * TM + a * MF + MM::row(e, g);
          epi[a][b][e] = (n < p.N && m < p.M) ? src[(long long)m * p.N + n] : 0.f;
        }
    }
  }
  lstore(0, 0);
  gload(kb0 + 1, 1);
  __syncthreads();
  lfrag(0, 0, 0);
  // Inside the loop the steps go in pairs with no branch between them: a conditional second step
  // there makes the compiler copy every accumulator out of and back into the MFMA register file at
  // the loop head, behind a wait for all loads.  The last step of an odd count follows the loop.
  int kb = kb0;
  for (; kb + 1 < kb_end; kb += 2) {
    step(kb, std::integral_constant<int, 0>{});
    step(kb + 1, std::integral_constant<int, 1>{});
  }
  if ((kb_end - kb0) & 1) step(kb, std::integral_constant<int, 0>{});  // odd count: the last step, after the loop

  // ---- split reduction: raw partial sums, slice blockIdx.y of out[splits][M][N] ----
  if (gridDim.y > 1) {
    float *part = p.out + (long long)blockIdx.y * p.M * p.N;
#pragma unroll
    for (int b = 0; b < NT; ++b) {
      const int n = n0 + wn * TN + b * MF + j;
      if (n >= p.N) continue;
#pragma unroll
      for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int e = 0; e < MM::NACC; ++e) {
          const int m = m0 + wm * TM + a * MF + MM::row(e, g);
          if (m < p.M) part[(long long)m * p.N + n] = acc[a][b][e];
        }
    }
    return;
  }

  // ---- epilogue: bias, identity shortcut, ReLU, mask; consecutive lanes store consecutive n ----
#pragma unroll
  for (int b = 0; b < NT; ++b) {
    const int n = n0 + wn * TN + b * MF + j;
    if (n >= p.N) continue;
    const float bias = p.bias ? p.bias[n] : 0.f;
#pragma unroll
    for (int a = 0; a < MT; ++a) {
#pragma unroll
      for (int e = 0; e < MM::NACC; ++e) {
        const int m = m0 + wm * TM + a * MF + MM::row(e, g);
        if (m >= p.M) continue;
        const long long o = (long long)m * p.N + n;
        float v = acc[a][b][e] + bias;
        if (p.addsrc) v += EPI ? epi[EPI ? a : 0][EPI ? b : 0][EPI ? e : 0] : p.addsrc[o];
        if (p.relu) v = v > 0.f ? v : 0.f;
        if (p.mask) v = (EPI ? epi[EPI ? a : 0][EPI ? b : 0][EPI ? e : 0] : p.mask[o]) > 0.f ? v : 0.f;
        p.out[o] = v;
      }
    }
  }

  // ---- pooled partial sums for the head (16x16x4 tiles, whole tiles only): the lane's four rows,
  // then the lane groups 0+1 and 2+3 (rows 0-7, 8-15 of the wave's 16), then both (fixed order) ----
  if constexpr (MF == 16 && MT == 1) {
    if (p.pool_part) {
      const int r16 = (m0 + wm * TM) >> 4;
#pragma unroll
      for (int b = 0; b < NT; ++b) {
        const int n = n0 + wn * TN + b * MF + j;
        const float bias = (n < p.N && p.bias) ? p.bias[n] : 0.f;
        float ps = 0.f;
#pragma unroll
        for (int e = 0; e < MM::NACC; ++e) {
          float v = acc[0][b][e] + bias;
          if (p.relu) v = v > 0.f ? v : 0.f;
          ps += v;
        }
        ps += __shfl_xor(ps, 16, 64);
        if (!p.pool_split) ps += __shfl_xor(ps, 32, 64);
        if (n < p.N && (g == 0 || (p.pool_split && g == 2)))
          p.pool_part[((long long)r16 * 2 + (g >> 1)) * p.N + n] = ps;
      }
    }
  }
}

template <int BM, int BN, int BK, int WM, int WN, int MF>
hipError_t launch_cfg(const FwdProblem &p, FastAux q, hipStream_t st) {
  const int tiles = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
  constexpr bool SCHED = MF == 32;
  q.nkb_conv = (p.RSC + BK - 1) / BK;
  q.nkb_proj = p.Cs ? (p.Cs + BK - 1) / BK : 0;
  q.div_taps = FastDiv(p.R * p.S);
  const int nkb = q.nkb_conv + q.nkb_proj;
  const int splits = p.ksplits > 1 ? p.ksplits : 1;
  q.kb_per = (nkb + splits - 1) / splits;
  const dim3 grid((unsigned)tiles, (unsigned)splits), block(WM * WN * 64);
  // exactly one of addsrc / mask, no projection, no split: prefetch it (MODE 2)
  const bool epi = !q.nkb_proj && splits == 1 && ((p.addsrc != nullptr) != (p.mask != nullptr));
  const int mode = q.nkb_proj ? 1 : epi ? 2 : 0;
  const bool ti = p.C % BK == 0 && p.R * p.S > 1;
#define NF_LAUNCH(MODE_, TI_) \
  hipLaunchKernelGGL((igemm_fwd_fast_kernel<BM, BN, BK, WM, WN, MF, MODE_, SCHED, TI_>), grid, block, 0, st, p, q)
  if (ti) {
    if (mode == 1) NF_LAUNCH(1, true);
    else if (mode == 2) NF_LAUNCH(2, true);
    else NF_LAUNCH(0, true);
  } else {
    if (mode == 1) NF_LAUNCH(1, false);
    else if (mode == 2) NF_LAUNCH(2, false);
    else NF_LAUNCH(0, false);
  }
#undef NF_LAUNCH
  return hipGetLastError();
}

}  // namespace

// Few output tiles with a long reduction leave most of the chip idle: each workgroup is a long
// serial chain of load -> LDS -> MFMA steps.  Splitting the reduction multiplies the workgroups;
// the consumer adds the partial sums in a fixed order.  Two cases: skinny outputs (few filters:
// the aux heads) and small M*N (late layers at 2x2 .. 4x4 resolution).  Kg = whole reduction
// length (filter taps * channels + projection channels).
int igemm_fwd_pick_ksplits(int M, int N, int Kg, int C, int taps) {
  if (C % 4 || taps > 32) return 1;
  const int nkb = (Kg + 31) / 32;
  if (N <= 32) {
    const int tiles = (M + 63) / 64;
    int s = 1024 / (tiles > 0 ? tiles : 1);
    if (s > nkb / 16) s = nkb / 16;
    if (s > 16) s = 16;
    return s > 1 ? s : 1;
  }
  // tile shape as launch_igemm_fwd_fast picks it
  const int bm = (N > 128 && Kg > 160) ? 128 : 64, bn = bm;
  const int tiles = ((M + bm - 1) / bm) * ((N + bn - 1) / bn);
  if (tiles >= 192) return 1;
  int s = 256 / tiles;
  if (s > nkb / 8) s = nkb / 8;
  if (s > 32) s = 32;
  return s > 1 ? s : 1;
}

bool fwd_pool_partials_applicable(const FwdProblem &p) {
  // the 64x32 / 64x16 tiles of launch_igemm_fwd_fast (16x16x4 MFMA, a wave = 16 consecutive rows),
  // whole tiles, plain epilogue (bias + ReLU), reduction not split over workgroups
  return igemm_fwd_fast_applicable(p) && p.N <= 32 && p.M % 64 == 0 && p.ksplits <= 1 && !p.addsrc && !p.mask &&
         !p.Cs;
}

bool igemm_fwd_fast_applicable(const FwdProblem &p) {
  const long long lim = 0x7FFFFFF0ll;
  const long long B = p.M / ((long long)p.Ho * p.Wo);
  if (p.C % 4 || p.Cs % 4 || p.R * p.S > 32) return false;
  if (B * p.H * p.W * p.C * 4 > lim || (long long)p.N * p.RSC * 4 > lim) return false;
  if (p.Cs && (B * p.Hs * p.Ws * p.Cs * 4 > lim || (long long)p.N * p.Cs * 4 > lim)) return false;
  return true;
}

hipError_t launch_igemm_fwd_fast(const FwdProblem &p, hipStream_t st, const char **kernel) {
  if (contraction_mode() != NF_CONTRACT_F32 && igemm_fwd_split_applicable(p))
    return launch_igemm_fwd_split(p, contraction_mode() == NF_CONTRACT_BF16X9, st, kernel);
  FastAux q;
  const long long B = p.M / ((long long)p.Ho * p.Wo);
  q.div_c = FastDiv(p.C), q.div_s = FastDiv(p.S);
  q.x_bytes = (uint32_t)(B * p.H * p.W * p.C * 4);
  q.w_bytes = (uint32_t)((long long)p.N * p.RSC * 4);
  q.xs_bytes = p.Cs ? (uint32_t)(B * p.Hs * p.Ws * p.Cs * 4) : 0;
  q.wp_bytes = p.Cs ? (uint32_t)((long long)p.N * p.Cs * 4) : 0;
  q.nkb_conv = q.nkb_proj = 0;  // set per tile configuration
  if (p.N > 128 && p.Kg > 160) {
    *kernel = "igemm_fwd_fast_128x128";
    return launch_cfg<128, 128, 32, 2, 2, 32>(p, q, st);
  }
  if (p.N > 32) {
    // at most 128 columns, or one to five reduction steps (bound by the output stream): small
    // tiles keep more workgroups in flight (measured 7-9 % faster than 128x64 at N = 64, 4 %
    // faster than 128x128 at N = 128)
    *kernel = "igemm_fwd_fast_64x64";
    return launch_cfg<64, 64, 32, 2, 2, 32>(p, q, st);
  }
  if (p.N > 16) {
    *kernel = "igemm_fwd_fast_64x32";
    return launch_cfg<64, 32, 32, 4, 1, 16>(p, q, st);  // 16x16x4 MFMA, waves of 16 x 32
  }
  *kernel = "igemm_fwd_fast_64x16";
  if (p.ksplits > 1) return launch_cfg<64, 16, 32, 4, 1, 16>(p, q, st);
  // long reductions: fewer, longer steps (the step cost of this tile is mostly the barrier)
  if (p.Kg > 1536) return launch_cfg<64, 16, 64, 4, 1, 16>(p, q, st);
  return launch_cfg<64, 16, 32, 4, 1, 16>(p, q, st);
}

}  // namespace nf
