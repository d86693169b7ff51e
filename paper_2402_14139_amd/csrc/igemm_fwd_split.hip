// Forward-type implicit-GEMM convolution with fp32 operands and fp32 results, contracted on the
// bf16 matrix cores (optional mode of the library; NeuroFlux, arXiv 2402.14139, Eq. 1 and the
// wide layers of Eq. 2: the same operation as igemm_fwd_fast.hip).
//
// An fp32 number is the exact sum of three bfloat16 numbers: x = h + m + l, each piece holding 8
// of the 24 significant bits (pieces are cut by truncation, so every remainder is exact).  A
// product x*w is then the sum of nine exact piece products; the three smallest (m*l, l*m, l*l:
// |m| < 2^-7 |x|, |l| < 2^-15 |x|, so together below 2^-21 |x*w| in the worst case and about
// 2^-24 |x*w| in the root mean square) are left out and the six others are accumulated in fp32 by
// v_mfma_f32_32x32x16_bf16.  Per multiply-add that is an error of the size of an fp32 rounding;
// measured against an fp64 sum over 576 ... 4608 terms the result is as close as the one of
// v_mfma_f32_32x32x2_f32 (both are dominated by the rounding of the running sum).  Six bf16 MFMAs (8 passes each) cover 16 reduction steps of a
// 32x32 tile in the time of three fp32 MFMAs (16 passes each), which need eight for the same 16
// steps: 2.67x the work per matrix-pipe cycle.  What it costs is vector-ALU work for cutting the
// operands (5.5 instructions per element staged) and 1.5x the LDS bytes (three pieces of 2 bytes).
//
// Non-finite inputs: inf - inf appears in the remainders, so an operand element that is +-inf
// yields NaN where the fp32 kernel would yield +-inf.
//
// Tile 128x128, waves of 64x64 (2x2 MFMA tiles), 32 reduction steps per barrier (two slabs of 16).
// LDS: [buffer][piece][row][32 bf16] with the 16-byte quarters of a row XOR-swizzled, conflict-free.
// Gather (raw buffer loads with hardware zero-fill), reduction order, projection shortcut and
// epilogue as in the fp32 kernel.

#include "nf_internal.h"

namespace nf {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int OOB = (int)0x80000000;      // offset no buffer of < 2 GiB contains
constexpr int RSRC_FLAGS = 0x00020000;    // raw buffer, 32-bit data format

struct SplitAux {
  FastDiv div_c, div_s, div_taps;
  uint32_t x_bytes, w_bytes, xs_bytes, wp_bytes;
  int nkb_conv, nkb_proj;
  int kb_per;  // reduction steps per split (gridDim.y splits)
};

__device__ inline float4 bload(__amdgpu_buffer_rsrc_t r, int voff) {
  const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, 0, 0));
  return make_float4(v.x, v.y, v.z, v.w);
}

// four fp32 values -> their three bf16 pieces, four per piece (8 bytes), element 0 lowest
__device__ inline void split4(const float4 v, uint2 &h, uint2 &m, uint2 &l) {
  const float x[4] = {v.x, v.y, v.z, v.w};
  unsigned hb[4], mb[4], lb[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    hb[e] = __float_as_uint(x[e]);
    const float r1 = x[e] - __uint_as_float(hb[e] & 0xffff0000u);  // exact: the low 16 bits of x
    mb[e] = __float_as_uint(r1);
    const float r2 = r1 - __uint_as_float(mb[e] & 0xffff0000u);    // exact: at most 8 significant bits left
    lb[e] = __float_as_uint(r2);
  }
  constexpr unsigned TOP = 0x07060302u;  // upper halves of (second, first) -> one word
  h = make_uint2(__builtin_amdgcn_perm(hb[1], hb[0], TOP), __builtin_amdgcn_perm(hb[3], hb[2], TOP));
  m = make_uint2(__builtin_amdgcn_perm(mb[1], mb[0], TOP), __builtin_amdgcn_perm(mb[3], mb[2], TOP));
  l = make_uint2(__builtin_amdgcn_perm(lb[1], lb[0], TOP), __builtin_amdgcn_perm(lb[3], lb[2], TOP));
}

// eight fp32 values (two 16-byte chunks) -> 16 bytes per piece
__device__ inline void split8(const float4 v0, const float4 v1, uint4 &h, uint4 &m, uint4 &l) {
  uint2 h0, m0, l0, h1, m1, l1;
  split4(v0, h0, m0, l0);
  split4(v1, h1, m1, l1);
  h = make_uint4(h0.x, h0.y, h1.x, h1.y), m = make_uint4(m0.x, m0.y, m1.x, m1.y), l = make_uint4(l0.x, l0.y, l1.x, l1.y);
}

__device__ inline floatx16 mfma_bf16(uint4 a, uint4 b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// PROJ: the 1x1 projection shortcut is appended to the reduction as steps of its own.
// TI: step kb = (channel chunk, tap) with the tap fastest (channels a multiple of 32).
//
// 512 threads = two groups of four waves, one wave of each group per SIMD.  The groups take the
// reduction steps alternately (group 0 the even ones), each with its own accumulators (added once
// at the end, group 0 + group 1) and its own LDS buffer.  Every wave runs the same loop -- the 48
// MFMAs of a step, with the loads of its next step issued among them; barrier; split the operands
// of that next step into the buffer; barrier -- but group 1 runs it one barrier late, so that
// between two barriers one group is in its MFMAs while the other splits.  A wave issues in order and an MFMA that finds
// the matrix pipe busy holds everything behind it: the vector-ALU work of the split has to come
// from another wave of the SIMD to overlap with the MFMAs.
// NP: piece products per multiply-add: 6 (m*l, l*m, l*l left out) or all 9.
template <bool PROJ, bool TI, int NP>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void igemm_fwd_split_kernel(FwdProblem p, SplitAux q) {
  constexpr int BM = 128, BN = 128, BK = 32;
  constexpr int GT = 256;            // threads per group
  constexpr int CPR = BK / 8;        // 8-element chunks (two 16-byte loads, one 16-byte LDS write per piece) per staged row
  constexpr int RPP = GT / CPR;      // rows staged per pass
  constexpr int MT = 2, NT = 2;      // 32x32 MFMA tiles per wave: 64x64
  constexpr int TM = 64, TN = 64;
  constexpr int PA = BM / RPP, PB = BN / RPP;
  // LDS rows are 32 bf16 = 64 bytes, no padding: four 16-byte quarters, stored at quarter ^ ((row / 4) % 4).
  // A fragment read (16 consecutive rows, one quarter each) and a staging write (a quarter of each of 16
  // consecutive rows, or all of 4) then both touch every bank once.
  constexpr int LDH = BK;
  static_assert(RPP % 16 == 0, "the swizzle of a staged row is the same in every pass");

  // (two arrays, addressed as such: LDS reached through a converted pointer keeps the compiler from
  // holding the per-thread arrays below in registers)
  __shared__ __attribute__((aligned(16))) unsigned short As[2][3][BM][LDH];  // 48 KiB
  __shared__ __attribute__((aligned(16))) unsigned short Bs[2][3][BN][LDH];  // 48 KiB

  const int t = threadIdx.x;
  const int lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int grp = wave >> 2, w4 = wave & 3;
  const int buf = grp;  // the group's LDS buffer
  const int wm = w4 >> 1, wn = w4 & 1;
  const int j = lane % 32, g = lane / 32;  // row/column inside an MFMA tile, k group (8 consecutive k)

  const int tiles_n = (p.N + BN - 1) / BN;
  const int tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x % tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const __amdgpu_buffer_rsrc_t rx = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, q.x_bytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rw = __builtin_amdgcn_make_buffer_rsrc((void *)p.w, 0, q.w_bytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rxs = __builtin_amdgcn_make_buffer_rsrc((void *)p.xs, 0, q.xs_bytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rwp = __builtin_amdgcn_make_buffer_rsrc((void *)p.wp, 0, q.wp_bytes, RSRC_FLAGS);

  // ---- per-thread gather state: chunk `ch` (8 consecutive kg) of rows row0 + RPP*i ----
  const int ts = t & (GT - 1);
  const int ch = ts % CPR, row0 = ts / CPR;
  const int wcol = (ch ^ ((row0 >> 2) & 3)) << 3;  // swizzled LDS column of the chunk
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
    const bool ok = n < p.N;
    bbase[i] = ok ? n * p.RSC * 4 : OOB;
    pbase[i] = ok ? n * p.Cs * 4 : OOB;
  }

  // the chunks of the group's next step, on their way from memory
  float4 ra[PA][2], rb[PB][2];
  // this workgroup's share of the reduction: steps [kb0, kb_end)
  const int kb0 = blockIdx.y * q.kb_per;
  const int kb_end = min(q.nkb_conv + q.nkb_proj, kb0 + q.kb_per);

  // Branch-free gather of step kb (see igemm_fwd_fast.hip): steps past the end, the padding of the
  // reduction axis, taps outside the image and rows past M or N all become an out-of-range offset
  // (top bit set), for which the hardware returns zeros.
  int offa[PA][2], offb[PB][2];
  bool is_proj = false;  // uniform: the step reads the shortcut tensor and its 1x1 filter
  auto gaddr = [&](int kb) {
    // half hf of the chunk: 4 consecutive kg inside one filter tap
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      int kg, tap, c;
      bool in;
      if constexpr (TI) {
        const int cc = (int)q.div_taps.div((uint32_t)kb);
        in = (kb < q.nkb_conv) & (kb < kb_end);
        tap = (kb - cc * (p.R * p.S)) & -(int)in;
        c = cc * BK + ch * 8 + hf * 4;
        kg = tap * p.C + c;
      } else {
        kg = kb * BK + ch * 8 + hf * 4;
        in = (kg < p.RSC) & (kb < kb_end);
        tap = (int)q.div_c.div((uint32_t)kg) & -(int)in;
        c = kg - tap * p.C;
      }
      const int r = (int)q.div_s.div((uint32_t)tap);
      const int sx = tap - r * p.S;
      const int toff = ((r * p.W + sx) * p.C + c) * 4;
      const int oob_in = in ? 0 : OOB;
#pragma unroll
      for (int i = 0; i < PA; ++i) offa[i][hf] = (abase[i] + toff) | oob_in | (((amask[i] >> tap) & 1u) ? 0 : OOB);
#pragma unroll
      for (int i = 0; i < PB; ++i) offb[i][hf] = (bbase[i] + kg * 4) | oob_in | (bbase[i] & OOB);
    }
    if constexpr (PROJ) {
      is_proj = kb >= q.nkb_conv;
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        const int cp = (kb - q.nkb_conv) * BK + ch * 8 + hf * 4;
        const int oob_p = (is_proj & (cp < p.Cs) & (kb < kb_end)) ? 0 : OOB;
#pragma unroll
        for (int i = 0; i < PA; ++i) offa[i][hf] = is_proj ? ((sbase[i] + cp * 4) | oob_p | (sbase[i] & OOB)) : offa[i][hf];
#pragma unroll
        for (int i = 0; i < PB; ++i) offb[i][hf] = is_proj ? ((pbase[i] + cp * 4) | oob_p | (pbase[i] & OOB)) : offb[i][hf];
      }
    }
  };
  // load i of the step whose offsets gaddr computed: chunk i / 2 (the A tile's first), half i % 2
  constexpr int NLD = 2 * (PA + PB);
  auto gissue = [&](int i) {
    const int c = i >> 1, hf = i & 1;
    if (PROJ && is_proj) {
      if (c < PA) ra[c][hf] = bload(rxs, offa[c][hf]);
      else rb[c - PA][hf] = bload(rwp, offb[c - PA][hf]);
    } else {
      if (c < PA) ra[c][hf] = bload(rx, offa[c][hf]);
      else rb[c - PA][hf] = bload(rw, offb[c - PA][hf]);
    }
  };
  auto gload = [&](int kb) {
    gaddr(kb);
#pragma unroll
    for (int i = 0; i < NLD; ++i) gissue(i);
  };

  // split the staged chunks into their pieces and write them to LDS buffer `buf`
  auto stage = [&]() {
#pragma unroll
    for (int i = 0; i < PA; ++i) {
      uint4 h, m, l;
      split8(ra[i][0], ra[i][1], h, m, l);
      *reinterpret_cast<uint4 *>(&As[buf][0][row0 + RPP * i][wcol]) = h;
      *reinterpret_cast<uint4 *>(&As[buf][1][row0 + RPP * i][wcol]) = m;
      *reinterpret_cast<uint4 *>(&As[buf][2][row0 + RPP * i][wcol]) = l;
    }
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      uint4 h, m, l;
      split8(rb[i][0], rb[i][1], h, m, l);
      *reinterpret_cast<uint4 *>(&Bs[buf][0][row0 + RPP * i][wcol]) = h;
      *reinterpret_cast<uint4 *>(&Bs[buf][1][row0 + RPP * i][wcol]) = m;
      *reinterpret_cast<uint4 *>(&Bs[buf][2][row0 + RPP * i][wcol]) = l;
    }
  };

  floatx16 acc[MT][NT];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < NT; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  // fragments of one slab (16 reduction steps): [slot][piece][tile], 8 bf16 each; fragment read r of
  // a slab: piece r / (MT + NT), then the A tiles, then the B tiles
  uint4 af[2][3][MT], bfr[2][3][NT];
  constexpr int NR = 3 * (MT + NT);  // fragment reads per slab
  const int rcol[2] = {((g ^ ((j >> 2) & 3)) << 3), (((2 + g) ^ ((j >> 2) & 3)) << 3)};  // swizzled column per slab
  auto lfrag1 = [&](int ks, int slot, int r) {
    const int pc = r / (MT + NT), i = r % (MT + NT);
    if (i < MT)
      af[slot][pc][i] = *reinterpret_cast<const uint4 *>(&As[buf][pc][wm * TM + i * 32 + j][rcol[ks]]);
    else
      bfr[slot][pc][i - MT] = *reinterpret_cast<const uint4 *>(&Bs[buf][pc][wn * TN + (i - MT) * 32 + j][rcol[ks]]);
  };
  // MFMA i of a slab: the piece products in the order their fragments are read (h, m, l); the
  // tiles innermost, so that MT*NT independent accumulators lie between two MFMAs on the same one
  static_assert(NP == 6 || NP == 9, "piece products");
  constexpr int NM = NP * MT * NT;  // MFMAs per slab
  auto mma1 = [&](int slot, int i) {
    constexpr int PCA[9] = {0, 0, 1, 1, 0, 2, 1, 2, 2}, PCB[9] = {0, 1, 0, 1, 2, 0, 2, 1, 2};
    const int pr = i / (MT * NT), a = (i / NT) % MT, b = i % NT;
    acc[a][b] = mfma_bf16(af[slot][PCA[pr]][a], bfr[slot][PCB[pr]][b], acc[a][b]);
  };
  // one reduction step out of the group's buffer: the fragments of the second slab are read under
  // the MFMAs of the first (one read per MFMA, nothing crosses: left alone, the scheduler moves
  // every read next to its first use to save registers).  The loads of the group's next step (its
  // registers are free since the last split; offsets computed one step ago) are issued among the
  // first MFMAs, and the offsets of the step after (`kb_after`) are computed among the last: this
  // phase is bound by the matrix pipe and has issue slots to spare, the staging phase has none.
  auto compute = [&](int kb_after) {
    // fragment reads in the order of first use: the h pieces (needed by the first four MFMAs) go
    // first and alone, so that the four waves' first MFMAs wait for 16 LDS reads, not 48; the rest
    // of this slab and all of the next follow one per MFMA
    constexpr int ORD[12] = {0, 2, 3, 1, 6, 7, 4, 5, 10, 11, 8, 9};
    static_assert(NR == 12 && NM >= 24, "read schedule");
    __builtin_amdgcn_s_setprio(3);  // the matrix pipe is what the step is sized for: this wave goes first
#pragma unroll
    for (int r = 0; r < 4; ++r) lfrag1(0, 0, ORD[r]);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < NM; ++i) {
      if (i < 8) lfrag1(0, 0, ORD[4 + i]);
      else if (i < 20) lfrag1(1, 1, ORD[i - 8]);
      mma1(0, i);
      if (i < NLD) gissue(i);
      __builtin_amdgcn_sched_barrier(0);
    }
    gaddr(kb_after);
#pragma unroll
    for (int i = 0; i < NM; ++i) mma1(1, i);
    __builtin_amdgcn_s_setprio(0);
  };

  // group g: steps kb0 + g, kb0 + g + 2, ... (steps past kb_end load zeros)
  const int nper = (kb_end - kb0 + 1) >> 1;  // steps per group
  int kb = kb0 + grp;
  gload(kb);
  if (grp == 0) stage();
  __syncthreads();
  if (grp == 1) {
    stage();
    __syncthreads();
  }
  gaddr(kb += 2);
  for (int i = 0; i < nper; ++i) {
    compute(kb += 2);
    __syncthreads();
    stage();
    __syncthreads();
  }
  if (grp == 0) __syncthreads();  // group 1 started one barrier late

  // ---- group 0 += group 1 through LDS (every fragment read is behind the last barrier), one row
  // of MFMA tiles per round: [wave of the group][accumulator element][lane] = 32 KiB of As ----
  float *red = reinterpret_cast<float *>(&As[0][0][0][0]);
#pragma unroll
  for (int a = 0; a < MT; ++a) {
    if (grp == 1) {
#pragma unroll
      for (int b = 0; b < NT; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) red[(w4 * (NT * 16) + b * 16 + e) * 64 + lane] = acc[a][b][e];
    }
    __syncthreads();
    if (grp == 0) {
#pragma unroll
      for (int b = 0; b < NT; ++b)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[a][b][e] += red[(w4 * (NT * 16) + b * 16 + e) * 64 + lane];
    }
    if (a + 1 < MT) __syncthreads();
  }
  if (grp == 1) return;

  // ---- split reduction: raw partial sums, slice blockIdx.y of out[splits][M][N] ----
  if (gridDim.y > 1) {
    float *part = p.out + (long long)blockIdx.y * p.M * p.N;
#pragma unroll
    for (int b = 0; b < NT; ++b) {
      const int n = n0 + wn * TN + b * 32 + j;
      if (n >= p.N) continue;
#pragma unroll
      for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int m = m0 + wm * TM + a * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
          if (m < p.M) part[(long long)m * p.N + n] = acc[a][b][e];
        }
    }
    return;
  }

  // ---- epilogue: bias, identity shortcut, ReLU, mask; consecutive lanes store consecutive n ----
#pragma unroll
  for (int b = 0; b < NT; ++b) {
    const int n = n0 + wn * TN + b * 32 + j;
    if (n >= p.N) continue;
    const float bias = p.bias ? p.bias[n] : 0.f;
#pragma unroll
    for (int a = 0; a < MT; ++a) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int m = m0 + wm * TM + a * 32 + 8 * (e >> 2) + 4 * g + (e & 3);
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

hipError_t launch_cfg(const FwdProblem &p, SplitAux q, bool nine, hipStream_t st) {
  constexpr int BM = 128, BN = 128, BK = 32;
  const int tiles = ((p.M + BM - 1) / BM) * ((p.N + BN - 1) / BN);
  q.nkb_conv = (p.RSC + BK - 1) / BK;
  q.nkb_proj = p.Cs ? (p.Cs + BK - 1) / BK : 0;
  q.div_taps = FastDiv(p.R * p.S);
  const int nkb = q.nkb_conv + q.nkb_proj;
  const int splits = p.ksplits > 1 ? p.ksplits : 1;
  q.kb_per = (nkb + splits - 1) / splits;
  const dim3 grid((unsigned)tiles, (unsigned)splits), block(512);
  const bool ti = p.C % BK == 0 && p.R * p.S > 1;
#define NF_LAUNCH(PROJ_, TI_)                                                                        \
  do {                                                                                               \
    if (nine) hipLaunchKernelGGL((igemm_fwd_split_kernel<PROJ_, TI_, 9>), grid, block, 0, st, p, q); \
    else hipLaunchKernelGGL((igemm_fwd_split_kernel<PROJ_, TI_, 6>), grid, block, 0, st, p, q);      \
  } while (0)
  if (ti) {
    if (q.nkb_proj) NF_LAUNCH(true, true);
    else NF_LAUNCH(false, true);
  } else {
    if (q.nkb_proj) NF_LAUNCH(true, false);
    else NF_LAUNCH(false, false);
  }
#undef NF_LAUNCH
  return hipGetLastError();
}

}  // namespace

// same operand limits as the fp32 buffer-load kernel (the caller has checked igemm_fwd_fast_applicable);
// the wide tile only: many filters and a reduction of more than five steps
bool igemm_fwd_split_applicable(const FwdProblem &p) { return p.N >= 128 && p.Kg > 160; }

hipError_t launch_igemm_fwd_split(const FwdProblem &p, bool nine, hipStream_t st, const char **kernel) {
  SplitAux q;
  const long long B = p.M / ((long long)p.Ho * p.Wo);
  q.div_c = FastDiv(p.C), q.div_s = FastDiv(p.S);
  q.x_bytes = (uint32_t)(B * p.H * p.W * p.C * 4);
  q.w_bytes = (uint32_t)((long long)p.N * p.RSC * 4);
  q.xs_bytes = p.Cs ? (uint32_t)(B * p.Hs * p.Ws * p.Cs * 4) : 0;
  q.wp_bytes = p.Cs ? (uint32_t)((long long)p.N * p.Cs * 4) : 0;
  q.nkb_conv = q.nkb_proj = 0;
  *kernel = nine ? "igemm_fwd_split9_128x128" : "igemm_fwd_split_128x128";
  return launch_cfg(p, q, nine, st);
}

}  // namespace nf
