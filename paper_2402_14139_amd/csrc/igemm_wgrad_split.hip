// Implicit-GEMM weight gradient with fp32 operands and fp32 results, contracted on the bf16 matrix
// cores (optional mode of the library; NeuroFlux, arXiv 2402.14139, gradient line of Algorithm 2:
// the same operation as igemm_wgrad_fast.hip, part[z][p][q] = sum over the rows m of split z of
// d[m][p] * col(x)[m][q]).
//
// Arithmetic as in igemm_fwd_split.hip: every operand element is cut into three bfloat16 pieces that
// sum to it exactly, six of the nine piece products are accumulated in fp32 by
// v_mfma_f32_32x32x16_bf16.
//
// Tile 128 (p) x 128 (q), 32 reduction rows per step.  The MFMA wants 8 consecutive reduction
// indices per lane, and the reduction index m is the slow axis of both operands in memory, so the
// tiles are transposed on the way into LDS: a staging thread loads 8 consecutive rows x 4 columns
// (eight 16-byte loads), and writes, per column and piece, the 8 row values as one 16-byte LDS
// word.  LDS rows are [column][32 m] as in the forward kernel (64 bytes, quarters XOR-swizzled);
// logical column c of a tile lives in LDS row (c % 4) * 32 + c / 4, so that the 16 lanes of a
// write pass (consecutive column chunks) hit consecutive LDS rows.  A wave's 64x64 block of the
// output is therefore the columns p = 4*i + (2*wm + a), q = 4*j + (2*wn + b) of the tile.
//
// 512 threads = two groups of four waves taking the reduction steps alternately, one computing
// while the other stages, as in the forward kernel; waves 0-1 of a group stage the d tile, waves
// 2-3 the im2col tile of x (row decode through a small table in LDS, one entry per reduction row).
#include "nf_internal.h"

namespace nf {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BKM = 32;                 // reduction rows staged per step
constexpr int OOB = (int)0x80000000;    // offset no buffer of < 2 GiB contains
constexpr int RSRC_FLAGS = 0x00020000;  // raw buffer, 32-bit data format

__device__ inline float4 bload(__amdgpu_buffer_rsrc_t r, int voff) {
  const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, voff, 0, 0));
  return make_float4(v.x, v.y, v.z, v.w);
}

// eight fp32 values -> their three bf16 pieces, 16 bytes per piece, element 0 lowest.
// x = h + m + l exactly: the pieces are cut by truncation, so both remainders are exact.
__device__ inline void split8(const float (&x)[8], uint4 &h, uint4 &m, uint4 &l) {
  unsigned hb[8], mb[8], lb[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    hb[e] = __float_as_uint(x[e]);
    const float r1 = x[e] - __uint_as_float(hb[e] & 0xffff0000u);
    mb[e] = __float_as_uint(r1);
    const float r2 = r1 - __uint_as_float(mb[e] & 0xffff0000u);
    lb[e] = __float_as_uint(r2);
  }
  constexpr unsigned TOP = 0x07060302u;  // upper halves of (second, first) -> one word
  h = make_uint4(__builtin_amdgcn_perm(hb[1], hb[0], TOP), __builtin_amdgcn_perm(hb[3], hb[2], TOP),
                 __builtin_amdgcn_perm(hb[5], hb[4], TOP), __builtin_amdgcn_perm(hb[7], hb[6], TOP));
  m = make_uint4(__builtin_amdgcn_perm(mb[1], mb[0], TOP), __builtin_amdgcn_perm(mb[3], mb[2], TOP),
                 __builtin_amdgcn_perm(mb[5], mb[4], TOP), __builtin_amdgcn_perm(mb[7], mb[6], TOP));
  l = make_uint4(__builtin_amdgcn_perm(lb[1], lb[0], TOP), __builtin_amdgcn_perm(lb[3], lb[2], TOP),
                 __builtin_amdgcn_perm(lb[5], lb[4], TOP), __builtin_amdgcn_perm(lb[7], lb[6], TOP));
}

__device__ inline floatx16 mfma_bf16(uint4 a, uint4 b, floatx16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// PROJ: the q axis ends with the channels of the 1x1 projection shortcut; RSC is a multiple of the
// tile width, so a tile is all filter taps or all projection channels (its source is picked per
// workgroup).
// NP: piece products per multiply-add: 6 (m*l, l*m, l*l left out) or all 9.
template <bool PROJ, int NP>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2))) void igemm_wgrad_split_kernel(WgradProblem p) {
  constexpr int BP = 128, BQ = 128;
  constexpr int MT = 2, NT = 2;  // 32x32 MFMA tiles per wave: 64x64
  constexpr int LDH = BKM;       // bf16 per LDS row: 64 bytes, quarter q stored at q ^ f(row), see the staging task

  // [operand: d, x][group][piece][LDS row][m]: 96 KiB (one array, addressed as such: LDS reached
  // through a converted pointer keeps the compiler from holding the per-thread arrays in registers)
  __shared__ __attribute__((aligned(16))) unsigned short Ts[2][2][3][128][LDH];
  __shared__ int Rt[2][4][4][BKM];  // [group][slot][field][row]: fields read as single words (broadcast reads)

  const int t = threadIdx.x;
  const int lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);
  const int grp = wave >> 2, w4 = wave & 3;
  const int buf = grp;  // the group's LDS buffer
  const int wm = w4 >> 1, wn = w4 & 1;
  const int j = lane % 32, g = lane / 32;  // row/column inside an MFMA tile, k group (8 consecutive m)

  // Workgroups are handed to the 8 XCDs (each with its own L2) round-robin by linear index.  The
  // index is re-mapped so that each XCD gets a contiguous run of (split, p-tile, q-tile) with the
  // tiles fastest: all tiles of one split read the same rows of d and x.
  const int gx = gridDim.x, gy = gridDim.y;
  const int nwg = gx * gy * (int)gridDim.z;
  const int lin = blockIdx.x + gx * (blockIdx.y + gy * blockIdx.z);
  const int per = nwg >> 3, rem = nwg & 7, xcd = lin & 7, slot = lin >> 3;
  const int log_id = xcd < rem ? xcd * (per + 1) + slot : rem * (per + 1) + (xcd - rem) * per + slot;
  const int bx = log_id % gx, byz = log_id / gx, by = byz % gy, bz = byz / gy;
  const int p0 = by * BP, q0 = bx * BQ;
  const int m_begin = bz * p.m_per_split;
  const int m_end = min(p.M, m_begin + p.m_per_split);

  // ---- staging task of this thread: 8 reduction rows (mg) x 4 columns (pc) of one operand ----
  const int ts = t & 255;
  const bool is_x = w4 >= 2;  // uniform per wave
  // (lanes along the columns: 512 contiguous bytes per row and load instruction)
  // Swizzle of the four 16-byte quarters of an LDS row, f(row) = ((row >> 1) ^ (row >> 2)) & 3: the
  // writes below go out 8 lanes = 8 consecutive rows at a time into a 128-byte window of banks and
  // want f distinct over rows of equal parity; the fragment reads go 16 consecutive rows at a time
  // into 256 bytes and want f distinct over rows that are equal mod 4.  This f gives both (counted
  // with SQ_LDS_BANK_CONFLICT per access pattern; (row >> 2) & 3 alone leaves the writes 2-way
  // conflicted, (row >> 1) & 3 alone the reads).
  const int u = ts & 127, pc = u % 32, mg = u / 32;
  const int wrow = pc;                                   // + 32 * (column within the chunk)
  const int wcol = (mg ^ (((pc >> 1) ^ (pc >> 2)) & 3)) << 3;  // swizzled LDS column of the 8 rows
  // d: columns p0 + pc*4 .. +3
  const int pcol = p0 + pc * 4;
  const int dcol_off = pcol < p.P ? pcol * 4 : OOB;
  // x: columns q0 + pc*4 .. +3, i.e. one fixed (r, s, c) or one fixed projection channel
  const int qcol = q0 + pc * 4;
  const bool tile_proj = PROJ && q0 >= p.RSC;  // uniform
  const bool is_tap = !tile_proj && qcol < p.RSC, is_proj = tile_proj && qcol < p.Q;
  int qr = 0, qs = 0, qc = 0;
  if (is_tap) {
    const int tap = qcol / p.C;
    qc = qcol - tap * p.C;
    qr = tap / p.S;
    qs = tap - qr * p.S;
  } else {
    qc = qcol - p.RSC;
  }
  const int xtap_off = ((qr * p.W + qs) * p.C + qc) * 4;

  const __amdgpu_buffer_rsrc_t rsd = __builtin_amdgcn_make_buffer_rsrc((void *)p.d, 0, p.d_bytes, RSRC_FLAGS);
  // the one source of this workgroup's x columns
  const __amdgpu_buffer_rsrc_t rsx = __builtin_amdgcn_make_buffer_rsrc(
      (void *)(tile_proj ? p.xs : p.x), 0, tile_proj ? p.xs_bytes : p.x_bytes, RSRC_FLAGS);

  float4 rd[8];  // the task's 8 rows, on their way from memory
  float bsum[4] = {0.f, 0.f, 0.f, 0.f};
  const bool do_bias = (bx == 0) && (p.part_b != nullptr);  // uniform
  const float bsel = (do_bias && !is_x) ? 1.f : 0.f;

  // The group's k-th step is global step 2*k + grp: reduction rows m_begin + 32*(2k + grp) .. +31.
  // Row table: entry r of Rt[grp][k & 3] describes row r of that step: {byte offset of its receptive
  // field's corner in x, hi0, wi0, byte offset of its pixel in the projection input}; hi0 is far
  // negative for rows past the split.  Written one step ahead of the loads that read it (four slots:
  // a slot is rewritten two barriers after its last read).
  auto rt_make = [&](int k) {
    if (ts < BKM) {
      const int m = m_begin + (2 * k + grp) * BKM + ts;
      const int img = (int)p.div_howo.div((uint32_t)m);
      const int rem2 = m - img * p.Ho * p.Wo;
      const int ho = (int)p.div_wo.div((uint32_t)rem2);
      const int wo = rem2 - ho * p.Wo;
      const int hi0 = ho * p.stride - p.pad, wi0 = wo * p.stride - p.pad;
      int4 e;
      e.x = ((img * p.H + hi0) * p.W + wi0) * p.C * 4;
      e.y = m < m_end ? hi0 : -(1 << 20);
      e.z = wi0;
      e.w = PROJ ? ((img * p.Hs + ho * p.ss) * p.Ws + wo * p.ss) * p.Cs * 4 : 0;
      Rt[grp][k & 3][0][ts] = e.x, Rt[grp][k & 3][1][ts] = e.y, Rt[grp][k & 3][2][ts] = e.z, Rt[grp][k & 3][3][ts] = e.w;
    }
  };

  // Branch-free gather of the group's k-th step: "no data here" (row past the split, tap outside
  // the image, column past P or Q) is an out-of-range offset that the hardware answers with zeros.
  int off[8];
  auto gaddr = [&](int k) {
    const int mb = m_begin + (2 * k + grp) * BKM + mg * 8;
    if (!is_x) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int m = mb + i;
        const bool ok = (m < m_end) & (dcol_off != OOB);
        off[i] = (m * p.P * 4 + dcol_off) | (ok ? 0 : OOB);
      }
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        int4 e;
        e.x = Rt[grp][k & 3][0][mg * 8 + i], e.y = Rt[grp][k & 3][1][mg * 8 + i], e.z = Rt[grp][k & 3][2][mg * 8 + i];
        e.w = PROJ ? Rt[grp][k & 3][3][mg * 8 + i] : 0;
        if (PROJ && tile_proj) {
          off[i] = (e.w + qc * 4) | ((is_proj & (e.y > -(1 << 19))) ? 0 : OOB);
        } else {
          const bool ok = is_tap & ((unsigned)(e.y + qr) < (unsigned)p.H) & ((unsigned)(e.z + qs) < (unsigned)p.W);
          off[i] = (e.x + xtap_off) | (ok ? 0 : OOB);
        }
      }
    }
  };
  auto gissue = [&](int i) { rd[i] = bload(is_x ? rsx : rsd, off[i]); };
  auto gload = [&](int k) {
    gaddr(k);
#pragma unroll
    for (int i = 0; i < 8; ++i) gissue(i);
  };

  // split the task's 32 values and write them, transposed, into the group's buffer: per column
  // and piece one 16-byte word holding the 8 rows
  auto stage = [&]() {
    const int op = is_x ? 1 : 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = e == 0 ? rd[i].x : e == 1 ? rd[i].y : e == 2 ? rd[i].z : rd[i].w;
      float cs = 0.f;
#pragma unroll
      for (int i = 0; i < 8; ++i) cs += v[i];
      bsum[e] += bsel * cs;
      uint4 h, m, l;
      split8(v, h, m, l);
      *reinterpret_cast<uint4 *>(&Ts[op][buf][0][e * 32 + wrow][wcol]) = h;
      *reinterpret_cast<uint4 *>(&Ts[op][buf][1][e * 32 + wrow][wcol]) = m;
      *reinterpret_cast<uint4 *>(&Ts[op][buf][2][e * 32 + wrow][wcol]) = l;
    }
  };

  floatx16 acc[MT][NT];
#pragma unroll
  for (int a = 0; a < MT; ++a)
#pragma unroll
    for (int b = 0; b < NT; ++b)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.f;

  // fragments of one slab (16 reduction rows): [slot][piece][tile], 8 bf16 each; fragment read r of
  // a slab: piece r / (MT + NT), then the d tiles, then the x tiles
  uint4 af[2][3][MT], bfr[2][3][NT];
  constexpr int NR = 3 * (MT + NT);
  const int fsw = ((j >> 1) ^ (j >> 2)) & 3;
  const int rcol[2] = {((g ^ fsw) << 3), (((2 + g) ^ fsw) << 3)};  // swizzled column per slab
  auto lfrag1 = [&](int ks, int slot, int r) {
    const int pcs = r / (MT + NT), i = r % (MT + NT);
    if (i < MT)
      af[slot][pcs][i] = *reinterpret_cast<const uint4 *>(&Ts[0][buf][pcs][wm * 64 + i * 32 + j][rcol[ks]]);
    else
      bfr[slot][pcs][i - MT] = *reinterpret_cast<const uint4 *>(&Ts[1][buf][pcs][wn * 64 + (i - MT) * 32 + j][rcol[ks]]);
  };
  // MFMA i of a slab: the piece products in the order their fragments are read (h, m, l); the
  // tiles innermost, so that MT*NT independent accumulators lie between two MFMAs on the same one
  static_assert(NP == 6 || NP == 9, "piece products");
  constexpr int NM = NP * MT * NT;
  auto mma1 = [&](int slot, int i) {
    constexpr int PCA[9] = {0, 0, 1, 1, 0, 2, 1, 2, 2}, PCB[9] = {0, 1, 0, 1, 2, 0, 2, 1, 2};
    const int pr = i / (MT * NT), a = (i / NT) % MT, b = i % NT;
    acc[a][b] = mfma_bf16(af[slot][PCA[pr]][a], bfr[slot][PCB[pr]][b], acc[a][b]);
  };
  // one reduction step out of the group's buffer: the fragments of the second slab are read under
  // the MFMAs of the first (one read per MFMA, nothing crosses).  The loads of the group's next step
  // (its registers are free since the last split; offsets computed one step ago) are issued among
  // the first MFMAs, and the offsets of the step after (`kafter`) are computed among the last: this
  // phase is bound by the matrix pipe and has issue slots to spare, the staging phase has none.
  auto compute = [&](int kafter) {
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
      if (i < 8) gissue(i);
      __builtin_amdgcn_sched_barrier(0);
    }
    gaddr(kafter);
#pragma unroll
    for (int i = 0; i < NM; ++i) mma1(1, i);
    __builtin_amdgcn_s_setprio(0);
  };

  // Every wave runs the same loop (compute + next loads; barrier; stage, table; barrier); group 1 runs it
  // one barrier late, so that between two barriers one group computes while the other stages.
  const int nsteps = (m_end - m_begin + BKM - 1) / BKM;
  const int nper = (nsteps + 1) >> 1;  // steps per group (rows past m_end load zeros)
  rt_make(0);
  rt_make(1);
  rt_make(2);
  __syncthreads();
  gload(0);
  if (grp == 0) stage();
  __syncthreads();
  if (grp == 1) {
    stage();
    __syncthreads();
  }
  gaddr(1);
  for (int k = 0; k < nper; ++k) {
    compute(k + 2);   // issues the loads of step k + 1; reads table slot (k + 2) & 3, written before the last barrier
    __syncthreads();
    stage();          // step k + 1
    rt_make(k + 3);   // slot (k + 3) & 3: last read in compute(k - 3)
    __syncthreads();
  }
  if (grp == 0) __syncthreads();  // group 1 started one barrier late

  // ---- group 0 += group 1 through LDS (every fragment read is behind the last barrier), one row
  // of MFMA tiles per round: [wave of the group][accumulator element][lane] = 32 KiB ----
  float *red = reinterpret_cast<float *>(&Ts[0][0][0][0][0]);
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
    __syncthreads();
  }

  // ---- store the partial tile: accumulator (a, b, e) of lane (j, g) is p = 4*row + 2*wm + a,
  // q = 4*j + 2*wn + b of the tile, row = 8*(e/4) + 4*g + e%4 ----
  if (grp == 0) {
    float *part = p.part + (long long)bz * p.P * p.Qld;
#pragma unroll
    for (int a = 0; a < MT; ++a) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = 8 * (e >> 2) + 4 * g + (e & 3);
        const int pr = p0 + 4 * row + 2 * wm + a;
        if (pr >= p.P) continue;
        const int q = q0 + 4 * j + 2 * wn;  // b = 0, 1: two consecutive q
        float *dst = part + (long long)pr * p.Qld + q;
        if (q + 1 < p.Q) {
          *reinterpret_cast<float2 *>(dst) = make_float2(acc[a][0][e], acc[a][1][e]);
        } else if (q < p.Q) {
          dst[0] = acc[a][0][e];
        }
      }
    }
  }

  // ---- bias-gradient partials: column sums of d over the split's rows = the staging threads' sums
  // over the 4 row groups of both wave groups, added in a fixed order ----
  if (do_bias) {  // uniform per workgroup
    float *redb = red;  // [group][row group][128 columns]; the accumulator exchange above is behind a barrier
    if (!is_x) {
#pragma unroll
      for (int e = 0; e < 4; ++e) redb[(grp * 4 + mg) * BP + pc * 4 + e] = bsum[e];
    }
    __syncthreads();
    if (t < BP && p0 + t < p.P) {
      float s = 0.f;
#pragma unroll
      for (int r = 0; r < 8; ++r) s += redb[r * BP + t];
      p.part_b[(long long)bz * p.P + p0 + t] = s;
    }
  }
}

}  // namespace

// the wide tile of the buffer-load kernel (the caller has checked igemm_wgrad_fast_applicable), with
// projection columns only where a tile is all taps or all projection channels
bool igemm_wgrad_split_applicable(const WgradProblem &p) {
  if (p.P <= 64 || p.P % 2 || p.Qld % 2) return false;
  if (p.Cs && p.RSC % 128) return false;
  return true;
}

hipError_t launch_igemm_wgrad_split(const WgradProblem &p0, bool nine, hipStream_t st, const char **kernel) {
  WgradProblem p = p0;
  const long long B = p.M / ((long long)p.Ho * p.Wo);
  p.d_bytes = (uint32_t)((long long)p.M * p.P * 4);
  p.x_bytes = (uint32_t)(B * p.H * p.W * p.C * 4);
  p.xs_bytes = p.Cs ? (uint32_t)(B * p.Hs * p.Ws * p.Cs * 4) : 0;
  *kernel = nine ? "igemm_wgrad_split9_128x128" : "igemm_wgrad_split_128x128";
  const dim3 grid((p.Q + 127) / 128, (p.P + 127) / 128, p.splits);
  if (p.Cs && nine)
    hipLaunchKernelGGL((igemm_wgrad_split_kernel<true, 9>), grid, dim3(512), 0, st, p);
  else if (p.Cs)
    hipLaunchKernelGGL((igemm_wgrad_split_kernel<true, 6>), grid, dim3(512), 0, st, p);
  else if (nine)
    hipLaunchKernelGGL((igemm_wgrad_split_kernel<false, 9>), grid, dim3(512), 0, st, p);
  else
    hipLaunchKernelGGL((igemm_wgrad_split_kernel<false, 6>), grid, dim3(512), 0, st, p);
  return hipGetLastError();
}

}  // namespace nf
