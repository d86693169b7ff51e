// Weight gradient of a 3x3 / stride 1 / pad 1 convolution with FEW output channels (P <= 16):
// the auxiliary head's conv beta_n (NeuroFlux, arXiv 2402.14139, Eq. 2; gradient line of
// Algorithm 2).  G[p][r][s][c] = sum over pixels m of dU[m][p] * y[m + (r-1, s-1)][c].
//
// The tiled implicit GEMM wastes most of a 32-row MFMA tile on P = 4..16 and streams every input
// element nine times (once per tap).  Here instead:
//   - v_mfma_f32_4x4x1_f32: 16 independent 4x4 outer products per instruction.  Rows = four
//     consecutive p, the 16 blocks x 4 columns = 64 channel slots, k = ONE pixel.  No padding of P
//     beyond a multiple of 4, and since every lane works on the same pixel, the nine taps of a
//     pixel are a 3x3 window of registers that slides along the image row: three new loads per
//     pixel instead of nine.
//   - a lane owns V consecutive channels (one 4*V-byte buffer load per row of the window), so a
//     wave covers 64*V channels and G groups of four output channels: G*9*V accumulators of 4
//     registers (144 for G*V = 4: one wave per SIMD).  Group g of a workgroup's 4*G output
//     channels is {g, g+G, g+2G, g+3G}, so that the G values a lane needs of dU are consecutive:
//     four loads per pixel in all (three window rows + dU) for 36 MFMAs.  The load unit, not the
//     MFMA pipe, is what a pixel step must be sized for.  No LDS and no barrier in the main
//     loop; loads run RING-3 pixels ahead through a register ring.
//   - image rows are flattened to a stream of W+2 elements each (columns -1 .. W); stream element e
//     carries the window column of its position and the dU of pixel (row, t); a step whose pixel
//     is a halo position gets dU = 0 from an out-of-range load, so the loop has no branches.
//   - the four waves of a workgroup take different rows; their accumulators are added in a fixed
//     order through LDS; the workgroup writes one partial tile in the layout of the tiled kernel,
//     and the same reduction kernel finishes the job.
#include "nf_internal.h"

namespace nf {
namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int RSRC_FLAGS = 0x00020000;  // raw buffer, 32-bit data format

template <int V>
struct VLoad;
template <>
struct VLoad<1> {
  static __device__ inline void ld(__amdgpu_buffer_rsrc_t r, int off, float *v) {
    v[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, off, 0, 0));
  }
};
template <>
struct VLoad<2> {
  static __device__ inline void ld(__amdgpu_buffer_rsrc_t r, int off, float *v) {
    const floatx2 t = __builtin_bit_cast(floatx2, __builtin_amdgcn_raw_buffer_load_b64(r, off, 0, 0));
    v[0] = t.x, v[1] = t.y;
  }
};
template <>
struct VLoad<4> {
  static __device__ inline void ld(__amdgpu_buffer_rsrc_t r, int off, float *v) {
    const floatx4 t = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, off, 0, 0));
    v[0] = t.x, v[1] = t.y, v[2] = t.z, v[3] = t.w;
  }
};

struct SmallAux {
  int total_rows;   // B * H image rows
  int rows_per_wg;  // image rows per workgroup (split index = blockIdx.z)
};

template <int G, int V, int RING>
__global__ __launch_bounds__(256, 1) void wgrad_small_kernel(WgradProblem p, SmallAux q) {
  constexpr int NACC = G * 9 * V;              // accumulators (4 registers each) per lane
  __shared__ float4 red[2][NACC][64];          // two waves' accumulators
  __shared__ float redb[4][G][4];
  __shared__ int4 desc[4][128];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int W2 = p.W + 2;

  // this lane's channels and output-channel rows
  const int c = blockIdx.x * (64 * V) + lane * V;
  // output channels of this workgroup: pbase + g + G*i (group g, row i); lane row i = lane & 3
  const int pbase = blockIdx.y * (4 * G);
  const int lane_p = pbase + G * (lane & 3);          // first of the lane's G consecutive channels
  // P % G == 0 (launcher): a lane's G channels are all inside P or all outside

  const __amdgpu_buffer_rsrc_t rsd = __builtin_amdgcn_make_buffer_rsrc((void *)p.d, 0, p.d_bytes, RSRC_FLAGS);
  const __amdgpu_buffer_rsrc_t rsx = __builtin_amdgcn_make_buffer_rsrc((void *)p.x, 0, p.x_bytes, RSRC_FLAGS);

  // rows of this wave: a quarter of the workgroup's
  const int wg_row0 = blockIdx.z * q.rows_per_wg;
  const int wg_row1 = min(q.total_rows, wg_row0 + q.rows_per_wg);
  const int rpw = (q.rows_per_wg + 3) >> 2;
  const int row_begin = min(wg_row1, wg_row0 + wave * rpw);
  const int row_end = min(wg_row1, row_begin + rpw);
  const int L = (row_end - row_begin) * W2;  // stream elements

  // Descriptor table (per wave, in LDS): for stream element e the byte offsets of its three
  // window-row loads and of its dU load, already out of range (bit 30: operands are < 1 GiB, and
  // the sum of two such markers still is) where there is no data.  One lane decodes one element,
  // 64 elements at a time, ahead of the loads; the main loop then pays one broadcast LDS read and
  // four adds per element instead of ~60 scalar instructions -- with 8-cycle MFMAs, the
  // instructions between them are what the step time is made of.
  constexpr int OOB30 = 0x40000000;
  const int lane_xo = c < p.C ? c * 4 : OOB30;
  const int lane_do = lane_p < p.P ? lane_p * 4 : OOB30;
  auto make_desc = [&](int chunk) {  // elements [64*chunk, 64*chunk + 64)
    const int e = chunk * 64 + lane;
    const int er = e / W2, t = e - er * W2;
    const int row = row_begin + er;
    const int n = row / p.H, h = row - n * p.H;
    const bool live = e < L;
    const int col = t - 1;
    const bool col_ok = live & ((unsigned)col < (unsigned)p.W);
    const int pix = (n * p.H + h) * p.W + t;  // pixel (row, w = t)
    int4 dsc;
    dsc.x = (col_ok & (h >= 1)) ? (pix - p.W - 1) * p.C * 4 : OOB30;
    dsc.y = col_ok ? (pix - 1) * p.C * 4 : OOB30;
    dsc.z = (col_ok & (h + 1 < p.H)) ? (pix + p.W - 1) * p.C * 4 : OOB30;
    dsc.w = (live & (t < p.W)) ? pix * p.P * 4 : OOB30;
    desc[wave][e & 127] = dsc;
  };

  int cur_e = 0;  // load cursor (uniform)
  float xr[RING][3][V], dr[RING][G];
  int4 dsc_next;  // descriptor of element cur_e, read one step before its loads are issued
  auto load_elem = [&](int slot) {
    const int4 dsc = dsc_next;
    VLoad<V>::ld(rsx, dsc.x + lane_xo, xr[slot][0]);
    VLoad<V>::ld(rsx, dsc.y + lane_xo, xr[slot][1]);
    VLoad<V>::ld(rsx, dsc.z + lane_xo, xr[slot][2]);
    VLoad<G>::ld(rsd, dsc.w + lane_do, dr[slot]);
    ++cur_e;
    dsc_next = desc[wave][cur_e & 127];  // same address in every lane
  };

  floatx4 acc[G][3][3][V];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
      for (int s = 0; s < 3; ++s)
#pragma unroll
        for (int i = 0; i < V; ++i) acc[g][r][s][i] = floatx4{0.f, 0.f, 0.f, 0.f};
  float bsum[G];
#pragma unroll
  for (int g = 0; g < G; ++g) bsum[g] = 0.f;

  // prologue: descriptors of the first 64 elements, then elements 0 .. RING-2
  make_desc(0);
  dsc_next = desc[wave][0];
#pragma unroll
  for (int i = 0; i + 1 < RING; ++i) load_elem(i);

  // step j (ring slot j % RING) uses elements j, j+1, j+2 and refills the slot of element j-1
  static_assert(64 % RING == 0, "a descriptor chunk is a whole number of ring rounds");
  for (int cb = 0; cb < L; cb += 64) {
    make_desc((cb >> 6) + 1);  // the cursor runs RING-1 elements ahead: next chunk's descriptors now
    const int rounds = min(64 / RING, (L - cb + RING - 1) / RING);
    for (int rd = 0; rd < rounds; ++rd) {
#pragma unroll
      for (int i = 0; i < RING; ++i) {
        load_elem((i + RING - 1) % RING);
#pragma unroll
        for (int g = 0; g < G; ++g) {
          const float a = dr[i][g];
          bsum[g] += a;
#pragma unroll
          for (int s = 0; s < 3; ++s)
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
              for (int v = 0; v < V; ++v)
                acc[g][r][s][v] =
                    __builtin_amdgcn_mfma_f32_4x4x1f32(a, xr[(i + s) % RING][r][v], acc[g][r][s][v], 0, 0, 0);
        }
        // nothing moves across a step boundary: left alone, the scheduler sinks the loads of a
        // whole ring round behind ~180 MFMAs and the round then starts with a wait for all of them
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  // ---- add the four waves' accumulators in a fixed order, (w0 + w2) + (w1 + w3), through LDS
  // with 16-byte accesses; the last addition and the store of the partial tile are shared by
  // waves 0 and 1 (each takes half of the (group, tap) pairs; a + b == b + a exactly) ----
  constexpr int NGT = G * 9, KH = (NGT + 1) / 2;  // (group, tap) pairs; size of the first half
  // part 0: pairs [0, KH), 1: pairs [KH, NGT), 2: all
  auto in_part = [&](int gt, int part) { return part == 2 || (part == 0 ? gt < KH : gt >= KH); };
  auto put = [&](int slot, int part) {
#pragma unroll
    for (int gt = 0; gt < NGT; ++gt)
#pragma unroll
      for (int v = 0; v < V; ++v)
        if (in_part(gt, part)) {
          const floatx4 t = acc[gt / 9][(gt % 9) / 3][gt % 3][v];
          red[slot][gt * V + v][lane] = make_float4(t[0], t[1], t[2], t[3]);
        }
  };
  auto add = [&](int slot, int part) {
#pragma unroll
    for (int gt = 0; gt < NGT; ++gt)
#pragma unroll
      for (int v = 0; v < V; ++v)
        if (in_part(gt, part)) {
          const float4 t = red[slot][gt * V + v][lane];
          floatx4 &d = acc[gt / 9][(gt % 9) / 3][gt % 3][v];
          d[0] += t.x, d[1] += t.y, d[2] += t.z, d[3] += t.w;
        }
  };
  if (lane < 4) {
#pragma unroll
    for (int g = 0; g < G; ++g) redb[wave][g][lane] = bsum[g];
  }
  if (wave >= 2) put(wave - 2, 2);
  __syncthreads();
  if (wave < 2) add(wave, 2);
  __syncthreads();
  if (wave == 1) put(0, 0);
  if (wave == 0) put(1, 1);
  __syncthreads();
  if (wave >= 2) return;
  const int my_part = wave;  // wave 0 finishes the first half, wave 1 the second
  if (wave == 0) add(0, 0);
  if (wave == 1) add(1, 1);

  // ---- partial tile, layout of the tiled kernel: part[split][p][Qld], q = (r*3 + s)*C + c ----
  float *part = p.part + (long long)blockIdx.z * p.P * p.Qld;
  if (c < p.C) {
#pragma unroll
    for (int gt = 0; gt < NGT; ++gt) {
      if (!in_part(gt, my_part)) continue;
      const int g = gt / 9, r = (gt % 9) / 3, sx = gt % 3;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int pr = pbase + g + G * e;
        if (pr >= p.P) continue;
        float *dst = part + (long long)pr * p.Qld + (r * 3 + sx) * p.C + c;
        if constexpr (V == 4) {
          *reinterpret_cast<float4 *>(dst) =
              make_float4(acc[g][r][sx][0][e], acc[g][r][sx][1][e], acc[g][r][sx][2][e], acc[g][r][sx][3][e]);
        } else if constexpr (V == 2) {
          *reinterpret_cast<float2 *>(dst) = make_float2(acc[g][r][sx][0][e], acc[g][r][sx][1][e]);
        } else {
          dst[0] = acc[g][r][sx][0][e];
        }
      }
    }
  }
  if (wave != 0) return;
  // bias-gradient partials (channel chunk 0 only): lanes 0..3 hold the four rows of each group
  if (blockIdx.x == 0 && p.part_b && lane < 4) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const int pr = pbase + g + G * lane;
      if (pr < p.P)
        p.part_b[(long long)blockIdx.z * p.P + pr] =
            (redb[0][g][lane] + redb[2][g][lane]) + (redb[1][g][lane] + redb[3][g][lane]);
    }
  }
}

struct SmallShape {
  int G, V;
};
inline SmallShape small_shape(int P, int C) {
  // G*V = 4 with P % G == 0: as many channels per lane as the output-channel groups leave room for
  if (P <= 4 && C >= 256) return {1, 4};
  if (P % 2 == 0 && P <= 8 && C >= 128) return {2, 2};
  if (P % 4 == 0) return {4, 1};
  return {1, 4};
}

}  // namespace

bool igemm_wgrad_small_applicable(const WgradProblem &p) {
  // operands below 1 GiB: the kernel marks "no data" with bit 30 of a byte offset
  const long long lim = 0x3FFFFFF0ll, B = p.M / ((long long)p.Ho * p.Wo);
  if (p.R != 3 || p.S != 3 || p.stride != 1 || p.pad != 1 || p.Cs != 0) return false;
  // measured: from 32 output channels on the tiled MFMA kernel is faster (no padding left to save)
  if (p.Ho != p.H || p.Wo != p.W || p.P > 16 || p.P % 4 || p.C % 4) return false;
  if ((long long)p.M * p.P * 4 > lim || B * p.H * p.W * p.C * 4 > lim) return false;
  return true;
}

// split count (image-row ranges): about two workgroups per CU over all chunks, at least 4 image
// rows per workgroup (one per wave)
int igemm_wgrad_small_splits(int P, int C, int B, int H) {
  const SmallShape sh = small_shape(P, C);
  const int chunks = ((C + 64 * sh.V - 1) / (64 * sh.V)) * ((P + 4 * sh.G - 1) / (4 * sh.G));
  const int rows = B * H;
  int S = 256 / (chunks > 0 ? chunks : 1);  // one workgroup per CU (measured: 128 and 512 are slower)
  if (S > rows / 4) S = rows / 4;
  return S > 1 ? S : 1;
}

hipError_t launch_igemm_wgrad_small(const WgradProblem &p0, hipStream_t st, const char **kernel) {
  WgradProblem p = p0;
  const long long B = p.M / ((long long)p.Ho * p.Wo);
  p.d_bytes = (uint32_t)((long long)p.M * p.P * 4);
  p.x_bytes = (uint32_t)(B * p.H * p.W * p.C * 4);
  const SmallShape sh = small_shape(p.P, p.C);
  SmallAux q;
  q.total_rows = (int)(B * p.H);
  q.rows_per_wg = (q.total_rows + p.splits - 1) / p.splits;
  const dim3 grid((unsigned)((p.C + 64 * sh.V - 1) / (64 * sh.V)), (unsigned)((p.P + 4 * sh.G - 1) / (4 * sh.G)),
                  (unsigned)p.splits);
  *kernel = "wgrad_small_4x4";
  if (sh.V == 4)
    hipLaunchKernelGGL((wgrad_small_kernel<1, 4, 8>), grid, dim3(256), 0, st, p, q);
  else if (sh.V == 2)
    hipLaunchKernelGGL((wgrad_small_kernel<2, 2, 8>), grid, dim3(256), 0, st, p, q);
  else
    hipLaunchKernelGGL((wgrad_small_kernel<4, 1, 8>), grid, dim3(256), 0, st, p, q);
  return hipGetLastError();
}

}  // namespace nf
