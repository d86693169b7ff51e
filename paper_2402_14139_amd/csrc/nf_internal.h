// Internal declarations shared by the translation units of libnf (host side + kernel
// argument structs).  Nothing here is part of the public ABI (include/nf.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/nf.h"

namespace nf {

// q = n / d for 0 <= n < 2^31 by multiply-high; computed once on the host.
struct FastDiv {
  uint32_t magic, shift, d;
  FastDiv() : magic(0), shift(0), d(1) {}
  explicit FastDiv(uint32_t div) : d(div) {
    uint32_t l = 0;
    while ((1u << l) < div) ++l;  // l = ceil(log2 d)
    magic = (uint32_t)(((1ull << (31 + l)) / div) + 1ull);
    shift = 31 + l;
  }
  __host__ __device__ inline uint32_t div(uint32_t n) const {
    return (uint32_t)(((uint64_t)n * magic) >> shift);
  }
};

// ---- implicit-GEMM forward-type convolution: out[m][n] = sum_kg col(x)[m][kg] * w[n][kg] ----
// m = (img, ho, wo) row-major; kg = (r, s, c) then an optional extra tap of Cs channels read
// from xs at (ho*ss, wo*ss) with weights wp[n][c] (the 1x1 strided projection shortcut).
struct FwdProblem {
  const float *x, *w, *xs, *wp, *bias;
  const float *addsrc;  // identity shortcut [M][N] added before the ReLU (or null)
  const float *mask;    // out is zeroed where mask[m][n] <= 0 (or null)
  float *out;           // [M][N]
  int H, W, C, N, R, S, stride, pad, Ho, Wo;
  int Cs, Hs, Ws, ss;
  int relu;
  int M, RSC, Kg;
  FastDiv div_howo, div_wo;
  // > 1: the reduction is cut into this many parts and `out` is [ksplits][M][N] raw partial sums
  // (no bias, shortcut, ReLU or mask); only with a value igemm_fwd_pick_ksplits returned
  int ksplits;
  // Column sums of the finished output over groups of 16 consecutive rows, for the head's average
  // pooling (skinny 16x16x4 tiles only, see fwd_pool_partials_applicable): pool_part[r16][2][N],
  // slot 0 = the sum over rows 16*r16 .. +7 (pool_split) or .. +15 (!pool_split), slot 1 = rows +8 .. +15
  // (pool_split only).  Null: not formed.
  float *pool_part;
  int pool_split;
};
// whether launch_igemm_fwd would run `p` on a tile that can form pool_part (M a multiple of 64)
bool fwd_pool_partials_applicable(const FwdProblem &p);
// how many reduction splits a skinny forward-type contraction should use (1 = none)
int igemm_fwd_pick_ksplits(int M, int N, int Kg, int C, int taps);
// out[m][n] = act(sum_z part[z][m][n] + bias[n] + addsrc[m][n]) zeroed where mask[m][n] <= 0:
// the epilogue of a forward-type contraction whose reduction was split
hipError_t launch_fwd_finish(const float *part, int splits, long long M, int N, const float *bias,
                             const float *addsrc, const float *mask, int relu, float *out, hipStream_t st);
// `*kernel` receives a static string naming the tile configuration that was launched
hipError_t launch_igemm_fwd(const FwdProblem &p, hipStream_t st, const char **kernel);
// branch-free buffer-load variant (igemm_fwd_fast.hip); launch_igemm_fwd picks it when applicable
bool igemm_fwd_fast_applicable(const FwdProblem &p);
hipError_t launch_igemm_fwd_fast(const FwdProblem &p, hipStream_t st, const char **kernel);

// current contraction mode (nf_contraction): NF_CONTRACT_F32, NF_CONTRACT_BF16X6 or NF_CONTRACT_BF16X9
int contraction_mode();
// true between nf_prof_begin and nf_prof_end (every launch is then bracketed by a pair of events)
bool prof_active();
// fp32 contraction on the bf16 matrix cores through three-way split operands (igemm_fwd_split.hip);
// launch_igemm_fwd_fast hands over to it in the NF_CONTRACT_BF16X* modes when applicable (nine: all
// nine piece products instead of six)
bool igemm_fwd_split_applicable(const FwdProblem &p);
hipError_t launch_igemm_fwd_split(const FwdProblem &p, bool nine, hipStream_t st, const char **kernel);

// first-layer shapes (stem.hip): the whole reduction R*S*C <= 32 in one staging step, channel counts
// that are not multiples of 4; launch_igemm_fwd / launch_igemm_wgrad pick them when applicable
bool stem_fwd_applicable(const FwdProblem &p);
hipError_t launch_stem_fwd(const FwdProblem &p, hipStream_t st, const char **kernel);

// ---- implicit-GEMM weight gradient: part[z][p][q] = sum_{m in split z} d[m][p] * col(x)[m][q]
struct WgradProblem {
  const float *d, *x, *xs;
  float *part;    // [splits][P][Qld]
  float *part_b;  // [splits][P] column sums of d (bias gradient partials)
  int H, W, C, R, S, stride, pad, Ho, Wo;
  int Cs, Hs, Ws, ss;
  int P, M, RSC, Q, Qld;
  int splits, m_per_split;
  FastDiv div_howo, div_wo;
  uint32_t d_bytes, x_bytes, xs_bytes;  // filled by the launcher for the buffer-load variant
};
// chooses the tile shape for (P,Q); reports how many splits of M it wants
int wgrad_pick_splits(int P, int Q, int M);
hipError_t launch_igemm_wgrad(const WgradProblem &p, hipStream_t st, const char **kernel);
// software-pipelined buffer-load variant (igemm_wgrad_fast.hip); launch_igemm_wgrad picks it when applicable
bool igemm_wgrad_fast_applicable(const WgradProblem &p);
hipError_t launch_igemm_wgrad_fast(const WgradProblem &p, hipStream_t st, const char **kernel);
// fp32 weight gradient on the bf16 matrix cores through three-way split operands
// (igemm_wgrad_split.hip); launch_igemm_wgrad_fast hands over to it in the NF_CONTRACT_BF16X* modes
bool igemm_wgrad_split_applicable(const WgradProblem &p);
hipError_t launch_igemm_wgrad_split(const WgradProblem &p, bool nine, hipStream_t st, const char **kernel);
// 3x3 / stride 1 / pad 1 with at most 32 output channels (igemm_wgrad_small.hip): 4x4x1 MFMA with a
// sliding register window; `splits` are ranges of image rows there (any count is valid)
bool igemm_wgrad_small_applicable(const WgradProblem &p);
int igemm_wgrad_small_splits(int P, int C, int B, int H);
hipError_t launch_igemm_wgrad_small(const WgradProblem &p, hipStream_t st, const char **kernel);
// gamma_n's gradient as a job of extra workgroups (head_gamma.h): dWf = dz^T Pq, dbf = column sums of
// dz, optionally followed by the update of Wf / bf; plus the batch mean of the per-sample losses.
struct GammaJob {
  int B, F, Cls;
  const float *Pq, *dz;
  float *dWf, *dbf;
  float *Wf, *bf, *vWf, *vbf;  // parameters / momentum buffers updated in place (Wf null: no update)
  float lr, mu;
  const float *loss_n;
  float *loss_out;             // null: no batch-mean job
  int fch, nchunks, nb_w, nb_l;  // filled by gamma_job_plan
};
// fills fch / nchunks / nb_w / nb_l; returns the number of workgroups the job needs
int gamma_job_plan(GammaJob &g);

bool stem_wgrad_applicable(const WgradProblem &p);
hipError_t launch_stem_wgrad(const WgradProblem &p, hipStream_t st, const char **kernel);

// One weight gradient to finish: out0[p][q] (q < Q0, row length Q0) and out1[p][q-Q0] (row length
// Q-Q0) = sum_z part[z][p][q]; ob[p] = sum_z part_b[z][p].  w*/v* (may be null): parameters and
// momentum buffers updated in place right after, same layout as out0/out1/ob.
struct WgradReduce {
  const float *part, *part_b;
  int splits, P, Q, Qld, Q0;
  float *out0, *out1, *ob;
  float *w0, *w1, *wb, *v0, *v1, *vb;
  int ZS, main_blocks, bias_blocks, vec4, direct;  // filled by the launcher
};
struct ReduceSgd {
  WgradReduce job[2];
  int njobs;
  // tensors whose gradient is final already (update only; used when lr/mu are given)
  float *xw[2];
  const float *xg[2];
  float *xv[2];
  long long xn[2];
  int xblocks[2];  // filled by the launcher
  int nx;
  float lr, mu;
  GammaJob gamma;  // extra workgroups after the above (gamma.dWf null: none)
};
hipError_t launch_wgrad_reduce_sgd(const ReduceSgd &r, hipStream_t st);

// ---- head (Eq. 2 after the aux conv, Eq. 3) ----
struct HeadShape {
  int B, Hu, Wu, A, oh, ow, F, Cls, relu;
  int pmax;  // F_n: 0 adaptive average pool, 1 adaptive max pool
  int mse;   // loss: 0 softmax cross-entropy, 1 mean squared error against the one-hot label
};
// Pq = adaptive average pool of U.  With splits > 0, U is first formed from the raw partial sums
// part[splits][B*Hu*Wu*A] of the aux convolution: U = act(sum_z part[z] + ba) (written out).
// parg [B][F] (max pooling only): flat position h*Wu+w each pooled feature was taken from.
hipError_t launch_head_pool(const HeadShape &h, float *U, const float *part, int splits, const float *ba, float *Pq,
                            int32_t *parg, hipStream_t st);
// logits, softmax cross-entropy, dz, per-sample losses and dPq = dz * Wf
hipError_t launch_head_fc(const HeadShape &h, const float *Pq, const int32_t *labels, const float *Wf,
                          const float *bf, float *dz, float *loss_n, float *dPq, hipStream_t st);
hipError_t launch_loss_mean(const float *loss_n, int B, float *loss_out, hipStream_t st);
// forward-only head: logits (optionally stored), predicted class per sample (largest logit, lowest
// index among equal maxima) and, with labels, a 0/1 hit flag per sample
hipError_t launch_head_predict(const HeadShape &h, const float *Pq, const int32_t *labels, const float *Wf,
                               const float *bf, float *logits_out, int32_t *pred, int32_t *hit, hipStream_t st);
// *out = (accumulate ? *out : 0) + sum of the B hit flags
hipError_t launch_count_hits(const int32_t *hit, int B, int32_t *out, bool accumulate, hipStream_t st);
// Whole per-sample chain of the head in one launch, one workgroup per sample, for heads whose
// activation map is small (head_sample_applicable): F_n, gamma_n, the loss and dL/dz, dPq and the
// backward through F_n and the aux ReLU (dU).  Leaves Pq, dz, loss_n (and the max-pooling
// selection) in global memory for the batch-reducing jobs (GammaJob).  Extra workgroups re-lay the
// aux filter for the data gradient when Wa is given: WaT[k][r][s][a] = Wa[a][R-1-r][S-1-s][k].
bool head_sample_applicable(const HeadShape &h);
hipError_t launch_head_sample(const HeadShape &h, float *U, const float *part, int splits, const float *ba,
                              const int32_t *labels, const float *Wf, const float *bf, float *Pq, int32_t *parg,
                              float *dz, float *loss_n, float *dU, const float *Wa, float *WaT, int R, int S, int K,
                              hipStream_t st);
// Everything after F_n for a large activation map in one launch (head_wide_applicable: a linear
// layer of at most 16384 weights): gamma_n, loss, dL/dz, dPq recomputed per slice of a sample, dU,
// and the re-laid aux filter when Wa is given.  Reads Pq (and the max-pooling selection) left by
// launch_head_pool; leaves dz and loss_n for the batch-reducing jobs (GammaJob).
// `ppart` (or null): column sums per 16 pixels from the aux convolution's epilogue
// (FwdProblem::pool_part, head_pool_partials_applicable); then F_n is formed here as well and Pq written.
bool head_wide_applicable(const HeadShape &h);
bool head_pool_partials_applicable(const HeadShape &h);
hipError_t launch_head_wide(const HeadShape &h, const float *U, float *Pq, const float *ppart, const int32_t *labels,
                            const float *Wf, const float *bf, float *dz, float *loss_n, const int32_t *parg,
                            float *dU, const float *Wa, float *WaT, int R, int S, int K, hipStream_t st);
// one launch: dWf, dbf; dU (pool + aux ReLU backward); WaT[k][r][s][a] = Wa[a][R-1-r][S-1-s][k] when Wa
// is given; the batch-mean loss when loss_out is given
hipError_t launch_head_bwd(const HeadShape &h, const float *Pq, const float *dz, float *dWf, float *dbf,
                           const float *U, const float *dPq, float *dU, const float *Wa, float *WaT, int R, int S,
                           int K, const float *loss_n, float *loss_out, const int32_t *parg, hipStream_t st);

// ---- elementwise / data movement ----
hipError_t launch_maxpool_fwd(const float *T, float *Y, uint8_t *arg, int B, int Ho, int Wo, int K, int Hp,
                              int Wp, int pk, int ps, int pp, hipStream_t st);
hipError_t launch_maxpool_bwd(const float *dY, const float *Y, const uint8_t *arg, float *dZ, int B, int Ho,
                              int Wo, int K, int Hp, int Wp, int pk, int ps, int pp, hipStream_t st);
struct SgdTensors {
  float *w[16];
  const float *g[16];
  float *v[16];
  long long numel[16];
  int n;
  float lr, mu;
};
hipError_t launch_sgd(const SgdTensors &t, hipStream_t st);
hipError_t launch_cache_copy(const float *src, float *dst, const int32_t *src_lab, int32_t *dst_lab,
                             long long sample_elems, long long src_first, long long dst_first,
                             const long long *idx, long long capacity, int B, hipStream_t st);

}  // namespace nf
