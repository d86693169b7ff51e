// Profiler and Partitioner of NeuroFlux (arXiv 2402.14139, "Modules", Algorithm 1) as host
// functions of libnf (include/nf.h).  No device work: the Profiler's measurements are replaced by
// the exact number of device bytes one local step of a layer needs with this library (the caller
// owns every buffer, so the figure is known without running anything), its linear models are
// least-squares lines through that figure at the given batch sizes, and Algorithm 1 groups the
// layers into blocks from those models.  nf_select_exit is the choice of the output model
// ("Trained Output CNN"): the early exit with the best validation accuracy and, among equals, the
// fewest parameters.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdlib>

#include "../../include/nf.h"

extern "C" {

int32_t nf_layer_step_bytes(const nf_layer_desc *d, const nf_aux_desc *a, int32_t B, int32_t with_momentum,
                            size_t *out) {
  if (!d || !a || !out) return NF_ERR_NULL;
  size_t ws = 0;
  int32_t rc = nf_workspace_bytes(d, a, B, &ws);
  if (rc) return rc;
  int32_t Hp = 0, Wp = 0;
  if ((rc = nf_layer_out_dims(d, nullptr, nullptr, &Hp, &Wp))) return rc;
  const size_t f = sizeof(float);
  // parameters of theta_n, beta_n, gamma_n; their gradients; optionally their momentum buffers
  size_t params = (size_t)d->C_out * d->R * d->S * d->C_in + d->C_out;
  if (d->skip_kind == 2) params += (size_t)d->C_out * d->skip_C;
  const size_t F = (size_t)a->A * a->pool_oh * a->pool_ow;
  params += (size_t)a->A * a->R * a->S * a->C_in + a->A + (size_t)a->n_classes * F + a->n_classes;
  const size_t fixed = params * f * (with_momentum ? 3 : 2);
  // per batch: input, shortcut input, emitted activation, labels, the loss scalar, workspace
  size_t act = (size_t)B * d->C_in * d->H_in * d->W_in + (size_t)B * d->C_out * Hp * Wp;
  if (d->skip_kind) act += (size_t)B * d->skip_C * d->skip_H * d->skip_W;
  *out = fixed + act * f + (size_t)B * sizeof(int32_t) + f + ws;
  return NF_OK;
}

int32_t nf_fit_linear(int32_t n, const double *batch, const double *bytes, nf_linear_model *out) {
  if (!batch || !bytes || !out) return NF_ERR_NULL;
  if (n < 2) return NF_ERR_BAD_DESC;
  double sx = 0, sy = 0, sxx = 0, sxy = 0;
  for (int i = 0; i < n; ++i) sx += batch[i], sy += bytes[i], sxx += batch[i] * batch[i], sxy += batch[i] * bytes[i];
  const double den = n * sxx - sx * sx;
  if (!(den > 0)) return NF_ERR_BAD_DESC;  // all batch sizes equal
  out->slope = (n * sxy - sx * sy) / den;
  out->intercept = (sy - out->slope * sx) / n;
  return NF_OK;
}

int32_t nf_profile_layer(const nf_layer_desc *d, const nf_aux_desc *a, int32_t with_momentum, int32_t n,
                         const int32_t *batches, nf_linear_model *out) {
  if (!batches || !out) return NF_ERR_NULL;
  if (n < 2 || n > 64) return NF_ERR_BAD_DESC;
  double x[64], y[64];
  for (int i = 0; i < n; ++i) {
    size_t bytes = 0;
    const int32_t rc = nf_layer_step_bytes(d, a, batches[i], with_momentum, &bytes);
    if (rc) return rc;
    x[i] = (double)batches[i], y[i] = (double)bytes;
  }
  return nf_fit_linear(n, x, y, out);
}

int32_t nf_partition(int32_t n_layers, const nf_linear_model *R, double M, int32_t B_limit, double rho,
                     int32_t *layer_batch, int32_t *block_first, int32_t *block_batch, int32_t *n_blocks) {
  if (!R || !block_first || !block_batch || !n_blocks) return NF_ERR_NULL;
  if (n_layers <= 0 || B_limit <= 0 || !(rho >= 0) || !(M >= 0)) return NF_ERR_BAD_DESC;
  int32_t *b = layer_batch;
  int32_t *own = nullptr;
  if (!b) {
    own = static_cast<int32_t *>(std::malloc(sizeof(int32_t) * (size_t)n_layers));
    if (!own) return NF_ERR_DEVICE;
    b = own;
  }
  // per layer: largest batch size whose model stays within the budget, capped at the limit
  for (int l = 0; l < n_layers; ++l) {
    double t;
    if (R[l].slope > 0)
      t = std::floor((M - R[l].intercept) / R[l].slope + 1e-12);
    else
      t = R[l].intercept <= M ? (double)B_limit : 0.0;
    t = std::max(0.0, std::min(t, (double)B_limit));
    b[l] = (int32_t)t;
  }
  // Blocks are the maximal runs of consecutive layers without a cut, where a cut separates layers i
  // and i+1 exactly when |b[i+1] - b[i]| > rho * b[i]; a block takes the smallest batch size of its
  // run.  (Algorithm 1's grouping loop, stated as the partition it produces.)
  int nb = 0;
  int32_t run_min = b[0];
  block_first[0] = 0;
  for (int i = 0; i + 1 < n_layers; ++i) {
    const bool cut = std::fabs((double)b[i + 1] - (double)b[i]) > rho * (double)b[i];
    if (cut) {
      block_batch[nb++] = run_min;
      block_first[nb] = i + 1;
      run_min = b[i + 1];
    } else {
      run_min = std::min(run_min, b[i + 1]);
    }
  }
  block_batch[nb++] = run_min;
  *n_blocks = nb;
  std::free(own);
  return NF_OK;
}

int32_t nf_select_exit(int32_t n_exits, const int64_t *n_correct, const int64_t *n_params, int32_t *exit_out) {
  if (!n_correct || !n_params || !exit_out) return NF_ERR_NULL;
  if (n_exits <= 0) return NF_ERR_BAD_DESC;
  int best = 0;
  for (int e = 1; e < n_exits; ++e)
    if (n_correct[e] > n_correct[best] || (n_correct[e] == n_correct[best] && n_params[e] < n_params[best])) best = e;
  *exit_out = best;
  return NF_OK;
}

}  // extern "C"
