// The optimizer loops -- oracle side (test infrastructure only).
//
// Alg. 1 (LPC-SVRG), Alg. 2 (ALPC-SVRG, strongly convex) and Alg. 3
// (ALPC-SVRG, general convex), one epoch per call, every step taken in the
// order of the paper's listings with the helper oracles of this directory.
#include <cmath>
#include <cstring>
#include <vector>

#include "lpco.h"

namespace {

// zeta of Theorem 3 with d_lambda = 0
double zeta_no_clip(const lpco_problem *p, const lpco_config *c) {
  double z = 1.0 / ((double)c->N * (double)c->B);
  if (c->bits < 32) {
    const double lam = (c->clip_mode == LPCO_CLIP_LAMBDA) ? (double)c->clip : 1.0;
    const double levels = (double)((1 << (c->bits - 1)) - 1);
    z += (double)p->d * lam * lam / (4.0 * levels * levels);
  }
  return z;
}

// communication step 2 for one iteration: U (N x d_pad) -> u_avg (d)
int exchange(const lpco_problem *p, const lpco_config *c, uint32_t epoch, uint32_t iter, const float *U,
             const double *stats, float *u_avg, std::vector<uint32_t> &packed, std::vector<float> &delta,
             std::vector<uint32_t> &nclip) {
  const int64_t d = p->d;
  if (c->bits >= 32) {  // quantization off: nothing is scaled or clipped
    for (int32_t i = 0; i < c->N; ++i) { delta[(size_t)i] = 0.0f; nclip[(size_t)i] = 0u; }
    return lpco_plain_avg(d, c->N, U, u_avg);
  }
  int rc;
  if (c->scheme == LPCO_SCHEME_A) {
    rc = lpco_quantize_clip(d, c->N, c->bits, c->clip_mode, c->clip, c->seed, epoch, iter, U, stats, nullptr,
                            packed.data(), delta.data(), nclip.data());
    if (rc != LPCO_OK) return rc;
    return lpco_dequantize_avg(d, c->N, c->bits, packed.data(), delta.data(), u_avg);
  }
  // schemes (b), (c): unify delta = max_i delta_i, then every worker quantizes with it
  float dmax = 0.0f;
  for (int32_t i = 0; i < c->N; ++i) {
    float di, th;
    rc = lpco_delta_from_stats(stats + 4 * (int64_t)i, d, c->bits, c->clip_mode, c->clip, &di, &th);
    if (rc != LPCO_OK) return rc;
    if (di > dmax) dmax = di;
  }
  std::vector<float> shared((size_t)c->N, dmax);
  rc = lpco_quantize_clip(d, c->N, c->bits, c->clip_mode, c->clip, c->seed, epoch, iter, U, stats, shared.data(),
                          packed.data(), delta.data(), nclip.data());
  if (rc != LPCO_OK) return rc;
  return lpco_dequantize_shared(d, c->N, c->bits, packed.data(), delta[0], c->scheme == LPCO_SCHEME_C ? 1 : 0,
                                c->seed, epoch, iter, u_avg, nullptr);
}

}  // namespace

// Parameter rules: Theorem 3 (alpha = 1/(6 tau1 L), tau1 = sqrt(m sigma/(6L)),
// tau2 = 5 zeta/3 + 1/(2B) <= 1/2) for Alg. 2; Alg. 3 step 3
// (tau1_s = 2/(s+4), alpha_s = 1/(6 L tau1_s)).  A non-zero field of the config
// overrides the rule; for Alg. 3 a non-zero alpha is the experiments' "learning
// rate", alpha_s = alpha / tau1_s (Sec. 6.1).
extern "C" int lpco_alpc_params(const lpco_problem *p, const lpco_config *c, uint32_t epoch, float *tau1,
                                float *tau2, float *alpha, float *theta) {
  if (!p || !c || !tau1 || !tau2 || !alpha || !theta) return LPCO_ENULL;
  if (!(c->L > 0.0f)) return LPCO_EINVAL;
  const double L = (double)c->L;
  const double sigma = c->sigma > 0.0f ? (double)c->sigma : (double)p->lambda2;
  double t2 = c->tau2 > 0.0f ? (double)c->tau2 : 5.0 * zeta_no_clip(p, c) / 3.0 + 1.0 / (2.0 * (double)c->B);
  if (t2 > 0.5) t2 = 0.5;
  double t1, a, th;
  if (c->algo == LPCO_ALGO_ALPC_SC) {
    t1 = c->tau1 > 0.0f ? (double)c->tau1 : std::sqrt((double)c->m * sigma / (6.0 * L));
    if (t1 > 0.5) t1 = 0.5;
    if (!(t1 > 0.0)) return LPCO_EINVAL;
    a = c->alpha > 0.0f ? (double)c->alpha : 1.0 / (6.0 * t1 * L);
    th = 1.0 + a * sigma;
  } else if (c->algo == LPCO_ALGO_ALPC_GC) {
    t1 = 2.0 / ((double)epoch + 4.0);
    a = c->alpha > 0.0f ? (double)c->alpha / t1 : 1.0 / (6.0 * L * t1);
    th = 1.0;
  } else {
    return LPCO_EINVAL;
  }
  *tau1 = (float)t1; *tau2 = (float)t2; *alpha = (float)a; *theta = (float)th;
  return LPCO_OK;
}

namespace {

// One epoch; delta_trace / nclip_trace / coded_trace ([m][N], may be NULL) receive, per inner iteration t and
// worker i, the scale factor delta_t^i the worker quantized with, its number of clipped coordinates d_lambda
// (Sec. 3.2) and the size in bits of the message's d codes after entropy coding (Sec. 6.1; 32*d with
// quantization off).
int epoch_impl(const lpco_problem *p, const lpco_config *c, float *w_snap, float *y, float *zacc, uint32_t epoch,
               uint64_t *bits_sent, float *delta_trace, uint32_t *nclip_trace, uint64_t *coded_trace) {
  if (!p || !c || !w_snap) return LPCO_ENULL;
  if (c->N <= 0 || c->B <= 0 || c->m <= 0) return LPCO_EINVAL;
  if (c->bits < 2 || (c->bits > 16 && c->bits < 32)) return LPCO_EINVAL;
  const int64_t d = p->d, dp = lpco_d_pad(d);
  const int32_t N = c->N;
  const bool quant = c->bits < 32;
  std::vector<float> mu((size_t)d), U((size_t)N * (size_t)dp), u_avg((size_t)d), w((size_t)d);
  std::vector<double> stats((size_t)N * 4);
  std::vector<uint32_t> packed(quant ? (size_t)N * (size_t)lpco_words_per_msg(d, c->bits) : 1);
  std::vector<float> delta((size_t)N);
  std::vector<uint32_t> nclip((size_t)N);
  auto record = [&](int32_t t) {
    for (int32_t i = 0; i < N; ++i) {
      if (delta_trace) delta_trace[(size_t)t * (size_t)N + (size_t)i] = delta[(size_t)i];
      if (nclip_trace) nclip_trace[(size_t)t * (size_t)N + (size_t)i] = nclip[(size_t)i];
      if (coded_trace) {
        uint64_t size = 32ull * (uint64_t)d;
        if (quant) {
          std::vector<uint64_t> counts((size_t)1 << c->bits);
          lpco_code_histogram(packed.data() + (size_t)i * (size_t)lpco_words_per_msg(d, c->bits), d, c->bits,
                              counts.data());
          size = lpco_huffman_bits(counts.data(), 1 << c->bits, nullptr);
        }
        coded_trace[(size_t)t * (size_t)N + (size_t)i] = size;
      }
    }
  };
  uint64_t bits = 0;

  // communication step 1: grad f at the snapshot, full precision
  int rc = lpco_full_grad(p, w_snap, c->n_full, mu.data(), nullptr, nullptr);
  if (rc != LPCO_OK) return rc;

  if (c->algo == LPCO_ALGO_LPC) {
    std::memcpy(w.data(), w_snap, sizeof(float) * (size_t)d);  // x_0 = x~
    for (int32_t t = 0; t < c->m; ++t) {
      rc = lpco_worker_vr_grad(p, c, w.data(), w_snap, epoch, (uint32_t)t, LPCO_TAG_BATCH, 0, N, U.data(),
                               stats.data());
      if (rc != LPCO_OK) return rc;
      rc = exchange(p, c, epoch, (uint32_t)t, U.data(), stats.data(), u_avg.data(), packed, delta, nclip);
      if (rc != LPCO_OK) return rc;
      record(t);
      bits += quant ? lpco_bits_per_iteration(d, c->bits, N, c->scheme) : 32ull * d * N * (N - 1);
      // v = u_avg + mu ; x <- prox_{eta h}(x - eta v)
      rc = lpco_prox_step(d, w.data(), u_avg.data(), mu.data(), c->eta, p->lambda1, p->lambda2);
      if (rc != LPCO_OK) return rc;
    }
    std::memcpy(w_snap, w.data(), sizeof(float) * (size_t)d);  // x~ <- x_m
    if (bits_sent) *bits_sent = bits;
    return LPCO_OK;
  }

  // ---- ALPC-SVRG (Alg. 2 / Alg. 3) ----
  if (!y || !zacc) return LPCO_ENULL;
  float tau1, tau2, alpha, theta;
  rc = lpco_alpc_params(p, c, epoch, &tau1, &tau2, &alpha, &theta);
  if (rc != LPCO_OK) return rc;
  const float step_y = (float)(1.0 / (4.0 * (double)c->L));
  std::vector<float> x((size_t)d), uhat((size_t)dp), ynew((size_t)d);
  std::vector<double> ysum((size_t)d, 0.0);
  double wsum = 0.0, wt = 1.0;
  const double c1 = (double)tau1, c2 = (double)tau2, c3 = 1.0 - (double)tau1 - (double)tau2;
  for (int32_t t = 0; t < c->m; ++t) {
    // x_{k+1} = tau1 z_k + tau2 x~ + (1 - tau1 - tau2) y_k
    for (int64_t j = 0; j < d; ++j)
      x[(size_t)j] = (float)(c1 * (double)zacc[j] + c2 * (double)w_snap[j] + c3 * (double)y[j]);
    // low-precision gradient v = Q-average + mu
    rc = lpco_worker_vr_grad(p, c, x.data(), w_snap, epoch, (uint32_t)t, LPCO_TAG_BATCH, 0, N, U.data(),
                             stats.data());
    if (rc != LPCO_OK) return rc;
    rc = exchange(p, c, epoch, (uint32_t)t, U.data(), stats.data(), u_avg.data(), packed, delta, nclip);
    if (rc != LPCO_OK) return rc;
    record(t);
    bits += quant ? lpco_bits_per_iteration(d, c->bits, N, c->scheme) : 32ull * d * N * (N - 1);
    // double sampling: shared batch J, full precision, never communicated
    rc = lpco_worker_vr_grad(p, c, x.data(), w_snap, epoch, (uint32_t)t, LPCO_TAG_SHARED, 0, 1, uhat.data(),
                             nullptr);
    if (rc != LPCO_OK) return rc;
    // y_{k+1} = argmin 2L|y - x|^2 + <v, y> + h(y) = prox_{h/(4L)}(x - v/(4L))
    std::memcpy(ynew.data(), x.data(), sizeof(float) * (size_t)d);
    rc = lpco_prox_step(d, ynew.data(), u_avg.data(), mu.data(), step_y, p->lambda1, p->lambda2);
    if (rc != LPCO_OK) return rc;
    // z_{k+1} = argmin |z - z_k|^2/(2 alpha) + <v^, z> + h(z) = prox_{alpha h}(z_k - alpha v^)
    rc = lpco_prox_step(d, zacc, uhat.data(), mu.data(), alpha, p->lambda1, p->lambda2);
    if (rc != LPCO_OK) return rc;
    std::memcpy(y, ynew.data(), sizeof(float) * (size_t)d);
    // snapshot weights theta^t (Alg. 2 step 15; theta = 1 gives Alg. 3 step 5)
    for (int64_t j = 0; j < d; ++j) ysum[(size_t)j] += wt * (double)y[j];
    wsum += wt;
    wt *= (double)theta;
  }
  for (int64_t j = 0; j < d; ++j) w_snap[j] = (float)(ysum[(size_t)j] / wsum);
  if (bits_sent) *bits_sent = bits;
  return LPCO_OK;
}

}  // namespace

extern "C" int lpco_epoch(const lpco_problem *p, const lpco_config *c, float *w_snap, float *y, float *zacc,
                          uint32_t epoch, uint64_t *bits_sent) {
  return epoch_impl(p, c, w_snap, y, zacc, epoch, bits_sent, nullptr, nullptr, nullptr);
}

extern "C" int lpco_epoch_traced(const lpco_problem *p, const lpco_config *c, float *w_snap, float *y, float *zacc,
                                 uint32_t epoch, float *delta_trace, uint32_t *nclip_trace, uint64_t *coded_trace) {
  return epoch_impl(p, c, w_snap, y, zacc, epoch, nullptr, delta_trace, nclip_trace, coded_trace);
}
