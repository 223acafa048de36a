// Gradient oracles, objective and proximal step for the linear models --
// oracle side (test infrastructure only).
//
// eq. (1): P(w) = (1/n) sum_i f_i(w) + h(w).  The paper names the models only
// as "linear regression" / "logistic regression"; the build fixes
//   logistic: f_i(w) = log(1 + exp(-y_i x_i'w)),  y_i in {-1,+1}
//   squared : f_i(w) = (1/2) (x_i'w - y_i)^2
//   h(w)    = lambda1 |w|_1 + (lambda2/2) |w|^2     (handled by the prox)
// Everything here accumulates in double and rounds once on output.
#include <cmath>
#include <cstring>
#include <vector>

#include "lpco.h"
#if defined(_OPENMP)
#include <omp.h>
#endif

int lpco_mlp_full_grad(const lpco_problem *p, const float *w, int64_t n_rows, float *mu, double *f_out);
int lpco_mlp_batch_grad(const lpco_problem *p, const float *w, const int64_t *idx, int32_t B, double *g_out);

namespace {

int g_threads = 1;

inline bool is_csr(const lpco_problem *p) { return p->X == nullptr; }

int check_problem(const lpco_problem *p) {
  if (!p) return LPCO_ENULL;
  if (p->n <= 0 || p->d <= 0) return LPCO_ESHAPE;
  if (!p->y) return LPCO_ENULL;
  if (p->X) {
    if (p->ldx < (p->loss == LPCO_LOSS_MLP_SOFTMAX ? (p->mlp_dims ? p->mlp_dims[0] : 0) : p->d)) return LPCO_ESHAPE;
  } else {
    if (!p->row_ptr || !p->col_idx || !p->vals) return LPCO_ENULL;
  }
  if (p->loss < 0 || p->loss > 2) return LPCO_EINVAL;
  if (p->lambda1 < 0.0f || p->lambda2 < 0.0f) return LPCO_EINVAL;
  return LPCO_OK;
}

double row_dot(const lpco_problem *p, int64_t i, const float *w) {
  double acc = 0.0;
  if (!is_csr(p)) {
    const float *x = p->X + i * p->ldx;
    for (int64_t j = 0; j < p->d; ++j) acc += (double)x[j] * (double)w[j];
  } else {
    for (int64_t e = p->row_ptr[i]; e < p->row_ptr[i + 1]; ++e) acc += (double)p->vals[e] * (double)w[p->col_idx[e]];
  }
  return acc;
}

void row_axpy(const lpco_problem *p, int64_t i, double coef, double *g) {
  if (!is_csr(p)) {
    const float *x = p->X + i * p->ldx;
    for (int64_t j = 0; j < p->d; ++j) g[j] += coef * (double)x[j];
  } else {
    for (int64_t e = p->row_ptr[i]; e < p->row_ptr[i + 1]; ++e) g[p->col_idx[e]] += coef * (double)p->vals[e];
  }
}

// f_i as a function of the margin z = x_i'w
double loss_value(int32_t loss, double z, double y) {
  if (loss == LPCO_LOSS_LOGISTIC) {
    const double t = -y * z;  // log(1 + exp(t)), stable on both sides
    return t > 0.0 ? t + std::log1p(std::exp(-t)) : std::log1p(std::exp(t));
  }
  return 0.5 * (z - y) * (z - y);
}

// d f_i / d z
double loss_slope(int32_t loss, double z, double y) {
  if (loss == LPCO_LOSS_LOGISTIC) return -y / (1.0 + std::exp(y * z));
  return z - y;
}

}  // namespace

extern "C" void lpco_set_threads(int32_t nthreads) { g_threads = nthreads > 0 ? nthreads : 1; }

// Alg. 1 step 4 (communication step 1): the snapshot gradient grad f(w) as the
// mean of the n per-sample gradients, with the margins z = Xw as by-product.
extern "C" int lpco_full_grad(const lpco_problem *p, const float *w, int64_t n_rows, float *mu, float *z,
                              double *f_out) {
  int rc = check_problem(p);
  if (rc != LPCO_OK) return rc;
  if (!w || !mu) return LPCO_ENULL;
  const int64_t n = (n_rows > 0 && n_rows < p->n) ? n_rows : p->n;
  if (p->loss == LPCO_LOSS_MLP_SOFTMAX) return lpco_mlp_full_grad(p, w, n, mu, f_out);
  const int64_t d = p->d;
  std::vector<double> g((size_t)d, 0.0);
  double fsum = 0.0;
#if defined(_OPENMP)
  if (g_threads > 1) {
    // timing aid for the cpu_baseline: rows split over threads, per-thread
    // double accumulators summed in thread order
    std::vector<std::vector<double>> part((size_t)g_threads, std::vector<double>((size_t)d, 0.0));
    std::vector<double> fpart((size_t)g_threads, 0.0);
#pragma omp parallel num_threads(g_threads)
    {
      const int tid = omp_get_thread_num();
      const int nt = omp_get_num_threads();
      const int64_t lo = n * tid / nt, hi = n * (tid + 1) / nt;
      for (int64_t i = lo; i < hi; ++i) {
        const double zi = row_dot(p, i, w);
        if (z) z[i] = (float)zi;
        fpart[(size_t)tid] += loss_value(p->loss, zi, (double)p->y[i]);
        row_axpy(p, i, loss_slope(p->loss, zi, (double)p->y[i]), part[(size_t)tid].data());
      }
    }
    for (int t = 0; t < g_threads; ++t) {
      fsum += fpart[(size_t)t];
      for (int64_t j = 0; j < d; ++j) g[(size_t)j] += part[(size_t)t][(size_t)j];
    }
  } else
#endif
  {
    for (int64_t i = 0; i < n; ++i) {
      const double zi = row_dot(p, i, w);
      if (z) z[i] = (float)zi;
      fsum += loss_value(p->loss, zi, (double)p->y[i]);
      row_axpy(p, i, loss_slope(p->loss, zi, (double)p->y[i]), g.data());
    }
  }
  for (int64_t j = 0; j < d; ++j) mu[j] = (float)(g[(size_t)j] / (double)n);
  if (f_out) *f_out = fsum / (double)n;
  return LPCO_OK;
}

// Alg. 1 step 6 / Alg. 2 steps 7 and 11:
//   u = (1/B) sum_{a in batch} [ grad f_a(w) - grad f_a(w_snap) ]
// written as in the paper: both per-sample gradients are formed and
// subtracted; nothing is cached from the snapshot pass.
extern "C" int lpco_worker_vr_grad(const lpco_problem *p, const lpco_config *c, const float *w, const float *w_snap,
                                   uint32_t epoch, uint32_t iter, uint32_t tag, int32_t worker_begin,
                                   int32_t worker_end, float *U, double *stats) {
  int rc = check_problem(p);
  if (rc != LPCO_OK) return rc;
  if (!c || !w || !w_snap || !U) return LPCO_ENULL;
  if (c->B <= 0 || c->N <= 0) return LPCO_EINVAL;
  if (tag != LPCO_TAG_BATCH && tag != LPCO_TAG_SHARED) return LPCO_EINVAL;
  if (worker_begin < 0 || worker_end < worker_begin) return LPCO_EINVAL;
  if (tag == LPCO_TAG_BATCH && worker_end > c->N) return LPCO_EINVAL;
  const int64_t d = p->d, dp = lpco_d_pad(d);
  const int32_t B = c->B;
  std::vector<int64_t> idx((size_t)B);
  std::vector<double> g((size_t)d), gs((size_t)d);
  int out_rc = LPCO_OK;
  for (int32_t i = worker_begin; i < worker_end; ++i) {
    const uint32_t stream_worker = (tag == LPCO_TAG_SHARED) ? 0xFFFFFFu : (uint32_t)i;
    rc = lpco_sample_batch(c->seed, epoch, iter, tag, stream_worker, B, p->n, idx.data());
    if (rc != LPCO_OK) return rc;
    std::fill(g.begin(), g.end(), 0.0);
    if (p->loss == LPCO_LOSS_MLP_SOFTMAX) {
      rc = lpco_mlp_batch_grad(p, w, idx.data(), B, g.data());
      if (rc != LPCO_OK) return rc;
      rc = lpco_mlp_batch_grad(p, w_snap, idx.data(), B, gs.data());
      if (rc != LPCO_OK) return rc;
      for (int64_t j = 0; j < d; ++j) g[(size_t)j] -= gs[(size_t)j];  // already divided by B
    } else {
      for (int32_t a = 0; a < B; ++a) {
        const int64_t r = idx[(size_t)a];
        const double yr = (double)p->y[r];
        const double slope_w = loss_slope(p->loss, row_dot(p, r, w), yr);
        const double slope_s = loss_slope(p->loss, row_dot(p, r, w_snap), yr);
        row_axpy(p, r, slope_w, g.data());    // + grad f_a(w)
        row_axpy(p, r, -slope_s, g.data());   // - grad f_a(w_snap)
      }
      for (int64_t j = 0; j < d; ++j) g[(size_t)j] /= (double)B;
    }
    float *u = U + (int64_t)i * dp;
    for (int64_t j = 0; j < d; ++j) u[j] = (float)g[(size_t)j];
    for (int64_t j = d; j < dp; ++j) u[j] = 0.0f;
    if (stats) {
      if (lpco_vector_stats(u, d, stats + 4 * (int64_t)i) == LPCO_ENONFINITE) out_rc = LPCO_ENONFINITE;
    }
    if (tag == LPCO_TAG_SHARED) break;  // one shared batch only
  }
  return out_rc;
}

// Sec. 3.3: prox_{step*h}(p) = argmin_y h(y) + |y - p|^2 / (2*step).  For
// h = lambda1|.|_1 + (lambda2/2)|.|^2 the minimiser is separable:
// soft-threshold by step*lambda1, then shrink by 1/(1 + step*lambda2).
// Alg. 1 steps 9-10: v = u_avg + mu (mu is added after averaging and is never
// quantized), w <- prox(w - step*v).
extern "C" int lpco_prox_step(int64_t d, float *w, const float *u_avg, const float *mu, float step, float lambda1,
                              float lambda2) {
  if (!w || !u_avg || !mu) return LPCO_ENULL;
  if (d <= 0 || !(step > 0.0f) || lambda1 < 0.0f || lambda2 < 0.0f) return LPCO_EINVAL;
  const double thr = (double)step * (double)lambda1;
  const double shrink = 1.0 / (1.0 + (double)step * (double)lambda2);
  for (int64_t j = 0; j < d; ++j) {
    const double v = (double)u_avg[j] + (double)mu[j];
    const double pt = (double)w[j] - (double)step * v;
    const double mag = std::fabs(pt) - thr;
    const double out = mag > 0.0 ? (pt > 0.0 ? mag : -mag) * shrink : 0.0;
    w[j] = (float)out;
  }
  return LPCO_OK;
}

extern "C" int lpco_objective(const lpco_problem *p, const float *w, double *P_out) {
  int rc = check_problem(p);
  if (rc != LPCO_OK) return rc;
  if (!w || !P_out) return LPCO_ENULL;
  double f = 0.0;
  if (p->loss == LPCO_LOSS_MLP_SOFTMAX) {
    std::vector<float> tmp((size_t)p->d);
    rc = lpco_mlp_full_grad(p, w, p->n, tmp.data(), &f);
    if (rc != LPCO_OK) return rc;
  } else {
    for (int64_t i = 0; i < p->n; ++i) f += loss_value(p->loss, row_dot(p, i, w), (double)p->y[i]);
    f /= (double)p->n;
  }
  double l1 = 0.0, l2 = 0.0;
  for (int64_t j = 0; j < p->d; ++j) {
    l1 += std::fabs((double)w[j]);
    l2 += (double)w[j] * (double)w[j];
  }
  *P_out = f + (double)p->lambda1 * l1 + 0.5 * (double)p->lambda2 * l2;
  return LPCO_OK;
}

// Convergence metric for nonconvex / nonsmooth problems (Sec. 3.3): the gradient mapping
//   G_eta(x) = (1/eta) [ x - prox_{eta h}(x - eta grad f(x)) ];  returns |G_eta(x)|^2.
extern "C" int lpco_gradient_mapping(const lpco_problem *p, const float *w, float eta, double *gm2_out) {
  int rc = check_problem(p);
  if (rc != LPCO_OK) return rc;
  if (!w || !gm2_out) return LPCO_ENULL;
  if (!(eta > 0.0f)) return LPCO_EINVAL;
  std::vector<float> mu((size_t)p->d);
  rc = lpco_full_grad(p, w, 0, mu.data(), nullptr, nullptr);
  if (rc != LPCO_OK) return rc;
  const double thr = (double)eta * (double)p->lambda1, shrink = 1.0 / (1.0 + (double)eta * (double)p->lambda2);
  double acc = 0.0;
  for (int64_t j = 0; j < p->d; ++j) {
    const double pt = (double)w[j] - (double)eta * (double)mu[j];
    const double mag = std::fabs(pt) - thr;
    const double px = mag > 0.0 ? (pt > 0.0 ? mag : -mag) * shrink : 0.0;
    const double g = ((double)w[j] - px) / (double)eta;
    acc += g * g;
  }
  *gm2_out = acc;
  return LPCO_OK;
}

// Left-hand side of the step-size conditions of Theorem 2 (eq. (6) for schemes (a)/(b), eq. (7) for (c)):
//   8 m^2 rho^2 [ c * d lambda^2/(2^(b-1)-1)^2 + d_lambda (1-lambda)^2 + 1/(N B) ] + rho,  c = 1/4 or 3/8.
// The theorem asks for a value <= 1 (and rho < 1/2).
extern "C" double lpco_theorem2_lhs(int64_t d, int32_t bits, double lambda, int64_t d_lambda, int32_t N, int32_t B,
                                    int32_t m, double rho, int32_t scheme) {
  const double levels = (double)((1 << (bits - 1)) - 1);
  const double c = scheme == LPCO_SCHEME_C ? 3.0 / 8.0 : 1.0 / 4.0;
  const double bracket = c * (double)d * lambda * lambda / (levels * levels) +
                         (double)d_lambda * (1.0 - lambda) * (1.0 - lambda) + 1.0 / ((double)N * (double)B);
  return 8.0 * (double)m * (double)m * rho * rho * bracket + rho;
}
