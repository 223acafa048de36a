// Multi-layer perceptron with ReLU hidden units and softmax cross-entropy --
// oracle side (test infrastructure only).
//
// The paper treats deep models as one more instance of eq. (1): f_i is the
// loss of sample i as a function of the flattened parameter vector, and the
// whole gradient vector is quantized with one scale factor (Sec. 3.2, last
// paragraph; Sec. 6.2).  The parameter vector is the concatenation, layer by
// layer, of the weight matrix W_l stored row-major as [in_l][out_l] and then
// the bias b_l [out_l].  Plain loops in double.
#include <cmath>
#include <vector>

#include "lpco.h"

namespace {

struct Shape {
  int32_t nl;
  std::vector<int64_t> dims, woff, boff;
  int64_t total;
};

bool shape_of(const lpco_problem *p, Shape &s) {
  if (!p->mlp_dims || p->mlp_nlayers < 1) return false;
  s.nl = p->mlp_nlayers;
  s.dims.assign(p->mlp_dims, p->mlp_dims + s.nl + 1);
  s.woff.resize((size_t)s.nl);
  s.boff.resize((size_t)s.nl);
  int64_t off = 0;
  for (int32_t l = 0; l < s.nl; ++l) {
    if (s.dims[(size_t)l] <= 0 || s.dims[(size_t)l + 1] <= 0) return false;
    s.woff[(size_t)l] = off; off += s.dims[(size_t)l] * s.dims[(size_t)l + 1];
    s.boff[(size_t)l] = off; off += s.dims[(size_t)l + 1];
  }
  s.total = off;
  return s.total == p->d;
}

// adds grad f_r(w) to g and returns f_r(w)
double sample_grad(const lpco_problem *p, const Shape &s, const float *w, int64_t r, double *g) {
  const int32_t nl = s.nl;
  std::vector<std::vector<double>> h((size_t)nl + 1), delta((size_t)nl + 1);
  h[0].resize((size_t)s.dims[0]);
  const float *x = p->X + r * p->ldx;
  for (int64_t k = 0; k < s.dims[0]; ++k) h[0][(size_t)k] = (double)x[k];
  for (int32_t l = 0; l < nl; ++l) {
    const int64_t in = s.dims[(size_t)l], out = s.dims[(size_t)l + 1];
    const float *W = w + s.woff[(size_t)l];
    const float *b = w + s.boff[(size_t)l];
    h[(size_t)l + 1].assign((size_t)out, 0.0);
    for (int64_t o = 0; o < out; ++o) {
      double a = (double)b[o];
      for (int64_t k = 0; k < in; ++k) a += h[(size_t)l][(size_t)k] * (double)W[k * out + o];
      h[(size_t)l + 1][(size_t)o] = (l + 1 < nl) ? (a > 0.0 ? a : 0.0) : a;  // ReLU on hidden layers
    }
  }
  // softmax cross-entropy at the class id y_r
  const int64_t C = s.dims[(size_t)nl];
  const std::vector<double> &logit = h[(size_t)nl];
  const int64_t cls = (int64_t)p->y[r];
  double mx = logit[0];
  for (int64_t o = 1; o < C; ++o) mx = logit[(size_t)o] > mx ? logit[(size_t)o] : mx;
  double sum = 0.0;
  for (int64_t o = 0; o < C; ++o) sum += std::exp(logit[(size_t)o] - mx);
  const double loss = std::log(sum) + mx - logit[(size_t)cls];
  delta[(size_t)nl].resize((size_t)C);
  for (int64_t o = 0; o < C; ++o)
    delta[(size_t)nl][(size_t)o] = std::exp(logit[(size_t)o] - mx) / sum - (o == cls ? 1.0 : 0.0);
  for (int32_t l = nl - 1; l >= 0; --l) {
    const int64_t in = s.dims[(size_t)l], out = s.dims[(size_t)l + 1];
    const float *W = w + s.woff[(size_t)l];
    double *gW = g + s.woff[(size_t)l];
    double *gb = g + s.boff[(size_t)l];
    for (int64_t o = 0; o < out; ++o) gb[o] += delta[(size_t)l + 1][(size_t)o];
    for (int64_t k = 0; k < in; ++k) {
      const double hk = h[(size_t)l][(size_t)k];
      if (hk != 0.0)
        for (int64_t o = 0; o < out; ++o) gW[k * out + o] += hk * delta[(size_t)l + 1][(size_t)o];
    }
    if (l > 0) {
      delta[(size_t)l].assign((size_t)in, 0.0);
      for (int64_t k = 0; k < in; ++k) {
        if (h[(size_t)l][(size_t)k] > 0.0) {  // ReLU derivative
          double acc = 0.0;
          for (int64_t o = 0; o < out; ++o) acc += (double)W[k * out + o] * delta[(size_t)l + 1][(size_t)o];
          delta[(size_t)l][(size_t)k] = acc;
        }
      }
    }
  }
  return loss;
}

}  // namespace

// Smallest |pre-activation| of any hidden (ReLU) unit over the given rows.  The gradient of a ReLU
// network is discontinuous where a pre-activation is zero; a float implementation may land on either
// side of such a kink, so the parity tests only demand tight agreement for batches whose margin is
// well above float rounding (and say so).
extern "C" int lpco_mlp_relu_margin(const lpco_problem *p, const float *w, const int64_t *idx, int32_t B,
                                    double *margin_out) {
  Shape s;
  if (!p || !w || !idx || !margin_out) return LPCO_ENULL;
  if (!p->X || !shape_of(p, s)) return LPCO_ESHAPE;
  double margin = 1e300;
  std::vector<double> h, hn;
  for (int32_t a = 0; a < B; ++a) {
    const float *x = p->X + idx[a] * p->ldx;
    h.assign(x, x + s.dims[0]);
    for (int32_t l = 0; l + 1 < s.nl; ++l) {
      const int64_t in = s.dims[(size_t)l], out = s.dims[(size_t)l + 1];
      const float *W = w + s.woff[(size_t)l];
      const float *b = w + s.boff[(size_t)l];
      hn.assign((size_t)out, 0.0);
      for (int64_t o = 0; o < out; ++o) {
        double acc = (double)b[o];
        for (int64_t k = 0; k < in; ++k) acc += h[(size_t)k] * (double)W[k * out + o];
        if (std::fabs(acc) < margin) margin = std::fabs(acc);
        hn[(size_t)o] = acc > 0.0 ? acc : 0.0;
      }
      h.swap(hn);
    }
  }
  *margin_out = margin;
  return LPCO_OK;
}

// mean gradient over the first n_rows samples (the snapshot pass)
int lpco_mlp_full_grad(const lpco_problem *p, const float *w, int64_t n_rows, float *mu, double *f_out) {
  Shape s;
  if (!p->X || !shape_of(p, s)) return LPCO_ESHAPE;
  std::vector<double> g((size_t)p->d, 0.0);
  double f = 0.0;
  for (int64_t r = 0; r < n_rows; ++r) f += sample_grad(p, s, w, r, g.data());
  for (int64_t j = 0; j < p->d; ++j) mu[j] = (float)(g[(size_t)j] / (double)n_rows);
  if (f_out) *f_out = f / (double)n_rows;
  return LPCO_OK;
}

// (1/B) sum over the batch of grad f_a(w), into g_out (overwritten)
int lpco_mlp_batch_grad(const lpco_problem *p, const float *w, const int64_t *idx, int32_t B, double *g_out) {
  Shape s;
  if (!p->X || !shape_of(p, s)) return LPCO_ESHAPE;
  for (int64_t j = 0; j < p->d; ++j) g_out[j] = 0.0;
  for (int32_t a = 0; a < B; ++a) sample_grad(p, s, w, idx[a], g_out);
  for (int64_t j = 0; j < p->d; ++j) g_out[j] /= (double)B;
  return LPCO_OK;
}
