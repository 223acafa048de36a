// Host-only logic of the library: argument validation, sizes, status strings, Table 1, Theorem 2's condition and
// the entropy coder's code construction.  Plain C++ with no device code and no HIP call, so that it can also be
// built with the host compiler's sanitizers (tests/test_sanitizers.py).
#include <cmath>
#include <cstring>
#include <functional>
#include <queue>
#include <vector>

#include "lpc_internal.h"

namespace lpc {

namespace {
inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }
}  // namespace

lpc_status check_problem(const lpc_problem *p) {
  if (!p) return LPC_ENULL;
  if (p->n <= 0 || p->d <= 0) return LPC_ESHAPE;
  // row indices, coordinate indices and segment counters are 32-bit (the random stream's counter word too)
  if (p->n > (int64_t)0xFFFFFFFFll || p->d > (int64_t)0xFFFFFFFFll) return LPC_ESHAPE;
  if (!p->y) return LPC_ENULL;
  if (p->loss != LPC_LOSS_LOGISTIC && p->loss != LPC_LOSS_SQUARED && p->loss != LPC_LOSS_MLP_SOFTMAX)
    return LPC_EINVAL;
  if (!(p->lambda1 >= 0.0f) || !(p->lambda2 >= 0.0f)) return LPC_EINVAL;
  if (p->X) {
    if (p->row_ptr || p->col_idx || p->vals) return LPC_EINVAL;  // exactly one storage format
    if (!aligned(p->X, 4)) return LPC_ESHAPE;
    if (p->loss != LPC_LOSS_MLP_SOFTMAX && p->ldx < p->d) return LPC_ESHAPE;
  } else {
    if (!p->row_ptr || !p->col_idx || !p->vals) return LPC_ENULL;
    if (!aligned(p->col_idx, 4) || !aligned(p->vals, 4) || !aligned(p->row_ptr, 4)) return LPC_ESHAPE;
    if (p->nnz < 0 || p->nnz > (int64_t)0x7FFFFFFFll) return LPC_ESHAPE;
    if (p->loss == LPC_LOSS_MLP_SOFTMAX) return LPC_EINVAL;
  }
  if (p->loss == LPC_LOSS_MLP_SOFTMAX) {
    if (!p->mlp_dims || p->mlp_nlayers < 1) return LPC_ENULL;
    int64_t total = 0;
    for (int32_t l = 0; l < p->mlp_nlayers; ++l) {
      if (p->mlp_dims[l] <= 0 || p->mlp_dims[l + 1] <= 0) return LPC_ESHAPE;
      total += (int64_t)p->mlp_dims[l] * p->mlp_dims[l + 1] + p->mlp_dims[l + 1];
    }
    if (total != p->d || p->ldx < p->mlp_dims[0]) return LPC_ESHAPE;
  }
  return LPC_OK;
}

lpc_status check_config(const lpc_problem *p, const lpc_config *c) {
  if (!c) return LPC_ENULL;
  if (c->algo != LPC_ALGO_LPC && c->algo != LPC_ALGO_ALPC_SC && c->algo != LPC_ALGO_ALPC_GC) return LPC_EINVAL;
  if (c->N <= 0 || c->B <= 0 || c->m <= 0) return LPC_EINVAL;
  if (c->N > 0xFFFFFE) return LPC_EINVAL;
  // bits = 1 makes the denominator 2^(b-1)-1 of eq. (3) zero
  if (c->bits < 2 || (c->bits > 16 && c->bits < 32)) return LPC_EINVAL;
  if (c->clip_mode != LPC_CLIP_LAMBDA && c->clip_mode != LPC_CLIP_CSIGMA) return LPC_EINVAL;
  if (!(c->clip > 0.0f)) return LPC_EINVAL;
  if (c->clip_mode == LPC_CLIP_LAMBDA && c->clip > 1.0f) return LPC_EINVAL;  // lambda in (0,1]
  if (c->scheme != LPC_SCHEME_A && c->scheme != LPC_SCHEME_B && c->scheme != LPC_SCHEME_C) return LPC_EINVAL;
  if (!(c->eta > 0.0f)) return LPC_EINVAL;
  if ((int64_t)c->N * c->B > p->n) return LPC_EINVAL;  // Theorem 1 assumes N*B <= n
  if (c->n_full < 0 || c->n_full > p->n) return LPC_EINVAL;
  if (c->algo != LPC_ALGO_LPC && !(c->L > 0.0f)) return LPC_EINVAL;
  if (c->tau1 < 0.0f || c->tau2 < 0.0f || c->alpha < 0.0f || c->sigma < 0.0f) return LPC_EINVAL;
  if (c->tau1 + c->tau2 > 1.0f) return LPC_EINVAL;
  return LPC_OK;
}

// Canonical prefix code: symbols ordered by (length, index); the first codeword is all zeros, each next one
// is the previous plus one, shifted left when the length grows.  The table keeps every codeword bit-reversed
// so that appending it to a little-endian bit stream puts its most significant bit first.
int huffman_canonical_table(const int32_t *lens, int32_t nsym, HuffEntry *table) {
  int32_t longest = 0;
  for (int32_t k = 0; k < nsym; ++k) {
    if (lens[k] < 0 || lens[k] > 32) return -1;
    longest = lens[k] > longest ? lens[k] : longest;
    table[k] = HuffEntry{0u, 0u};
  }
  uint64_t word = 0;   // next free codeword of the current length
  int32_t cur = 0;
  for (int32_t len = 1; len <= longest; ++len)
    for (int32_t k = 0; k < nsym; ++k) {
      if (lens[k] != len) continue;
      word <<= (len - cur);
      cur = len;
      if (word >= (1ull << len)) return -1;  // Kraft's inequality violated
      uint32_t rev = 0;
      for (int32_t i = 0; i < len; ++i) rev |= (uint32_t)((word >> i) & 1ull) << (len - 1 - i);
      table[k] = HuffEntry{rev, (uint32_t)len};
      ++word;
    }
  return 0;
}

// Optimal prefix-code lengths: repeatedly join the two lightest subtrees; each join puts every leaf below it
// one level deeper.  Subtrees are kept in a min-heap of (weight, node); parents are recorded so that a leaf's
// length is its distance to the root.  A lone used symbol still needs one bit per occurrence.
uint64_t huffman_code_lengths(const uint64_t *counts, int32_t nsym, int32_t *lens) {
  using Item = std::pair<uint64_t, int32_t>;
  std::priority_queue<Item, std::vector<Item>, std::greater<Item>> heap;
  std::vector<int32_t> parent((size_t)nsym, -1);
  for (int32_t k = 0; k < nsym; ++k) {
    if (lens) lens[k] = 0;
    if (counts[k]) heap.push({counts[k], k});
  }
  if (heap.empty()) return 0;
  if (heap.size() == 1) {
    const Item only = heap.top();
    if (lens) lens[only.second] = 1;
    return only.first;
  }
  uint64_t total = 0;
  while (heap.size() > 1) {
    const Item a = heap.top(); heap.pop();
    const Item b = heap.top(); heap.pop();
    const int32_t node = (int32_t)parent.size();
    parent.push_back(-1);
    parent[(size_t)a.second] = node;
    parent[(size_t)b.second] = node;
    total += a.first + b.first;
    heap.push({a.first + b.first, node});
  }
  if (lens) {
    for (int32_t k = 0; k < nsym; ++k) {
      if (!counts[k]) continue;
      int32_t depth = 0;
      for (int32_t v = k; parent[(size_t)v] >= 0; v = parent[(size_t)v]) ++depth;
      lens[k] = depth;
    }
  }
  return total;
}

}  // namespace lpc

using namespace lpc;

extern "C" {

int64_t lpc_d_pad(int64_t d) { return (d + 31) / 32 * 32; }
int64_t lpc_words_per_msg(int64_t d, int32_t bits) { return (d + 31) / 32 * (int64_t)bits; }

const char *lpc_status_string(lpc_status s) {
  switch (s) {
    case LPC_OK: return "ok";
    case LPC_EINVAL: return "invalid argument";
    case LPC_ENULL: return "null pointer";
    case LPC_ESHAPE: return "shape, leading dimension or alignment mismatch";
    case LPC_EWORKSPACE: return "workspace missing, misaligned or too small";
    case LPC_ENONFINITE: return "non-finite value in a vector handed to the quantizer";
    case LPC_EDEVICE: return "HIP call failed";
    case LPC_EUNSUPPORTED: return "not supported by this build";
  }
  return "unknown status";
}

lpc_status lpc_theorem2_lhs(int64_t d, int32_t bits, double lambda, int64_t d_lambda, int32_t N, int32_t B,
                            int32_t m, double rho, int32_t scheme, double *out_host) {
  if (!out_host) return LPC_ENULL;
  if (bits < 2 || bits > 16 || d < 0 || d_lambda < 0 || N < 1 || B < 1 || m < 1) return LPC_EINVAL;
  if (scheme != LPC_SCHEME_A && scheme != LPC_SCHEME_B && scheme != LPC_SCHEME_C) return LPC_EINVAL;
  const double steps = (double)((1 << (bits - 1)) - 1);   // delta = lambda*|u|_inf/steps, eq. (3)
  const double rounding = (scheme == LPC_SCHEME_C ? 0.375 : 0.25) * (double)d * (lambda / steps) * (lambda / steps);
  const double clipping = (double)d_lambda * (1.0 - lambda) * (1.0 - lambda);
  const double sampling = 1.0 / ((double)N * (double)B);
  const double mr = (double)m * rho;
  *out_host = 8.0 * mr * mr * (rounding + clipping + sampling) + rho;
  return LPC_OK;
}

lpc_status lpc_bits_per_iteration(int64_t d, int32_t bits, int32_t N, int32_t scheme, uint64_t *out_host) {
  if (!out_host) return LPC_ENULL;
  if (d < 0 || N < 1 || bits < 2 || (bits > 16 && bits < 32)) return LPC_EINVAL;
  if (scheme != LPC_SCHEME_A && scheme != LPC_SCHEME_B && scheme != LPC_SCHEME_C) return LPC_EINVAL;
  const uint64_t dd = (uint64_t)d, nn = (uint64_t)N;
  if (bits >= 32) {  // quantization off: every worker sends its d floats to every other worker
    *out_host = 32ull * dd * nn * (nn - 1ull);
    return LPC_OK;
  }
  const uint64_t bd = (uint64_t)bits * dd;
  uint64_t ceil_log2 = 0;
  while ((1ull << ceil_log2) < nn) ++ceil_log2;
  if (scheme == LPC_SCHEME_A) *out_host = (32ull + bd) * nn * (nn - 1ull);            // all-to-all, message 32 + bd
  else if (scheme == LPC_SCHEME_B) *out_host = nn * (64ull + 2ull * bd + dd * ceil_log2);  // sums carry log2 N more bits
  else *out_host = nn * (64ull + 2ull * bd);                                          // re-quantized broadcast
  return LPC_OK;
}

lpc_status lpc_huffman_bits(const uint64_t *counts_host, int32_t nsym, int32_t *lens_out_host,
                            uint64_t *bits_out_host) {
  if (!counts_host || !bits_out_host) return LPC_ENULL;
  if (nsym < 1 || nsym > (1 << 16)) return LPC_EINVAL;
  *bits_out_host = huffman_code_lengths(counts_host, nsym, lens_out_host);
  return LPC_OK;
}

}  // extern "C"
