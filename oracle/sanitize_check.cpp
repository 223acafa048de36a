// Driver for a sanitizer build of the oracle (g++ -fsanitize=address,undefined): walks every entry point of
// lpco.h over small, ragged inputs, so that an out-of-bounds access, a signed overflow or a misaligned access in
// the checker itself shows up as a sanitizer report.  Test infrastructure only (tests/test_sanitizers.py builds
// and runs it); results are checked elsewhere, here only a few invariants that keep the calls honest.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "lpco.h"

#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      std::exit(1);                                                        \
    }                                                                      \
  } while (0)

static uint32_t rng_state = 12345u;
static float rnd() {  // small deterministic generator for inputs (not the method's stream)
  rng_state = rng_state * 1664525u + 1013904223u;
  return ((float)(rng_state >> 8) / 8388608.0f) - 1.0f;
}

static void quantizer_round_trip() {
  for (int bits = 2; bits <= 16; ++bits) {
    for (int64_t d : {1, 31, 32, 33, 100, 257}) {
      const int N = 3;
      const int64_t dp = lpco_d_pad(d), W = lpco_words_per_msg(d, bits);
      std::vector<float> U((size_t)(N * dp), 0.0f), delta((size_t)N), avg((size_t)d);
      for (int i = 0; i < N; ++i)
        for (int64_t j = 0; j < d; ++j) U[(size_t)(i * dp + j)] = rnd() * (float)(i + 1);
      for (int64_t j = 0; j < d; ++j) U[(size_t)j] = 0.0f;  // worker 0: the all-zero vector
      std::vector<uint32_t> packed((size_t)(N * W)), nclip((size_t)N);
      for (int mode = 0; mode < 2; ++mode) {
        CHECK(lpco_quantize_clip(d, N, bits, mode, mode ? 2.0f : 0.9f, 7, 1, 2, U.data(), nullptr, nullptr, packed.data(),
                                 delta.data(), nclip.data()) == LPCO_OK);
        CHECK(delta[0] == 0.0f);
        CHECK(lpco_dequantize_avg(d, N, bits, packed.data(), delta.data(), avg.data()) == LPCO_OK);
        std::vector<int32_t> codes((size_t)d), sums((size_t)d);
        CHECK(lpco_unpack(packed.data() + W, d, bits, codes.data()) == LPCO_OK);
        std::vector<uint32_t> again((size_t)W);
        CHECK(lpco_pack(codes.data(), d, bits, again.data()) == LPCO_OK);
        for (int64_t k = 0; k < W; ++k) CHECK(again[(size_t)k] == packed[(size_t)(W + k)]);
        CHECK(lpco_dequantize_shared(d, N, bits, packed.data(), delta[1], 1, 7, 1, 2, avg.data(), sums.data()) == LPCO_OK);
        // entropy coding of one message and its inverse
        std::vector<uint64_t> counts((size_t)1 << bits);
        CHECK(lpco_code_histogram(packed.data() + W, d, bits, counts.data()) == LPCO_OK);
        std::vector<int32_t> lens((size_t)1 << bits);
        const uint64_t total = lpco_huffman_bits(counts.data(), 1 << bits, lens.data());
        std::vector<uint32_t> stream((size_t)(total / 32 + 2));
        uint64_t got = 0;
        CHECK(lpco_huffman_encode(packed.data() + W, d, bits, lens.data(), stream.data(), (int64_t)stream.size(), &got) ==
              LPCO_OK);
        CHECK(got == total);
        std::vector<int32_t> back((size_t)d);
        CHECK(lpco_huffman_decode(stream.data(), total, d, bits, lens.data(), back.data()) == LPCO_OK);
        for (int64_t j = 0; j < d; ++j) CHECK(back[(size_t)j] == codes[(size_t)j]);
      }
    }
  }
}

static void epochs(int loss, bool csr, int algo, int bits, int scheme) {
  const int64_t n = 37, d = csr ? 45 : 19;
  std::vector<float> X, vals, y((size_t)n), w((size_t)d, 0.0f), yy((size_t)d, 0.0f), zz((size_t)d, 0.0f);
  std::vector<int32_t> row_ptr, col_idx;
  lpco_problem p{};
  p.n = n; p.d = d; p.loss = loss; p.lambda1 = 1e-3f; p.lambda2 = 1e-2f;
  for (int64_t r = 0; r < n; ++r) y[(size_t)r] = loss == LPCO_LOSS_SQUARED ? rnd() : (rnd() > 0 ? 1.0f : -1.0f);
  if (csr) {
    row_ptr.push_back(0);
    for (int64_t r = 0; r < n; ++r) {
      for (int32_t c = (int32_t)(r % 3); c < d; c += 1 + (int32_t)(r % 7)) { col_idx.push_back(c); vals.push_back(rnd()); }
      row_ptr.push_back((int32_t)col_idx.size());
    }
    p.row_ptr = row_ptr.data(); p.col_idx = col_idx.data(); p.vals = vals.data(); p.nnz = (int64_t)vals.size();
  } else {
    X.resize((size_t)(n * d));
    for (auto &v : X) v = rnd();
    p.X = X.data(); p.ldx = d;
  }
  p.y = y.data();
  lpco_config c{};
  c.algo = algo; c.N = 3; c.B = 4; c.m = 3; c.bits = bits; c.clip_mode = LPCO_CLIP_LAMBDA; c.clip = 0.9f;
  c.scheme = scheme; c.eta = 0.05f; c.L = 4.0f; c.tau2 = 0.5f; c.seed = 11; c.n_full = csr ? 30 : 0;
  std::vector<float> dtr((size_t)(c.m * c.N));
  std::vector<uint32_t> ntr((size_t)(c.m * c.N));
  std::vector<uint64_t> ctr((size_t)(c.m * c.N));
  uint64_t sent = 0;
  for (uint32_t s = 0; s < 2; ++s) {
    CHECK(lpco_epoch(&p, &c, w.data(), yy.data(), zz.data(), s, &sent) == LPCO_OK);
    CHECK(lpco_epoch_traced(&p, &c, w.data(), yy.data(), zz.data(), s + 2, dtr.data(), ntr.data(),
                            bits < 32 ? ctr.data() : nullptr) == LPCO_OK);
  }
  double P = 0.0, gm = 0.0;
  CHECK(lpco_objective(&p, w.data(), &P) == LPCO_OK && std::isfinite(P));
  CHECK(lpco_gradient_mapping(&p, w.data(), 0.1f, &gm) == LPCO_OK && gm >= 0.0);
  std::vector<float> mu((size_t)d), zrow((size_t)n);
  double f = 0.0;
  CHECK(lpco_full_grad(&p, w.data(), 0, mu.data(), zrow.data(), &f) == LPCO_OK);
  lpco_set_threads(3);
  CHECK(lpco_full_grad(&p, w.data(), 20, mu.data(), nullptr, nullptr) == LPCO_OK);
  lpco_set_threads(1);
}

static void mlp() {
  const int32_t dims[4] = {5, 4, 3, 3};
  const int64_t n = 12, d = 5 * 4 + 4 + 4 * 3 + 3 + 3 * 3 + 3;
  std::vector<float> X((size_t)(n * 5)), y((size_t)n), w((size_t)d), ws((size_t)d);
  for (auto &v : X) v = rnd();
  for (int64_t r = 0; r < n; ++r) y[(size_t)r] = (float)(r % 3);
  for (int64_t j = 0; j < d; ++j) { w[(size_t)j] = 0.5f * rnd(); ws[(size_t)j] = w[(size_t)j] + 0.05f * rnd(); }
  lpco_problem p{};
  p.n = n; p.d = d; p.loss = LPCO_LOSS_MLP_SOFTMAX; p.X = X.data(); p.ldx = 5; p.y = y.data(); p.mlp_dims = dims;
  p.mlp_nlayers = 3;
  lpco_config c{};
  c.N = 2; c.B = 3; c.m = 2; c.bits = 4; c.clip = 0.85f; c.eta = 0.05f; c.seed = 5;
  const int64_t dp = lpco_d_pad(d);
  std::vector<float> U((size_t)(2 * dp));
  std::vector<double> stats(8);
  CHECK(lpco_worker_vr_grad(&p, &c, w.data(), ws.data(), 0, 1, LPCO_TAG_BATCH, 0, 2, U.data(), stats.data()) == LPCO_OK);
  CHECK(lpco_worker_vr_grad(&p, &c, w.data(), ws.data(), 0, 1, LPCO_TAG_SHARED, 0, 1, U.data(), stats.data()) == LPCO_OK);
  int64_t idx[3];
  CHECK(lpco_sample_batch(5, 0, 1, LPCO_TAG_BATCH, 1, 3, n, idx) == LPCO_OK);
  double margin = 0.0;
  CHECK(lpco_mlp_relu_margin(&p, w.data(), idx, 3, &margin) == LPCO_OK && margin >= 0.0);
  CHECK(lpco_epoch(&p, &c, w.data(), nullptr, nullptr, 0, nullptr) == LPCO_OK);
}

int main() {
  uint32_t ctr[4] = {0, 0, 0, 0}, key[2] = {0, 0}, out[4];
  lpco_philox4x32_10(ctr, key, out);
  CHECK(out[0] == 0x6627e8d5u);  // published known-answer vector of Philox4x32-10 for the all-zero input
  quantizer_round_trip();
  for (int bits : {2, 5, 32})
    for (int scheme = 0; scheme < 3; ++scheme) {
      epochs(LPCO_LOSS_LOGISTIC, false, LPCO_ALGO_LPC, bits, scheme);
      epochs(LPCO_LOSS_LOGISTIC, true, LPCO_ALGO_LPC, bits, scheme);
      epochs(LPCO_LOSS_SQUARED, false, LPCO_ALGO_ALPC_SC, bits, scheme);
      epochs(LPCO_LOSS_SQUARED, true, LPCO_ALGO_ALPC_GC, bits, scheme);
    }
  mlp();
  CHECK(lpco_theorem2_lhs(100, 4, 0.9, 3, 8, 16, 10, 0.01, 0) > 0.0);
  CHECK(lpco_bits_per_iteration(64, 2, 4, 0) == 1920u && lpco_bits_per_message(64, 2) == 160u);
  std::puts("oracle sanitizer walk: ok");
  return 0;
}
