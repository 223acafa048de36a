// Driver for a sanitizer build of the library's host-only translation unit (csrc/lpc_host.cpp, built by
// tests/test_sanitizers.py with g++ -fsanitize=address,undefined): walks argument validation, the size helpers,
// Table 1, Theorem 2's condition and the entropy coder's code construction over ordinary, boundary and invalid
// inputs.  No device memory is touched: the validation reads only the structs, never what their pointers name.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "lpc_internal.h"

#define CHECK(cond)                                                                  \
  do {                                                                               \
    if (!(cond)) {                                                                   \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      std::exit(1);                                                                  \
    }                                                                                \
  } while (0)

static float fake_storage[64];  // addresses only: validation checks alignment and NULL, never dereferences

static void validation() {
  const float *dev = fake_storage;
  const int32_t *idev = (const int32_t *)fake_storage;
  lpc_problem p{};
  p.n = 100; p.d = 20; p.loss = LPC_LOSS_LOGISTIC; p.X = dev; p.ldx = 20; p.y = dev; p.lambda1 = 1e-3f; p.lambda2 = 0.0f;
  CHECK(lpc::check_problem(&p) == LPC_OK);
  CHECK(lpc::check_problem(nullptr) == LPC_ENULL);
  { lpc_problem q = p; q.n = 0; CHECK(lpc::check_problem(&q) == LPC_ESHAPE); }
  { lpc_problem q = p; q.d = (int64_t)1 << 32; CHECK(lpc::check_problem(&q) == LPC_ESHAPE); }
  { lpc_problem q = p; q.ldx = 19; CHECK(lpc::check_problem(&q) == LPC_ESHAPE); }
  { lpc_problem q = p; q.y = nullptr; CHECK(lpc::check_problem(&q) == LPC_ENULL); }
  { lpc_problem q = p; q.loss = 9; CHECK(lpc::check_problem(&q) == LPC_EINVAL); }
  { lpc_problem q = p; q.lambda1 = -1.0f; CHECK(lpc::check_problem(&q) == LPC_EINVAL); }
  { lpc_problem q = p; q.X = (const float *)((const char *)dev + 1); CHECK(lpc::check_problem(&q) == LPC_ESHAPE); }
  { lpc_problem q = p; q.row_ptr = idev; CHECK(lpc::check_problem(&q) == LPC_EINVAL); }  // two storage formats
  lpc_problem s = p;
  s.X = nullptr; s.row_ptr = idev; s.col_idx = idev; s.vals = dev; s.nnz = 50;
  CHECK(lpc::check_problem(&s) == LPC_OK);
  { lpc_problem q = s; q.vals = nullptr; CHECK(lpc::check_problem(&q) == LPC_ENULL); }
  { lpc_problem q = s; q.nnz = (int64_t)1 << 31; CHECK(lpc::check_problem(&q) == LPC_ESHAPE); }
  { lpc_problem q = s; q.loss = LPC_LOSS_MLP_SOFTMAX; CHECK(lpc::check_problem(&q) == LPC_EINVAL); }
  const int32_t dims[3] = {4, 3, 2};
  lpc_problem m = p;
  m.loss = LPC_LOSS_MLP_SOFTMAX; m.mlp_dims = dims; m.mlp_nlayers = 2; m.d = 4 * 3 + 3 + 3 * 2 + 2; m.ldx = 4;
  CHECK(lpc::check_problem(&m) == LPC_OK);
  { lpc_problem q = m; q.d += 1; CHECK(lpc::check_problem(&q) == LPC_ESHAPE); }
  { lpc_problem q = m; q.ldx = 3; CHECK(lpc::check_problem(&q) == LPC_ESHAPE); }
  { lpc_problem q = m; q.mlp_dims = nullptr; CHECK(lpc::check_problem(&q) == LPC_ENULL); }
  const int32_t bad_dims[3] = {4, 0, 2};
  { lpc_problem q = m; q.mlp_dims = bad_dims; CHECK(lpc::check_problem(&q) == LPC_ESHAPE); }

  lpc_config c{};
  c.algo = LPC_ALGO_LPC; c.N = 4; c.B = 5; c.m = 3; c.bits = 4; c.clip_mode = LPC_CLIP_LAMBDA; c.clip = 0.9f;
  c.scheme = LPC_SCHEME_A; c.eta = 0.1f;
  CHECK(lpc::check_config(&p, &c) == LPC_OK);
  CHECK(lpc::check_config(&p, nullptr) == LPC_ENULL);
  { lpc_config q = c; q.bits = 1; CHECK(lpc::check_config(&p, &q) == LPC_EINVAL); }
  { lpc_config q = c; q.bits = 17; CHECK(lpc::check_config(&p, &q) == LPC_EINVAL); }
  { lpc_config q = c; q.bits = 32; CHECK(lpc::check_config(&p, &q) == LPC_OK); }
  { lpc_config q = c; q.N = 30; CHECK(lpc::check_config(&p, &q) == LPC_EINVAL); }  // N*B > n
  { lpc_config q = c; q.N = 0x7FFFFFFF; q.B = 0x7FFFFFFF; CHECK(lpc::check_config(&p, &q) == LPC_EINVAL); }
  { lpc_config q = c; q.clip = 1.5f; CHECK(lpc::check_config(&p, &q) == LPC_EINVAL); }
  { lpc_config q = c; q.clip_mode = LPC_CLIP_CSIGMA; q.clip = 1.5f; CHECK(lpc::check_config(&p, &q) == LPC_OK); }
  { lpc_config q = c; q.eta = 0.0f; CHECK(lpc::check_config(&p, &q) == LPC_EINVAL); }
  { lpc_config q = c; q.n_full = 101; CHECK(lpc::check_config(&p, &q) == LPC_EINVAL); }
  { lpc_config q = c; q.algo = LPC_ALGO_ALPC_GC; CHECK(lpc::check_config(&p, &q) == LPC_EINVAL); }  // L missing
  { lpc_config q = c; q.algo = LPC_ALGO_ALPC_GC; q.L = 2.0f; CHECK(lpc::check_config(&p, &q) == LPC_OK); }
  { lpc_config q = c; q.tau1 = 0.7f; q.tau2 = 0.5f; CHECK(lpc::check_config(&p, &q) == LPC_EINVAL); }
  { lpc_config q = c; q.scheme = 3; CHECK(lpc::check_config(&p, &q) == LPC_EINVAL); }
}

static void sizes_and_formulas() {
  CHECK(lpc_d_pad(1) == 32 && lpc_d_pad(32) == 32 && lpc_d_pad(33) == 64);
  CHECK(lpc_words_per_msg(33, 3) == 6 && lpc_words_per_msg(0, 5) == 0);
  for (int s = 0; s >= -8; --s) CHECK(lpc_status_string((lpc_status)s) != nullptr);
  uint64_t bits = 0;
  CHECK(lpc_bits_per_iteration(64, 2, 4, LPC_SCHEME_A, &bits) == LPC_OK && bits == (32u + 128u) * 12u);
  CHECK(lpc_bits_per_iteration(64, 2, 4, LPC_SCHEME_B, &bits) == LPC_OK && bits == 4u * (64u + 256u + 128u));
  CHECK(lpc_bits_per_iteration(64, 2, 4, LPC_SCHEME_C, &bits) == LPC_OK && bits == 4u * (64u + 256u));
  CHECK(lpc_bits_per_iteration(64, 2, 1, LPC_SCHEME_B, &bits) == LPC_OK && bits == 64u + 256u);
  CHECK(lpc_bits_per_iteration((int64_t)0xFFFFFFFFll, 16, 1 << 20, LPC_SCHEME_A, &bits) == LPC_OK);  // no signed overflow
  CHECK(lpc_bits_per_iteration(64, 2, 4, LPC_SCHEME_A, nullptr) == LPC_ENULL);
  CHECK(lpc_bits_per_iteration(64, 1, 4, LPC_SCHEME_A, &bits) == LPC_EINVAL);
  CHECK(lpc_bits_per_iteration(-1, 4, 4, LPC_SCHEME_A, &bits) == LPC_EINVAL);
  double lhs = 0.0;
  CHECK(lpc_theorem2_lhs(100, 4, 0.9, 3, 8, 16, 10, 0.01, LPC_SCHEME_A, &lhs) == LPC_OK && lhs > 0.01);
  CHECK(lpc_theorem2_lhs(100, 16, 1.0, 0, 1, 1, 1, 0.25, LPC_SCHEME_C, &lhs) == LPC_OK);
  CHECK(lpc_theorem2_lhs(100, 1, 0.9, 3, 8, 16, 10, 0.01, LPC_SCHEME_A, &lhs) == LPC_EINVAL);
  CHECK(lpc_theorem2_lhs(100, 4, 0.9, 3, 8, 16, 10, 0.01, LPC_SCHEME_A, nullptr) == LPC_ENULL);
}

static void entropy_code() {
  // skewed, flat, single-symbol, empty and 2^16-symbol histograms; Kraft's equality for every optimal code
  std::vector<std::vector<uint64_t>> hists = {{5, 1, 1, 1}, {3, 3, 3, 3, 3, 3, 3, 3}, {0, 9, 0, 0}, {0, 0}, {1},
                                             {1, 1, 2, 3, 5, 8, 13, 21, 34, 55, 89, 144, 233, 377, 610, 987}};
  std::vector<uint64_t> wide((size_t)1 << 16);
  for (size_t k = 0; k < wide.size(); ++k) wide[k] = (k * 2654435761u) % 97u;
  hists.push_back(wide);
  for (const auto &h : hists) {
    const int32_t nsym = (int32_t)h.size();
    std::vector<int32_t> lens((size_t)nsym, -7);
    uint64_t total = 123;
    CHECK(lpc_huffman_bits(h.data(), nsym, lens.data(), &total) == LPC_OK);
    uint64_t expect = 0, used = 0;
    long double kraft = 0.0L;
    for (int32_t k = 0; k < nsym; ++k) {
      CHECK((h[(size_t)k] == 0) == (lens[(size_t)k] == 0));
      expect += h[(size_t)k] * (uint64_t)lens[(size_t)k];
      if (lens[(size_t)k]) { kraft += 1.0L / (long double)(1ull << lens[(size_t)k]); ++used; }
    }
    CHECK(total == expect);
    if (used >= 2) CHECK(kraft > 0.999999L && kraft < 1.000001L);
    uint64_t only_total = 0;
    CHECK(lpc_huffman_bits(h.data(), nsym, nullptr, &only_total) == LPC_OK && only_total == total);
    std::vector<lpc::HuffEntry> table((size_t)nsym);
    CHECK(lpc::huffman_canonical_table(lens.data(), nsym, table.data()) == 0);
    for (int32_t k = 0; k < nsym; ++k) CHECK(table[(size_t)k].len == (uint32_t)lens[(size_t)k]);
  }
  const int32_t over[3] = {1, 1, 1};   // three one-bit codewords do not exist
  lpc::HuffEntry t3[3];
  CHECK(lpc::huffman_canonical_table(over, 3, t3) == -1);
  const int32_t too_long[2] = {33, 1};
  CHECK(lpc::huffman_canonical_table(too_long, 2, t3) == -1);
  const int32_t deep[2] = {32, 32};    // the longest codeword the table holds
  CHECK(lpc::huffman_canonical_table(deep, 2, t3) == 0 && t3[1].len == 32u);
  uint64_t dummy = 0;
  CHECK(lpc_huffman_bits(nullptr, 4, nullptr, &dummy) == LPC_ENULL);
  CHECK(lpc_huffman_bits(wide.data(), 0, nullptr, &dummy) == LPC_EINVAL);
  CHECK(lpc_huffman_bits(wide.data(), (1 << 16) + 1, nullptr, &dummy) == LPC_EINVAL);
}

int main() {
  validation();
  sizes_and_formulas();
  entropy_code();
  std::puts("host sanitizer walk: ok");
  return 0;
}
