// Low-precision representation (delta, b), the quantizer Q_(delta,b) and the
// message format -- oracle side (test infrastructure only).
//
// Follows Sec. 3.2 (codebook dom(delta,b), rules (1) and (2)), eq. (3) for the
// scale factor, Sec. 4.2 for the message (b bits per coordinate plus one
// 32-bit scale factor) and eq. (4)/(5) for the averaging at the receiver.
//
// Arithmetic that decides an integer code is written out in float, one
// operation per statement, and this file is compiled with contraction off.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <utility>
#include <vector>

#include "lpco.h"

namespace {

inline bool bits_ok(int32_t b) { return b >= 2 && b <= 16; }

// code k of one coordinate.  rdelta = float(1/delta).
inline int32_t code_of(float u, float rdelta, int32_t bits, uint32_t word) {
  const float hi = (float)((1 << (bits - 1)) - 1);  // largest code, 2^(b-1)-1
  const float lo = -(float)(1 << (bits - 1));       // smallest code, -2^(b-1)
  float s = u * rdelta;                             // position on the grid
  s = std::fmin(std::fmax(s, lo), hi);              // rule (2): project onto the hull
  const float base = std::floor(s);                 // z / delta
  const float frac = s - base;                      // (x - z) / delta, exact
  const float unif = (float)(word >> 8) * 0x1.0p-24f;  // uniform on [0,1)
  // rule (1): up with probability (x - z)/delta, down otherwise
  return (int32_t)base + ((unif < frac) ? 1 : 0);
}

}  // namespace

extern "C" int64_t lpco_d_pad(int64_t d) { return ((d + 31) / 32) * 32; }
extern "C" int64_t lpco_words_per_msg(int64_t d, int32_t b) { return ((d + 31) / 32) * (int64_t)b; }

extern "C" uint64_t lpco_bits_per_message(int64_t d, int32_t bits) {
  // Sec. 4.2: b bits for each coordinate and one extra float
  return 32ull + (uint64_t)bits * (uint64_t)d;
}

extern "C" uint64_t lpco_bits_per_iteration(int64_t d, int32_t bits, int32_t N, int32_t scheme) {
  // Table 1
  const uint64_t bd = (uint64_t)bits * (uint64_t)d;
  uint64_t ceil_log = 0;
  while ((1ull << ceil_log) < (uint64_t)N) ++ceil_log;
  switch (scheme) {
    case LPCO_SCHEME_A: return (32ull + bd) * (uint64_t)N * (uint64_t)(N - 1);
    case LPCO_SCHEME_B: return (uint64_t)N * (64ull + 2ull * bd + (uint64_t)d * ceil_log);
    case LPCO_SCHEME_C: return (uint64_t)N * (64ull + 2ull * bd);
    default: return 0;
  }
}

extern "C" int lpco_vector_stats(const float *u, int64_t d, double stats[4]) {
  if (!u || !stats) return LPCO_ENULL;
  if (d < 0) return LPCO_EINVAL;
  double amax = 0.0, sum = 0.0, sumsq = 0.0, bad = 0.0;
  for (int64_t j = 0; j < d; ++j) {
    const double v = (double)u[j];
    if (!std::isfinite(v)) { bad += 1.0; continue; }
    const double a = std::fabs(v);
    if (a > amax) amax = a;
    sum += v;
    sumsq += v * v;
  }
  stats[0] = amax; stats[1] = sum; stats[2] = sumsq; stats[3] = bad;
  return bad > 0.0 ? LPCO_ENONFINITE : LPCO_OK;
}

// eq. (3): delta = lambda * |u|_inf / (2^(b-1) - 1).
// In c*sigma mode the clipping parameter is lambda = min(1, c*sigma/|u|_inf)
// with sigma the population standard deviation of the coordinates (the
// "[-c sigma, c sigma]" region of Sec. 4.1); this convention is the build's.
extern "C" int lpco_delta_from_stats(const double stats[4], int64_t d, int32_t bits, int32_t clip_mode, float clip,
                                     float *delta_out, float *thresh_out) {
  if (!stats || !delta_out) return LPCO_ENULL;
  if (!bits_ok(bits) || d <= 0) return LPCO_EINVAL;
  if (!(clip > 0.0f)) return LPCO_EINVAL;
  if (clip_mode == LPCO_CLIP_LAMBDA && clip > 1.0f) return LPCO_EINVAL;
  const float amax = (float)stats[0];
  float lambda;
  if (clip_mode == LPCO_CLIP_LAMBDA) {
    lambda = clip;
  } else if (clip_mode == LPCO_CLIP_CSIGMA) {
    if (amax > 0.0f) {
      const double mean = stats[1] / (double)d;
      double var = stats[2] / (double)d - mean * mean;
      if (var < 0.0) var = 0.0;
      const double ratio = (double)clip * std::sqrt(var) / (double)amax;
      lambda = ratio < 1.0 ? (float)ratio : 1.0f;
    } else {
      lambda = 1.0f;
    }
  } else {
    return LPCO_EINVAL;
  }
  const float thresh = lambda * amax;
  const float levels = (float)((1 << (bits - 1)) - 1);
  const float delta = thresh / levels;
  *delta_out = delta;
  if (thresh_out) *thresh_out = thresh;
  return LPCO_OK;
}

extern "C" int lpco_quantize_codes(const float *u, int64_t d, int32_t bits, float delta, float thresh, uint64_t seed,
                                   uint32_t epoch, uint32_t iter, uint32_t tag, uint32_t worker, int32_t *codes_out,
                                   uint32_t *n_clipped) {
  if (!u || !codes_out) return LPCO_ENULL;
  if (!bits_ok(bits) || d < 0) return LPCO_EINVAL;
  uint32_t clipped = 0;
  const float rdelta = (float)(1.0 / (double)delta);
  // delta == 0 happens whenever u == 0 (x_0 = x~ at the first inner iteration
  // of every epoch of Alg. 1); the message is then all zeros.
  if (!(delta > 0.0f) || !std::isfinite(rdelta)) {
    for (int64_t j = 0; j < d; ++j) codes_out[j] = 0;
    if (n_clipped) *n_clipped = 0;
    return LPCO_OK;
  }
  // a coordinate "exceeds dom(delta,b)" (Lemma 2) when it lies above the
  // positive clip threshold lambda*|u|_inf or below the smallest codebook
  // value -2^(b-1)*delta (a power-of-two multiple, exact in float).
  const float neg_edge = -(float)(1 << (bits - 1)) * delta;
  for (int64_t j = 0; j < d; ++j) {
    const uint32_t word = lpco_stream_word(seed, epoch, iter, tag, worker, (uint64_t)j);
    codes_out[j] = code_of(u[j], rdelta, bits, word);
    if (u[j] > thresh || u[j] < neg_edge) ++clipped;
  }
  if (n_clipped) *n_clipped = clipped;
  return LPCO_OK;
}

// Message layout: code j is stored as a b-bit two's-complement field in bits
// [j*b, j*b + b) of a little-endian bit stream; stream bit p is bit (p & 31)
// of word (p >> 5).  Coordinates d..d_pad-1 are code 0.
extern "C" int lpco_pack(const int32_t *codes, int64_t d, int32_t bits, uint32_t *words) {
  if (!codes || !words) return LPCO_ENULL;
  if (!bits_ok(bits) || d < 0) return LPCO_EINVAL;
  const int64_t W = lpco_words_per_msg(d, bits);
  for (int64_t w = 0; w < W; ++w) words[w] = 0u;
  const uint32_t mask = (1u << bits) - 1u;
  for (int64_t j = 0; j < d; ++j) {
    const uint32_t field = (uint32_t)codes[j] & mask;
    for (int32_t t = 0; t < bits; ++t) {
      const int64_t p = j * (int64_t)bits + t;
      if ((field >> t) & 1u) words[p >> 5] |= (1u << (p & 31));
    }
  }
  return LPCO_OK;
}

extern "C" int lpco_unpack(const uint32_t *words, int64_t d, int32_t bits, int32_t *codes_out) {
  if (!words || !codes_out) return LPCO_ENULL;
  if (!bits_ok(bits) || d < 0) return LPCO_EINVAL;
  for (int64_t j = 0; j < d; ++j) {
    uint32_t field = 0;
    for (int32_t t = 0; t < bits; ++t) {
      const int64_t p = j * (int64_t)bits + t;
      field |= ((words[p >> 5] >> (p & 31)) & 1u) << t;
    }
    int32_t k = (int32_t)field;
    if (field & (1u << (bits - 1))) k -= (1 << bits);  // sign-extend
    codes_out[j] = k;
  }
  return LPCO_OK;
}

extern "C" int lpco_quantize_clip(int64_t d, int32_t N, int32_t bits, int32_t clip_mode, float clip, uint64_t seed,
                                  uint32_t epoch, uint32_t iter, const float *U, const double *stats,
                                  const float *delta_in, uint32_t *packed, float *delta_out, uint32_t *n_clipped) {
  if (!U || !packed || !delta_out) return LPCO_ENULL;
  if (!bits_ok(bits) || d <= 0 || N <= 0) return LPCO_EINVAL;
  const int64_t dp = lpco_d_pad(d);
  const int64_t W = lpco_words_per_msg(d, bits);
  std::vector<int32_t> codes((size_t)d);
  int rc = LPCO_OK;
  for (int32_t i = 0; i < N; ++i) {
    const float *u = U + (int64_t)i * dp;
    double st[4];
    if (stats) {
      std::memcpy(st, stats + 4 * (int64_t)i, sizeof(st));
    } else {
      lpco_vector_stats(u, d, st);
    }
    if (st[3] > 0.0) rc = LPCO_ENONFINITE;
    float delta, thresh;
    if (delta_in) {
      delta = delta_in[i];
      thresh = delta * (float)((1 << (bits - 1)) - 1);
    } else {
      const int r = lpco_delta_from_stats(st, d, bits, clip_mode, clip, &delta, &thresh);
      if (r != LPCO_OK) return r;
    }
    uint32_t nc = 0;
    lpco_quantize_codes(u, d, bits, delta, thresh, seed, epoch, iter, LPCO_TAG_QUANT, (uint32_t)i, codes.data(), &nc);
    const float rdelta = (float)(1.0 / (double)delta);
    delta_out[i] = (delta > 0.0f && std::isfinite(rdelta)) ? delta : 0.0f;
    if (n_clipped) n_clipped[i] = nc;
    lpco_pack(codes.data(), d, bits, packed + (int64_t)i * W);
  }
  return rc;
}

// eq. (4): every receiver recovers each peer's vector with that peer's own
// scale factor and averages.  Fixed worker order, one fused multiply-add per
// worker, one multiply by 1/N at the end.
extern "C" int lpco_dequantize_avg(int64_t d, int32_t N, int32_t bits, const uint32_t *packed, const float *delta,
                                   float *u_avg) {
  if (!packed || !delta || !u_avg) return LPCO_ENULL;
  if (!bits_ok(bits) || d <= 0 || N <= 0) return LPCO_EINVAL;
  const int64_t W = lpco_words_per_msg(d, bits);
  std::vector<int32_t> codes((size_t)N * (size_t)d);
  for (int32_t i = 0; i < N; ++i) lpco_unpack(packed + (int64_t)i * W, d, bits, codes.data() + (int64_t)i * d);
  const float inv_n = 1.0f / (float)N;
  for (int64_t j = 0; j < d; ++j) {
    float acc = 0.0f;
    for (int32_t i = 0; i < N; ++i) acc = std::fmaf(delta[i], (float)codes[(int64_t)i * d + j], acc);
    u_avg[j] = acc * inv_n;
  }
  return LPCO_OK;
}

extern "C" int lpco_plain_avg(int64_t d, int32_t N, const float *U, float *u_avg) {
  if (!U || !u_avg) return LPCO_ENULL;
  if (d <= 0 || N <= 0) return LPCO_EINVAL;
  const int64_t dp = lpco_d_pad(d);
  const float inv_n = 1.0f / (float)N;
  for (int64_t j = 0; j < d; ++j) {
    float acc = 0.0f;
    for (int32_t i = 0; i < N; ++i) acc = acc + U[(int64_t)i * dp + j];
    u_avg[j] = acc * inv_n;
  }
  return LPCO_OK;
}

// Schemes (b) and (c) of Sec. 4.2: all workers use delta = max_i delta_i, so
// codes add as integers (ceil(log N) overflow bits) and a single scaling
// recovers the average.  With requantize != 0 the average is stochastically
// rounded once more onto dom(delta, b) (eq. (5)); it lies in the hull, so
// this second rounding is unbiased.
extern "C" int lpco_dequantize_shared(int64_t d, int32_t N, int32_t bits, const uint32_t *packed, float delta_shared,
                                      int32_t requantize, uint64_t seed, uint32_t epoch, uint32_t iter, float *u_avg,
                                      int32_t *code_sums) {
  if (!packed || !u_avg) return LPCO_ENULL;
  if (!bits_ok(bits) || d <= 0 || N <= 0) return LPCO_EINVAL;
  const int64_t W = lpco_words_per_msg(d, bits);
  std::vector<int32_t> sums((size_t)d, 0), codes((size_t)d);
  for (int32_t i = 0; i < N; ++i) {
    lpco_unpack(packed + (int64_t)i * W, d, bits, codes.data());
    for (int64_t j = 0; j < d; ++j) sums[j] += codes[j];
  }
  if (code_sums) std::memcpy(code_sums, sums.data(), sizeof(int32_t) * (size_t)d);
  const float inv_n = 1.0f / (float)N;
  for (int64_t j = 0; j < d; ++j) {
    const float mean_code = (float)sums[j] * inv_n;  // position of the average on the grid
    if (!requantize) {
      u_avg[j] = delta_shared * mean_code;
    } else {
      const uint32_t word = lpco_stream_word(seed, epoch, iter, LPCO_TAG_REQUANT, 0u, (uint64_t)j);
      const int32_t k = code_of(mean_code, 1.0f, bits, word);
      u_avg[j] = delta_shared * (float)k;
    }
  }
  return LPCO_OK;
}

// Entropy coding of the code stream (Sec. 6.1: "adopt the entropy encoding scheme [Huffman 1952] to
// further reduce the communication overhead").  Given the counts of the 2^b code values, the length
// of an optimal prefix code for each value by Huffman's merging of the two least frequent subtrees;
// returns the number of bits of the encoded message, sum_k count_k * len_k (a lone symbol costs 1
// bit per coordinate).  lens_out may be NULL.
extern "C" uint64_t lpco_huffman_bits(const uint64_t *counts, int32_t nsym, int32_t *lens_out) {
  if (!counts || nsym <= 0) return 0;
  struct Node { uint64_t w; int32_t left, right; };
  std::vector<Node> nodes;
  std::vector<int32_t> alive;
  for (int32_t k = 0; k < nsym; ++k) {
    nodes.push_back(Node{counts[k], -1, -1});
    if (counts[k] > 0) alive.push_back(k);
  }
  std::vector<int32_t> lens((size_t)nsym, 0);
  if (alive.size() == 1) lens[(size_t)alive[0]] = 1;
  while (alive.size() > 1) {
    // two smallest weights (ties: lowest index first); plain selection, the alphabet is tiny
    size_t a = 0, b = 1;
    if (nodes[(size_t)alive[b]].w < nodes[(size_t)alive[a]].w) std::swap(a, b);
    for (size_t t = 2; t < alive.size(); ++t) {
      const uint64_t wt = nodes[(size_t)alive[t]].w;
      if (wt < nodes[(size_t)alive[a]].w) { b = a; a = t; }
      else if (wt < nodes[(size_t)alive[b]].w) { b = t; }
    }
    const int32_t ia = alive[a], ib = alive[b];
    nodes.push_back(Node{nodes[(size_t)ia].w + nodes[(size_t)ib].w, ia, ib});
    const int32_t merged = (int32_t)nodes.size() - 1;
    if (a > b) std::swap(a, b);
    alive.erase(alive.begin() + (long)b);
    alive.erase(alive.begin() + (long)a);
    alive.push_back(merged);
  }
  if (!alive.empty() && alive.size() == 1 && nodes.size() > (size_t)nsym) {
    // depth of every leaf below the root
    std::vector<std::pair<int32_t, int32_t>> stack{{alive[0], 0}};
    while (!stack.empty()) {
      const auto [id, depth] = stack.back();
      stack.pop_back();
      if (nodes[(size_t)id].left < 0) { lens[(size_t)id] = depth; continue; }
      stack.push_back({nodes[(size_t)id].left, depth + 1});
      stack.push_back({nodes[(size_t)id].right, depth + 1});
    }
  }
  uint64_t bits = 0;
  for (int32_t k = 0; k < nsym; ++k) {
    bits += counts[k] * (uint64_t)lens[(size_t)k];
    if (lens_out) lens_out[k] = lens[(size_t)k];
  }
  return bits;
}

// counts of the 2^b code values of one packed message (coordinates 0..d-1); bin k holds code k - 2^(b-1)
extern "C" int lpco_code_histogram(const uint32_t *words, int64_t d, int32_t bits, uint64_t *counts) {
  if (!words || !counts) return LPCO_ENULL;
  if (!bits_ok(bits) || d < 0) return LPCO_EINVAL;
  std::vector<int32_t> codes((size_t)d);
  lpco_unpack(words, d, bits, codes.data());
  for (int32_t k = 0; k < (1 << bits); ++k) counts[k] = 0;
  for (int64_t j = 0; j < d; ++j) counts[codes[(size_t)j] + (1 << (bits - 1))] += 1;
  return LPCO_OK;
}

// ---- the entropy-coded bit stream itself ----
// The paper names Huffman coding and no format.  Reading taken: the prefix code is the CANONICAL one for
// the given code lengths -- symbols (bin index k = code + 2^(b-1)) ordered by (length, k), the first gets
// the all-zero codeword, each next one the previous codeword plus one, shifted left by the growth in
// length -- and the codewords of coordinates 0, 1, ..., d-1 follow one another most significant bit first;
// stream bit p lives in word p/32 at bit p%32 (the bit order of the packed messages).
namespace {

// codeword of every symbol for the given lengths, or false if the lengths do not form a prefix code
bool canonical_codes(const int32_t *lens, int32_t nsym, std::vector<uint64_t> &code) {
  code.assign((size_t)nsym, 0);
  int32_t maxlen = 0;
  for (int32_t k = 0; k < nsym; ++k) {
    if (lens[k] < 0 || lens[k] > 57) return false;
    if (lens[k] > maxlen) maxlen = lens[k];
  }
  uint64_t next = 0;
  int32_t prev_len = 0;
  for (int32_t len = 1; len <= maxlen; ++len) {
    for (int32_t k = 0; k < nsym; ++k) {
      if (lens[k] != len) continue;
      next <<= (len - prev_len);
      prev_len = len;
      if (next >> len) return false;  // more codewords of this length than the shorter ones leave room for
      code[(size_t)k] = next;
      next += 1;
    }
  }
  return true;
}

}  // namespace

// Encodes the first d coordinates of one packed message.  out_words (capacity_words words, zero-filled
// here) receives the stream, *total_bits_out its length.  LPCO_EINVAL if the lengths are no prefix code,
// a coordinate's symbol has length 0, or the stream does not fit.
extern "C" int lpco_huffman_encode(const uint32_t *words, int64_t d, int32_t bits, const int32_t *lens,
                                   uint32_t *out_words, int64_t capacity_words, uint64_t *total_bits_out) {
  if (!words || !lens || !out_words || !total_bits_out) return LPCO_ENULL;
  if (!bits_ok(bits) || d < 0 || capacity_words < 0) return LPCO_EINVAL;
  const int32_t nsym = 1 << bits;
  std::vector<uint64_t> code;
  if (!canonical_codes(lens, nsym, code)) return LPCO_EINVAL;
  std::vector<int32_t> codes((size_t)d);
  lpco_unpack(words, d, bits, codes.data());
  for (int64_t w = 0; w < capacity_words; ++w) out_words[w] = 0u;
  uint64_t pos = 0;
  for (int64_t j = 0; j < d; ++j) {
    const int32_t k = codes[(size_t)j] + (nsym >> 1);
    const int32_t len = lens[k];
    if (len == 0) return LPCO_EINVAL;
    for (int32_t i = len - 1; i >= 0; --i) {  // most significant bit of the codeword first
      if ((int64_t)(pos >> 5) >= capacity_words) return LPCO_EINVAL;
      if ((code[(size_t)k] >> i) & 1u) out_words[pos >> 5] |= 1u << (pos & 31u);
      ++pos;
    }
  }
  *total_bits_out = pos;
  return LPCO_OK;
}

// Decodes d coordinates from such a stream, reading bit by bit until the bits read so far are a codeword.
extern "C" int lpco_huffman_decode(const uint32_t *stream, uint64_t total_bits, int64_t d, int32_t bits,
                                   const int32_t *lens, int32_t *codes_out) {
  if (!stream || !lens || !codes_out) return LPCO_ENULL;
  if (!bits_ok(bits) || d < 0) return LPCO_EINVAL;
  const int32_t nsym = 1 << bits;
  std::vector<uint64_t> code;
  if (!canonical_codes(lens, nsym, code)) return LPCO_EINVAL;
  uint64_t pos = 0;
  for (int64_t j = 0; j < d; ++j) {
    uint64_t acc = 0;
    int32_t len = 0, found = -1;
    while (found < 0) {
      if (pos >= total_bits || len >= 57) return LPCO_EINVAL;
      acc = (acc << 1) | ((stream[pos >> 5] >> (pos & 31u)) & 1u);
      ++pos; ++len;
      for (int32_t k = 0; k < nsym; ++k)
        if (lens[k] == len && code[(size_t)k] == acc) { found = k; break; }
    }
    codes_out[j] = found - (nsym >> 1);
  }
  return pos == total_bits ? LPCO_OK : LPCO_EINVAL;
}
