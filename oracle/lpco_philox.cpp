// Counter-based random stream of the oracle (test infrastructure only).
//
// Philox4x32 with 10 rounds as published by Salmon, Moraes, Dror and Shaw,
// "Parallel random numbers: as easy as 1, 2, 3" (SC'11): a 4x32-bit counter
// and a 2x32-bit key; each round multiplies two counter words by fixed odd
// constants, swaps high/low halves with an xor of the key, and the key is
// bumped by two Weyl constants between rounds.
//
// The paper only says "with probability ..." (Sec. 3.2) and "uniformly and
// independently samples (with replacement)" (Alg. 1 step 6); the stream
// layout below is this build's convention:
//   key     = (seed low 32 bits, seed high 32 bits)
//   counter = (index >> 2, tag << 24 | worker, iter, epoch)
//   word    = output lane (index & 3)
#include "lpco.h"

namespace {
const uint32_t kMul0 = 0xD2511F53u;
const uint32_t kMul1 = 0xCD9E8D57u;
const uint32_t kWeyl0 = 0x9E3779B9u;  // golden ratio
const uint32_t kWeyl1 = 0xBB67AE85u;  // sqrt(3) - 1
}  // namespace

extern "C" void lpco_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  for (int round = 0; round < 10; ++round) {
    const uint64_t p0 = (uint64_t)kMul0 * (uint64_t)c0;
    const uint64_t p1 = (uint64_t)kMul1 * (uint64_t)c2;
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c1 ^ k0;
    const uint32_t n1 = lo1;
    const uint32_t n2 = hi0 ^ c3 ^ k1;
    const uint32_t n3 = lo0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += kWeyl0;
    k1 += kWeyl1;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

extern "C" uint32_t lpco_stream_word(uint64_t seed, uint32_t epoch, uint32_t iter, uint32_t tag, uint32_t worker,
                                     uint64_t index) {
  const uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
  const uint32_t ctr[4] = {(uint32_t)(index >> 2), (tag << 24) | (worker & 0xFFFFFFu), iter, epoch};
  uint32_t out[4];
  lpco_philox4x32_10(ctr, key, out);
  return out[index & 3u];
}

// Alg. 1 step 6 (and Alg. 2 step 11 with the shared tag): position p of the
// batch takes word p of its stream and maps it to floor(word * n / 2^32),
// which is exactly uniform when n is a power of two and has bias at most
// n / 2^32 otherwise.  Repeated indices are kept (sampling with replacement).
extern "C" int lpco_sample_batch(uint64_t seed, uint32_t epoch, uint32_t iter, uint32_t tag, uint32_t worker,
                                 int32_t B, int64_t n, int64_t *idx_out) {
  if (!idx_out) return LPCO_ENULL;
  if (B <= 0 || n <= 0 || n > (int64_t)0xFFFFFFFFll) return LPCO_EINVAL;
  for (int32_t p = 0; p < B; ++p) {
    const uint32_t word = lpco_stream_word(seed, epoch, iter, tag, worker, (uint64_t)p);
    idx_out[p] = (int64_t)(((uint64_t)word * (uint64_t)n) >> 32);
  }
  return LPCO_OK;
}
