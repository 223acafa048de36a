// Device-side helpers: the counter-based random stream and wavefront reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lpc_internal.h"

namespace lpc {

// Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).  One block
// yields the four 32-bit words of indices 4q .. 4q+3 of a stream.
struct Philox4 {
  uint32_t x, y, z, w;
};

__device__ __forceinline__ Philox4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                 uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    c1 = (uint32_t)p1;
    c3 = (uint32_t)p0;
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Philox4{c0, c1, c2, c3};
}

__device__ __forceinline__ Philox4 stream_block(const StreamKey &k, uint32_t tag, uint32_t worker, uint32_t q) {
  return philox4x32_10(q, (tag << 24) | (worker & 0xFFFFFFu), k.iter, k.epoch, k.seed_lo, k.seed_hi);
}

__device__ __forceinline__ uint32_t stream_word(const StreamKey &k, uint32_t tag, uint32_t worker, uint32_t index) {
  const Philox4 b = stream_block(k, tag, worker, index >> 2);
  const uint32_t lane = index & 3u;
  return lane == 0 ? b.x : lane == 1 ? b.y : lane == 2 ? b.z : b.w;
}

// position `pos` of a batch -> row index, floor(word * n / 2^32)
__device__ __forceinline__ int64_t sample_row(const StreamKey &k, uint32_t tag, uint32_t worker, uint32_t pos,
                                              int64_t n) {
  return (int64_t)(((uint64_t)stream_word(k, tag, worker, pos) * (uint64_t)n) >> 32);
}

// ---- wavefront (64 lanes) butterflies: every lane ends with the same bits ----
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ double wave_max(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmax(v, __shfl_xor(v, off, 64));
  return v;
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

}  // namespace lpc
