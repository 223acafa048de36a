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
    // three-input exclusive-or in one instruction (truth table 0x96)
    const uint32_t n0 = __builtin_amdgcn_bitop3_b32((uint32_t)(p1 >> 32), c1, k0, 0x96);
    const uint32_t n2 = __builtin_amdgcn_bitop3_b32((uint32_t)(p0 >> 32), c3, k1, 0x96);
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

// Requests every 64-byte line of the kernel's argument block with one burst of scalar loads and waits for them
// once.  A kernel whose arguments are a large structure otherwise fetches its fields where it first needs them: the
// compiler places those scalar loads block by block, each first touch of a line is a round trip to memory (the
// host wrote the block, so no cache holds it), and a latency-bound kernel starts with several of them in a row.
// BYTES = size of the argument block (the kernel's parameters in declaration order).
template <int BYTES>
__device__ __forceinline__ void touch_kernel_arguments() {
  typedef const uint32_t __attribute__((address_space(4))) *KernargWords;
  KernargWords ka = (KernargWords)__builtin_amdgcn_kernarg_segment_ptr();
  uint32_t seen = 0;
#pragma unroll
  for (int k = 0; k < (BYTES + 63) / 64; ++k) seen |= ka[k * 16 < BYTES / 4 ? k * 16 : BYTES / 4 - 1];
  asm volatile("" ::"s"(seen));
}

// ---- wavefront (64 lanes) reductions: every lane ends with the same bits ----
// Lanes exchange values with data-parallel-primitive moves inside their row of 16 (no trip through the
// LDS crossbar): after xor-1, xor-2, half-mirror and mirror steps every lane of a row holds the row's
// result; the four row results are then read as scalars and combined in a fixed order.  The whole
// wavefront must be active at the call (row16_* only needs whole rows of 16 active).
template <int CTRL>
__device__ __forceinline__ int dpp_move(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, dpp_move<CTRL>(__builtin_bit_cast(int, v)));
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v) {
  return (uint32_t)dpp_move<CTRL>((int)v);
}
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  const uint64_t b = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = dpp_move<CTRL>((uint32_t)b), hi = dpp_move<CTRL>((uint32_t)(b >> 32));
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ float read_lane(float v, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
__device__ __forceinline__ uint32_t read_lane(uint32_t v, int l) { return (uint32_t)__builtin_amdgcn_readlane((int)v, l); }
__device__ __forceinline__ double read_lane(double v, int l) {
  const uint64_t b = __builtin_bit_cast(uint64_t, v);
  const uint32_t lo = read_lane((uint32_t)b, l), hi = read_lane((uint32_t)(b >> 32), l);
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
constexpr int kDppXor1 = 0xB1;         // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;         // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;  // lane i <-> 7-i inside each half row
constexpr int kDppMirror = 0x140;      // lane i <-> 15-i inside the row

template <class T>
__device__ __forceinline__ T row16_sum(T v) {
  v += dpp_move<kDppXor1>(v);
  v += dpp_move<kDppXor2>(v);
  v += dpp_move<kDppHalfMirror>(v);
  v += dpp_move<kDppMirror>(v);
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_move<kDppXor1>(v));
  v = fmaxf(v, dpp_move<kDppXor2>(v));
  v = fmaxf(v, dpp_move<kDppHalfMirror>(v));
  v = fmaxf(v, dpp_move<kDppMirror>(v));
  return v;
}
__device__ __forceinline__ double row16_max(double v) {
  v = fmax(v, dpp_move<kDppXor1>(v));
  v = fmax(v, dpp_move<kDppXor2>(v));
  v = fmax(v, dpp_move<kDppHalfMirror>(v));
  v = fmax(v, dpp_move<kDppMirror>(v));
  return v;
}
template <class T>
__device__ __forceinline__ T wave_sum_t(T v) {
  v = row16_sum(v);
  return (read_lane(v, 0) + read_lane(v, 16)) + (read_lane(v, 32) + read_lane(v, 48));
}
__device__ __forceinline__ float wave_sum(float v) { return wave_sum_t(v); }
__device__ __forceinline__ double wave_sum(double v) { return wave_sum_t(v); }
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) { return wave_sum_t(v); }
__device__ __forceinline__ float wave_max(float v) {
  v = row16_max(v);
  return fmaxf(fmaxf(read_lane(v, 0), read_lane(v, 16)), fmaxf(read_lane(v, 32), read_lane(v, 48)));
}
__device__ __forceinline__ double wave_max(double v) {
  v = row16_max(v);
  return fmax(fmax(read_lane(v, 0), read_lane(v, 16)), fmax(read_lane(v, 32), read_lane(v, 48)));
}

// ---- pieces shared by the quantizer's launches and the resident inner loop ---------------------------------------
// (the translation units that use them are compiled with floating-point contraction off)
struct QuantSpec {
  int32_t bits;
  int32_t clip_mode;
  float clip;
  int32_t enabled;
};

// eq. (3): delta = lambda*|u|_inf/(2^(b-1)-1); in c*sigma mode
// lambda = min(1, c*sigma/|u|_inf) with sigma the population standard deviation.
__device__ inline QParams make_qparams(const QuantSpec &qs, double amax_d, double sum, double sumsq, int64_t d) {
  QParams q;
  const float amax = (float)amax_d;
  float lambda;
  if (qs.clip_mode == LPC_CLIP_LAMBDA) {
    lambda = qs.clip;
  } else if (amax > 0.0f) {
    const double mean = sum / (double)d;
    double var = sumsq / (double)d - mean * mean;
    if (var < 0.0) var = 0.0;
    const double ratio = (double)qs.clip * sqrt(var) / (double)amax;
    lambda = ratio < 1.0 ? (float)ratio : 1.0f;
  } else {
    lambda = 1.0f;
  }
  const float thresh = lambda * amax;
  const float levels = (float)((1 << (qs.bits - 1)) - 1);
  const float delta = thresh / levels;
  const float rdelta = (float)(1.0 / (double)delta);
  const bool live = delta > 0.0f && isfinite(rdelta);
  q.delta = live ? delta : 0.0f;
  q.rdelta = live ? rdelta : 0.0f;
  q.thresh = thresh;
  q.neg_edge = -(float)(1 << (qs.bits - 1)) * delta;
  return q;
}

// prox_{step*h}(w - step*v) for h = lambda1*|.|_1 + (lambda2/2)*|.|^2 (Alg. 1 steps 9-10): thr = step*lambda1,
// shrink = 1/(1 + step*lambda2)
__device__ __forceinline__ float prox_scalar(float w, float v, float step, float thr, float shrink) {
  const float p = w - step * v;
  const float mag = fabsf(p) - thr;
  return mag > 0.0f ? copysignf(mag * shrink, p) : 0.0f;
}

// derivative of the per-sample loss with respect to the margin z = x'w (logistic with labels +-1, or squared)
__device__ __forceinline__ float loss_slope(int32_t loss, float z, float y) {
  if (loss == LPC_LOSS_LOGISTIC) return -y / (1.0f + expf(y * z));
  return z - y;
}

// ---- partial dot products of sampled rows with one 128-column tile of an iterate -------------------------------
// (the small-d inner iteration's margins: see the column-tile worker pass in lpc_dense.hip)
constexpr int kColTile = 128;     // columns per tile / workgroup
constexpr int kColThreads = 512;  // 16 groups of 32 lanes; a group takes one row at a time, a lane four columns
constexpr int kDotRows = 8 * (kColThreads / 32);  // rows one load / finish pair covers: eight per group

__device__ __forceinline__ float4 load_slice(const float *p, int64_t room, bool vec4) {
  float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
  if (room <= 0) return t;
  if (vec4) return *reinterpret_cast<const float4 *>(p);
  t.x = p[0];
  if (room > 1) t.y = p[1];
  if (room > 2) t.z = p[2];
  if (room > 3) t.w = p[3];
  return t;
}

// sum over the 32 adjacent lanes of a group (a fixed order); every lane of the wavefront takes part
__device__ __forceinline__ float group32_sum(float v, int lane) {
  v = row16_sum(v);
  const float lo = read_lane(v, 0) + read_lane(v, 16), hi = read_lane(v, 32) + read_lane(v, 48);
  return lane < 32 ? lo : hi;
}

// pd[row][c] = x_row[tile c] . w[tile c] for the rows that the vectors [worker_begin, worker_begin + nvec) sample at
// `key` (the last one the shared batch when shared_rel says so); row = vector * B + batch position.
struct DotsArgs {
  const float *X;
  int64_t ldx, d, n;
  const float *w;
  float *pd;
  int32_t C, B, nvec, worker_begin, shared_rel, rows_per_wg, vec4;
  StreamKey key;
  uint32_t tag;
};

// request the tile-c slices of rows [first, first + count), count <= kDotRows, of the launch's row list
__device__ __forceinline__ void tile_dots_load(const DotsArgs &a, int32_t c, int32_t first, int32_t count, int tid,
                                               float4 (&x)[8]) {
  constexpr int GROUPS = kColThreads / 32;
  const int rg = tid >> 5, l = tid & 31;
  const int64_t j = (int64_t)c * kColTile + 4 * l;
  const int64_t room = a.d - j;
  const int32_t total = a.nvec * a.B;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const int32_t i = first + k * GROUPS + rg;
    x[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (k * GROUPS + rg < count && i < total) {
      const int32_t wrel = i / a.B, pos = i % a.B;
      const uint32_t tag = wrel == a.shared_rel ? kTagShared : a.tag;
      const uint32_t worker = tag == kTagShared ? kSharedWorkerField : (uint32_t)(a.worker_begin + wrel);
      const int64_t row = sample_row(a.key, tag, worker, (uint32_t)pos, a.n);
      x[k] = load_slice(a.X + row * a.ldx + j, room, a.vec4 != 0);
    }
  }
}

// ... and their dot products with the tile's slice of the iterate held in wsh (LDS, 128 floats, zero past d)
__device__ __forceinline__ void tile_dots_finish(const DotsArgs &a, const float *wsh, int32_t c, int32_t first,
                                                 int32_t count, int tid, const float4 (&x)[8]) {
  constexpr int GROUPS = kColThreads / 32;
  const int lane = tid & 63, rg = tid >> 5, l = tid & 31;
  const float4 w4 = *reinterpret_cast<const float4 *>(wsh + 4 * l);
  const int32_t total = a.nvec * a.B;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    float s = x[k].x * w4.x;
    s = fmaf(x[k].y, w4.y, s); s = fmaf(x[k].z, w4.z, s); s = fmaf(x[k].w, w4.w, s);
    s = group32_sum(s, lane);
    const int32_t i = first + k * GROUPS + rg;
    if (l == 0 && k * GROUPS + rg < count && i < total) a.pd[(int64_t)i * a.C + c] = s;
  }
}

}  // namespace lpc
