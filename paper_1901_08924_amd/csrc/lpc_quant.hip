// Quantizer, message format, receiver-side averaging, proximal step and the
// small reductions around them (gfx950).
//
// This translation unit is compiled with floating-point contraction OFF: the
// quantizer's float arithmetic decides integer codes and must be the written
// sequence of IEEE operations (Sec. 3.2, rules (1) and (2); eq. (3)).
//
// Data layout.  A worker's vector u (d_pad floats) is cut into segments of 32
// consecutive coordinates; segment s becomes `bits` consecutive 32-bit words of
// the message (coordinate j occupies bits [j*bits, (j+1)*bits) of a
// little-endian bit stream, so a segment never straddles its words).  In the
// throughput-bound dense quantizer one thread owns one segment: it needs 8
// Philox blocks and emits whole words, so no cross-lane traffic is needed for
// packing; HBM accesses stay coalesced by staging a tile of 256 segments
// through LDS with a row pitch of 36 floats (pitch mod 32 banks = 4, so eight
// consecutive lanes reading 16 bytes each hit disjoint banks).  In the
// latency-bound launches (small-d fused exchange, sparse quantizer) a lane
// takes four coordinates = one Philox block, the codes meet in LDS and the
// words are assembled from there.
#include <hip/hip_runtime.h>

#include "lpc_device.h"
#include "lpc_internal.h"

namespace lpc {

namespace {

constexpr int kThreads = 256;
constexpr int kSegFloats = 32;
constexpr int kPitch = 36;
constexpr int kTileFloats = kThreads * kSegFloats;  // 8192 coordinates per workgroup

struct StatSinks {
  double *stat_part;
  double *stats;
  QParams *qparams;
  uint32_t *flags;
  uint32_t *n_clipped;
  double *stats_out;  // caller's buffer or nullptr
  int32_t stat_slots;
};

__device__ inline QParams qparams_from_delta(const QuantSpec &qs, float delta) {
  QParams q;
  const float rdelta = (float)(1.0 / (double)delta);
  const bool live = delta > 0.0f && isfinite(rdelta);
  q.delta = live ? delta : 0.0f;
  q.rdelta = live ? rdelta : 0.0f;
  q.thresh = delta * (float)((1 << (qs.bits - 1)) - 1);
  q.neg_edge = -(float)(1 << (qs.bits - 1)) * delta;
  return q;
}

// Fold the statistic partials of one vector in a fixed order (lane k takes slots k, k+64, ...; then
// a butterfly).  Called by one full wavefront; every lane returns the same four numbers.
__device__ inline void fold_stat_slots(const double *p, int32_t nslots, int lane, double &a, double &s,
                                       double &s2, double &b) {
  a = 0.0; s = 0.0; s2 = 0.0; b = 0.0;
  int32_t k = lane;
  // many slots (the MLP has several hundred): four of a lane's slots are requested before the first is added, in
  // the same order
  for (; k + 192 < nslots; k += 256) {
    double2 lo[4], hi[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      lo[q] = *reinterpret_cast<const double2 *>(p + (k + 64 * q) * 4);
      hi[q] = *reinterpret_cast<const double2 *>(p + (k + 64 * q) * 4 + 2);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) { a = fmax(a, lo[q].x); s += lo[q].y; s2 += hi[q].x; b += hi[q].y; }
  }
  for (; k < nslots; k += 64) {
    const double2 lo = *reinterpret_cast<const double2 *>(p + k * 4);
    const double2 hi = *reinterpret_cast<const double2 *>(p + k * 4 + 2);
    a = fmax(a, lo.x);
    s += lo.y;
    s2 += hi.x;
    b += hi.y;
  }
  a = wave_max(a); s = wave_sum(s); s2 = wave_sum(s2); b = wave_sum(b);
}

// Wave 0 of a workgroup publishes the statistics of its slice as one partial.  The fold of the partials
// is done by the consumer: the finalize kernel below, or the small-d exchange kernel itself.  (A
// "last workgroup folds" scheme needs a device-scope fence per workgroup, which on a multi-XCD part
// costs an L2 write-back each time; a tiny second launch is cheaper and just as deterministic.)
__device__ inline void publish_stats(const StatSinks &sk, int32_t vec, int32_t slot, double amax, double sum,
                                     double sumsq, double bad) {
  const int tid = threadIdx.x;
  if (tid < 64) {
    amax = wave_max(amax);
    sum = wave_sum(sum);
    sumsq = wave_sum(sumsq);
    bad = wave_sum(bad);
    if (tid == 0) {
      double *p = sk.stat_part + ((int64_t)vec * sk.stat_slots + slot) * 4;
      p[0] = amax; p[1] = sum; p[2] = sumsq; p[3] = bad;
    }
  }
}

// one wavefront per vector: fold its partials, store the statistics and the quantizer parameters
__global__ __launch_bounds__(64) void finalize_stats_kernel(StatSinks sk, QuantSpec qs, int32_t vec_begin,
                                                            int32_t nslots, int64_t d) {
  touch_kernel_arguments<(int)(sizeof(StatSinks) + sizeof(QuantSpec) + 16)>();
  const int32_t rel = blockIdx.x, vec = vec_begin + rel;
  double a, s, s2, b;
  fold_stat_slots(sk.stat_part + (int64_t)vec * sk.stat_slots * 4, nslots, threadIdx.x, a, s, s2, b);
  if (threadIdx.x == 0) {
    double *o = sk.stats + (int64_t)vec * 4;
    o[0] = a; o[1] = s; o[2] = s2; o[3] = b;
    if (sk.stats_out) {
      double *u = sk.stats_out + (int64_t)rel * 4;
      u[0] = a; u[1] = s; u[2] = s2; u[3] = b;
    }
    if (b > 0.0) atomicOr(&sk.flags[0], 1u);
    if (qs.enabled) {
      sk.qparams[vec] = make_qparams(qs, a, s, s2, d);
      sk.n_clipped[vec] = 0u;
    }
  }
}

// out[v][j] = scale * sum_p part[(v*parts + p)*d + j], j < d; zero for d <= j < d_pad.
// 64 columns per workgroup; the NWF wavefronts take interleaved parts and are combined in wavefront order.
template <int NWF>
__global__ __launch_bounds__(64 * NWF) void reduce_parts_kernel(const float *__restrict__ part, int32_t parts,
                                                                int64_t d, int64_t d_pad, float scale,
                                                                float *__restrict__ out, int64_t ld_out,
                                                                int32_t vec_begin, int32_t want_stats, StatSinks sk) {
  touch_kernel_arguments<(int)(64 + sizeof(StatSinks))>();
  __shared__ float red[NWF][64];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int32_t vec = blockIdx.y;
  const int64_t col = (int64_t)blockIdx.x * 64 + lane;
  float acc = 0.0f;
  if (col < d) {
    const float *src = part + (int64_t)vec * parts * d + col;
    for (int32_t p = wv; p < parts; p += 8 * NWF) {  // eight partial rows in flight per step
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = p + NWF * j < parts ? src[(int64_t)(p + NWF * j) * d] : 0.0f;
#pragma unroll
      for (int j = 0; j < 8; ++j) acc += v[j];
    }
  }
  red[wv][lane] = acc;
  __syncthreads();
  double amax = 0.0, sum = 0.0, sumsq = 0.0, bad = 0.0;
  if (wv == 0) {
    float v = red[0][lane];
#pragma unroll
    for (int q = 1; q < NWF; ++q) v += red[q][lane];
    v = v * scale;
    if (col >= d) v = 0.0f;
    if (col < d_pad) out[(int64_t)vec * ld_out + col] = v;
    if (isfinite(v)) {
      amax = fabs((double)v); sum = (double)v; sumsq = (double)v * (double)v;
    } else {
      bad = 1.0;
    }
  }
  if (want_stats != kStatsNone) publish_stats(sk, vec_begin + vec, blockIdx.x, amax, sum, sumsq, bad);
}

// statistics of rows of an existing matrix; each workgroup takes `chunk` columns (a multiple of 4; rows are 16-byte
// aligned), four 16-byte loads in flight per thread
__global__ __launch_bounds__(kThreads) void vector_stats_kernel(const float *__restrict__ U, int64_t ld, int64_t d,
                                                                int64_t chunk, int32_t vec_begin, StatSinks sk) {
  __shared__ double red[4][4];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int32_t vec = blockIdx.y;
  const int64_t lo = (int64_t)blockIdx.x * chunk;
  const int64_t hi = (lo + chunk < d) ? lo + chunk : d;
  const float *u = U + (int64_t)vec * ld + lo;
  const int64_t len = hi - lo, n4 = len / 4;
  double sum = 0.0, sumsq = 0.0;
  float fmx = 0.0f;
  uint32_t nbad = 0;
  auto take = [&](float x) {
    const bool fin = isfinite(x);
    const float y = fin ? x : 0.0f;  // a zero adds nothing to any of the three
    nbad += fin ? 0u : 1u;
    fmx = fmaxf(fmx, fabsf(y)); sum += (double)y; sumsq += (double)y * (double)y;
  };
  for (int64_t i = tid; i < n4; i += 4 * kThreads) {
    float4 t[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int64_t k = i + q * kThreads;
      t[q] = *reinterpret_cast<const float4 *>(u + 4 * (k < n4 ? k : i));
      if (k >= n4) t[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) { take(t[q].x); take(t[q].y); take(t[q].z); take(t[q].w); }
  }
  if (tid < (int)(len - 4 * n4)) take(u[4 * n4 + tid]);  // the last one to three columns of the row
  double amax = (double)fmx, bad = (double)nbad;
  amax = wave_max(amax); sum = wave_sum(sum); sumsq = wave_sum(sumsq); bad = wave_sum(bad);
  if (lane == 0) { red[wv][0] = amax; red[wv][1] = sum; red[wv][2] = sumsq; red[wv][3] = bad; }
  __syncthreads();
  amax = 0.0; sum = 0.0; sumsq = 0.0; bad = 0.0;
  if (tid == 0) {
    for (int k = 0; k < 4; ++k) { amax = fmax(amax, red[k][0]); sum += red[k][1]; sumsq += red[k][2]; bad += red[k][3]; }
  }
  publish_stats(sk, vec_begin + vec, blockIdx.x, amax, sum, sumsq, bad);
}

// statistic partials of short column ranges of rows of U: workgroup (r, vec) reduces range r of vector vec
__global__ __launch_bounds__(kThreads) void range_stats_kernel(const float *__restrict__ U, int64_t ld, StatRange rg,
                                                               int32_t vec_begin, int32_t slot0, StatSinks sk) {
  __shared__ double red[4][4];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int32_t vec = blockIdx.y;
  const float *u = U + (int64_t)vec * ld + rg.begin[blockIdx.x];
  const int64_t len = rg.len[blockIdx.x];
  double sum = 0.0, sumsq = 0.0, bad = 0.0;
  float fmx = 0.0f;
  for (int64_t j = tid; j < len; j += 8 * kThreads) {  // eight elements in flight per thread
    float v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = j + q * kThreads < len ? u[j + q * kThreads] : 0.0f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      if (isfinite(v[q])) {
        fmx = fmaxf(fmx, fabsf(v[q])); sum += (double)v[q]; sumsq += (double)v[q] * (double)v[q];
      } else {
        bad += 1.0;
      }
    }
  }
  fmx = wave_max(fmx);
  sum = wave_sum(sum); sumsq = wave_sum(sumsq); bad = wave_sum(bad);
  if (lane == 0) { red[wv][0] = (double)fmx; red[wv][1] = sum; red[wv][2] = sumsq; red[wv][3] = bad; }
  __syncthreads();
  if (tid == 0) {
    double amax = 0.0;
    sum = 0.0; sumsq = 0.0; bad = 0.0;
    for (int k = 0; k < 4; ++k) { amax = fmax(amax, red[k][0]); sum += red[k][1]; sumsq += red[k][2]; bad += red[k][3]; }
    double *p = sk.stat_part + ((int64_t)(vec_begin + vec) * sk.stat_slots + slot0 + blockIdx.x) * 4;
    p[0] = amax; p[1] = sum; p[2] = sumsq; p[3] = bad;
  }
}

__global__ void prepare_qparams_kernel(const double *stats, const float *delta_in, int32_t nvec, int64_t d,
                                       QuantSpec qs, QParams *qp, uint32_t *n_clipped, uint32_t *flags) {
  const int v = blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= nvec) return;
  if (delta_in) {
    qp[v] = qparams_from_delta(qs, delta_in[v]);
  } else {
    const double *s = stats + (int64_t)v * 4;
    qp[v] = make_qparams(qs, s[0], s[1], s[2], d);
  }
  if (stats && stats[(int64_t)v * 4 + 3] > 0.0) atomicOr(&flags[0], 1u);
  n_clipped[v] = 0u;
}

// Sec. 3.2 rules (1), (2) with the scale of eq. (3) for four consecutive coordinates 4*block .. 4*block+3 of
// one worker's vector (they share one Philox block): code[t] receives the integer codes; returns the number
// of coordinates outside dom(delta, b).  All arithmetic is fp32 without contraction:
//   s = u*(1/delta), clamp to [-2^(b-1), 2^(b-1)-1], lo = floor(s), frac = s - lo (exact),
//   U = (word >> 8)*2^-24, code = lo + (U < frac).
// COUNT = false leaves the clip count out (it returns 0): the count is wanted by evaluation runs only.
// SKIP: on-grid groups (zeros in particular) draw no random numbers -- worth a branch where vectors are mostly
// zero (sparse data), a loss where they are dense (the branches keep the compiler from interleaving the eight
// generator chains of a segment).
template <int B, bool COUNT = true, bool SKIP = true>
__device__ __forceinline__ uint32_t quantize_four(const float4 v4, const QParams &q, const StreamKey &key,
                                                  uint32_t worker, uint32_t block, int32_t (&code)[4]) {
  const float hi = (float)((1 << (B - 1)) - 1);
  const float lo = -(float)(1 << (B - 1));
  const bool count = COUNT && q.delta > 0.0f;
  uint32_t clipped = 0;
  const float vals[4] = {v4.x, v4.y, v4.z, v4.w};
  float base[4], frac[4];
  bool any = false;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    float s = vals[t] * q.rdelta;        // position on the grid
    s = fminf(fmaxf(s, lo), hi);         // rule (2): project onto the hull
    base[t] = floorf(s);
    frac[t] = s - base[t];               // exact
    any = any || (frac[t] != 0.0f);
    if (count && (vals[t] > q.thresh || vals[t] < q.neg_edge)) ++clipped;
  }
  uint32_t rnd[4] = {0u, 0u, 0u, 0u};
  if (!SKIP || any) {  // an on-grid value keeps its code whatever the draw
    const Philox4 blk = stream_block(key, kTagQuant, worker, block);
    rnd[0] = blk.x; rnd[1] = blk.y; rnd[2] = blk.z; rnd[3] = blk.w;
  }
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const float unif = (float)(rnd[t] >> 8) * 0x1.0p-24f;
    code[t] = (int32_t)base[t] + ((unif < frac[t]) ? 1 : 0);  // rule (1)
    if (!(q.delta > 0.0f)) code[t] = 0;  // an all-zero vector: every code is 0, also where the vector holds a NaN
  }
  return clipped;
}

// Quantize the 32 coordinates of segment `seg` of one worker's vector and store its B packed words at dst.
// load4(k) returns coordinates 4k..4k+3.  Returns the number of coordinates outside dom(delta, b).
template <int B, bool COUNT, bool SKIP, class Load4>
__device__ __forceinline__ uint32_t quantize_segment(Load4 load4, const QParams &q, const StreamKey &key,
                                                     uint32_t worker, int64_t seg, uint32_t *__restrict__ dst) {
  constexpr uint32_t mask = (B >= 32) ? 0xFFFFFFFFu : ((1u << B) - 1u);
  uint32_t clipped = 0;
  uint32_t words[B];
  uint64_t bitbuf = 0;
  int nb = 0, wi = 0;
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    int32_t code[4];
    clipped += quantize_four<B, COUNT, SKIP>(load4(k), q, key, worker, (uint32_t)(seg * 8 + k), code);
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      bitbuf |= (uint64_t)((uint32_t)code[t] & mask) << nb;
      nb += B;
      if (nb >= 32) {
        words[wi++] = (uint32_t)bitbuf;
        bitbuf >>= 32;
        nb -= 32;
      }
    }
  }
  if constexpr (B % 4 == 0) {
#pragma unroll
    for (int i = 0; i < B; i += 4)
      *reinterpret_cast<uint4 *>(dst + i) = make_uint4(words[i], words[i + 1], words[i + 2], words[i + 3]);
  } else if constexpr (B % 2 == 0) {
#pragma unroll
    for (int i = 0; i < B; i += 2) *reinterpret_cast<uint2 *>(dst + i) = make_uint2(words[i], words[i + 1]);
  } else {
#pragma unroll
    for (int i = 0; i < B; ++i) dst[i] = words[i];
  }
  return clipped;
}

// Word w (of B) of a segment's message from its 32 codes: stream bits [32w, 32w+32), code c at bits [cB, cB+B).
template <int B>
__device__ __forceinline__ uint32_t assemble_word(const int32_t *__restrict__ codes, int w) {
  constexpr uint32_t mask = (1u << B) - 1u;
  const int bit0 = 32 * w, c0 = bit0 / B;
  uint32_t word = 0u;
#pragma unroll
  for (int t = 0; t < 32 / B + 2; ++t) {
    const int c = c0 + t;
    if (c < 32 && c * B < bit0 + 32) {
      const uint32_t field = (uint32_t)codes[c] & mask;
      const int sh = c * B - bit0;
      word |= sh >= 0 ? (field << sh) : (field >> (-sh));
    }
  }
  return word;
}

// ---------------------------------------------------------------------------
// Quantize + pack.  grid = (tiles of 8192 coordinates, N workers).
template <int B, bool COUNT, bool SKIP>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const float *__restrict__ U, int64_t d, int64_t d_pad,
                                                            const QParams *__restrict__ qp, StreamKey key,
                                                            uint32_t *__restrict__ packed, int64_t W,
                                                            float *__restrict__ delta_out,
                                                            uint32_t *__restrict__ n_clipped) {
  __shared__ __attribute__((aligned(16))) float tile[kThreads * kPitch];
  const int tid = threadIdx.x;
  const uint32_t worker = blockIdx.y;
  const int64_t tile_base = (int64_t)blockIdx.x * kTileFloats;
  const float *u = U + (int64_t)worker * d_pad;
  if (tile_base + kTileFloats <= d) {  // uniform: a tile inside the vector needs no checks
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int e = r * kThreads + tid;
      *reinterpret_cast<float4 *>(&tile[(e >> 3) * kPitch + (e & 7) * 4]) =
          *reinterpret_cast<const float4 *>(u + tile_base + (int64_t)e * 4);
    }
  } else {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int e = r * kThreads + tid;
      const int64_t j = tile_base + (int64_t)e * 4;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j < d_pad) {
        v = *reinterpret_cast<const float4 *>(u + j);
        if (j + 3 >= d) {  // the zero padding of the last segment carries code 0 whatever the buffer holds
          if (j + 0 >= d) v.x = 0.f;
          if (j + 1 >= d) v.y = 0.f;
          if (j + 2 >= d) v.z = 0.f;
          v.w = 0.f;
        }
      }
      *reinterpret_cast<float4 *>(&tile[(e >> 3) * kPitch + (e & 7) * 4]) = v;
    }
  }
  __syncthreads();
  const QParams q = qp[worker];
  if (blockIdx.x == 0 && tid == 0) delta_out[worker] = q.delta;
  const int64_t seg = tile_base / kSegFloats + tid;
  const bool active = seg * kSegFloats < d_pad;
  uint32_t clipped = 0;
  if (active) {
    const float *mine = &tile[tid * kPitch];
    clipped = quantize_segment<B, COUNT, SKIP>([&](int k) { return *reinterpret_cast<const float4 *>(mine + k * 4); }, q, key,
                                         worker, seg, packed + (int64_t)worker * W + seg * B);
  }
  if (COUNT) {
    clipped = wave_sum(clipped);
    if ((tid & 63) == 0 && clipped) atomicAdd(&n_clipped[worker], clipped);
  }
}

// Quantize + pack for the bit widths whose words hold whole groups of four codes (B = 2, 4, 8): one packed word per
// thread.  A thread reads the 32/B consecutive coordinates of its word straight from memory (8/B loads of 16 bytes),
// draws their 8/B Philox blocks and stores the word; a wavefront's stores are 256 contiguous bytes.  No LDS and no
// barrier, so the registers alone bound the number of resident wavefronts.  The pass is bound by the vector unit:
// one generator block (18 64-bit multiply-adds, 35 exclusive-ors) and about 45 other instructions per four
// coordinates; with neither loads nor stores it runs 6 % faster.  Measured and dropped: workgroups that walk the
// message with a grid stride and request their next word's coordinates ahead (8 to 10 % slower than a thread per
// word: fresh workgroups cost less than the loop).  Codes, draws and bit layout are those of quantize_kernel.
// grid = (words of a message / kThreads, N workers).
template <int B, bool COUNT, bool SKIP>
__global__ __launch_bounds__(kThreads) void quantize_word_kernel(const float *__restrict__ U, int64_t d, int64_t d_pad,
                                                                 const QParams *__restrict__ qp, StreamKey key,
                                                                 uint32_t *__restrict__ packed, int64_t W,
                                                                 float *__restrict__ delta_out,
                                                                 uint32_t *__restrict__ n_clipped) {
  touch_kernel_arguments<(int)(80)>();
  static_assert(B == 2 || B == 4 || B == 8, "a word holds whole groups of four codes");
  constexpr int kCoords = 32 / B;  // coordinates per word
  constexpr int kBlocks = kCoords / 4;
  constexpr uint32_t mask = (1u << B) - 1u;
  const uint32_t worker = blockIdx.y;
  const QParams q = qp[worker];
  if (blockIdx.x == 0 && threadIdx.x == 0) delta_out[worker] = q.delta;
  const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;  // word of the message
  uint32_t clipped = 0;
  if (t < W) {  // W * kCoords == d_pad: every load stays inside the vector's d_pad floats
    const float *u = U + (int64_t)worker * d_pad;
    float4 v[kBlocks];
#pragma unroll
    for (int k = 0; k < kBlocks; ++k) v[k] = *reinterpret_cast<const float4 *>(u + t * kCoords + 4 * k);
    const int64_t j0 = t * kCoords;
    if (j0 + kCoords > d) {  // the zero padding of the last segment carries code 0 whatever the buffer holds
#pragma unroll
      for (int k = 0; k < kBlocks; ++k) {
        const int64_t j = j0 + 4 * k;
        if (j + 0 >= d) v[k].x = 0.f;
        if (j + 1 >= d) v[k].y = 0.f;
        if (j + 2 >= d) v[k].z = 0.f;
        if (j + 3 >= d) v[k].w = 0.f;
      }
    }
    uint32_t word = 0u;
    if constexpr (!COUNT && !SKIP) {
      // The arithmetic of quantize_four with a code travelling as code + 2^(B-1), a B-bit non-negative number that
      // one shift-or places in the word; flipping bit B-1 of every field at the end gives the two's-complement
      // fields.
      constexpr uint32_t kBias = 1u << (B - 1);
      constexpr uint32_t kFlip = (uint32_t)(0xFFFFFFFFull / mask) * kBias;  // bit B-1 of every field
      const float lo = -(float)(1 << (B - 1)), hi = (float)((1 << (B - 1)) - 1);
#pragma unroll
      for (int k = 0; k < kBlocks; ++k) {
        const float vals[4] = {v[k].x, v[k].y, v[k].z, v[k].w};
        float base[4], frac[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float sc = fminf(fmaxf(vals[c] * q.rdelta, lo), hi);
          base[c] = floorf(sc);
          frac[c] = sc - base[c];
        }
        const Philox4 blk = stream_block(key, kTagQuant, worker, (uint32_t)(j0 / 4 + k));
        const uint32_t rnd[4] = {blk.x, blk.y, blk.z, blk.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const float unif = (float)(rnd[c] >> 8) * 0x1.0p-24f;
          const uint32_t biased = (uint32_t)((int32_t)base[c] + (int32_t)kBias + ((unif < frac[c]) ? 1 : 0));
          word |= biased << ((4 * k + c) * B);
        }
      }
      word ^= kFlip;
      if (!(q.delta > 0.0f)) word = 0u;  // an all-zero vector: every code is 0, also where the vector holds a NaN
    } else {
#pragma unroll
      for (int k = 0; k < kBlocks; ++k) {
        int32_t code[4];
        clipped += quantize_four<B, COUNT, SKIP>(v[k], q, key, worker, (uint32_t)(j0 / 4 + k), code);
#pragma unroll
        for (int c = 0; c < 4; ++c) word |= ((uint32_t)code[c] & mask) << ((4 * k + c) * B);
      }
    }
    packed[(int64_t)worker * W + t] = word;
  }
  if (COUNT) {
    clipped = wave_sum(clipped);
    if ((threadIdx.x & 63) == 0 && clipped) atomicAdd(&n_clipped[worker], clipped);
  }
}

// ---------------------------------------------------------------------------
// Receiver: unpack, eq. (4), optional fused proximal step.
template <int B>
__device__ __forceinline__ void load_words(const uint32_t *__restrict__ src, uint32_t (&words)[B]) {
  if constexpr (B % 4 == 0) {
#pragma unroll
    for (int i = 0; i < B; i += 4) {
      const uint4 t = *reinterpret_cast<const uint4 *>(src + i);
      words[i] = t.x; words[i + 1] = t.y; words[i + 2] = t.z; words[i + 3] = t.w;
    }
  } else if constexpr (B % 2 == 0) {
#pragma unroll
    for (int i = 0; i < B; i += 2) {
      const uint2 t = *reinterpret_cast<const uint2 *>(src + i);
      words[i] = t.x; words[i + 1] = t.y;
    }
  } else {
#pragma unroll
    for (int i = 0; i < B; ++i) words[i] = src[i];
  }
}

constexpr int kQuarterThreads = 128;

// acc[c] = fma(delta, code_c, acc[c]) for the 32 codes of one segment; returns the OR of the words
template <int B>
__device__ __forceinline__ uint32_t accumulate_words(const uint32_t (&words)[B], float delta, float (&acc)[32]) {
  uint32_t any = 0u;
#pragma unroll
  for (int i = 0; i < B; ++i) any |= words[i];
#pragma unroll
  for (int c = 0; c < 32; ++c) {
    const int p = c * B, wi = p >> 5, sh = p & 31;
    uint32_t field = words[wi] >> sh;
    if (sh + B > 32) field |= words[wi + 1] << (32 - sh);
    const int32_t code = (int32_t)(field << (32 - B)) >> (32 - B);  // sign-extend the B-bit field
    acc[c] = __builtin_fmaf(delta, (float)code, acc[c]);
  }
  return any;
}

template <int B>
__device__ __forceinline__ void unpack_accumulate(const uint32_t *__restrict__ src, float delta, float (&acc)[32]) {
  uint32_t words[B];
  load_words<B>(src, words);
  accumulate_words<B>(words, delta, acc);
}

struct ProxArgs {
  const float *mu;
  float *w;
  float step, thr, shrink;
  // sparse inner iteration: consumed non-zero words are set back to zero (rezero aliases the packed
  // messages, N <= 64) and the touched-segment bitmap is cleared
  uint32_t *rezero;
  uint32_t *touched;
  int64_t bitmap_words;
};

// The receiver for the bit widths that do not divide a word.  TPB threads per workgroup (one segment each): 256
// for long vectors, 64 when that would leave CUs without work
template <int B, bool PROX, int TPB>
__global__ __launch_bounds__(TPB) void dequantize_kernel(const uint32_t *packed, int64_t W,
                                                              const float *__restrict__ delta, int32_t N, int64_t d,
                                                              int64_t d_pad, float *__restrict__ u_avg, ProxArgs pa) {
  __shared__ __attribute__((aligned(16))) float tile[TPB * kPitch];
  const int tid = threadIdx.x;
  const int64_t tile_base = (int64_t)blockIdx.x * (TPB * kSegFloats);
  const int64_t seg = tile_base / kSegFloats + tid;
  // the proximal step's operands are requested before the messages are unpacked (one round trip, not two)
  float4 w_pre[8], mu_pre[8];
  if constexpr (PROX) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      const int64_t j = tile_base + (int64_t)(r * TPB + tid) * 4;
      w_pre[r] = mu_pre[r] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j + 4 <= d) {
        mu_pre[r] = *reinterpret_cast<const float4 *>(pa.mu + j);
        w_pre[r] = *reinterpret_cast<const float4 *>(pa.w + j);
      }
    }
  }
  if (seg * kSegFloats < d_pad) {
    float acc[32];
#pragma unroll
    for (int c = 0; c < 32; ++c) acc[c] = 0.0f;
    // several messages in flight at a time (as many as the word count lets the registers hold);
    // accumulation stays in worker order
    constexpr int kInFlight = B <= 2 ? 16 : (B <= 8 ? 8 : 4);  // measured for B = 4: 8 in flight 22.5 us, 16: 29.2, 4: 23.6
    uint64_t nonzero = 0;
    for (int32_t i0 = 0; i0 < N; i0 += kInFlight) {
      uint32_t wds[kInFlight][B];
#pragma unroll
      for (int q = 0; q < kInFlight; ++q) {
        const int32_t i = i0 + q < N ? i0 + q : N - 1;  // past the end: a repeated load, ignored below
        load_words<B>(packed + (int64_t)i * W + seg * B, wds[q]);
      }
#pragma unroll
      for (int q = 0; q < kInFlight; ++q) {
        if (i0 + q < N) {
          if (accumulate_words<B>(wds[q], delta[i0 + q], acc)) nonzero |= 1ull << ((i0 + q) & 63);
        }
      }
    }
    if constexpr (PROX) {
      if (pa.rezero) {
        while (nonzero) {
          const int k = __builtin_ctzll(nonzero);
          nonzero &= nonzero - 1;
          uint32_t *z = pa.rezero + (int64_t)k * W + seg * B;
#pragma unroll
          for (int q = 0; q < B; ++q) z[q] = 0u;
        }
        // the 32 segments of one bitmap word belong to this wavefront, and no pass reads the bitmap here
        if ((seg & 31) == 0)
          for (int32_t k = 0; k < N; ++k) pa.touched[(int64_t)k * pa.bitmap_words + (seg >> 5)] = 0u;
      }
    }
    const float inv_n = 1.0f / (float)N;
#pragma unroll
    for (int k = 0; k < 8; ++k)
      *reinterpret_cast<float4 *>(&tile[tid * kPitch + k * 4]) =
          make_float4(acc[4 * k] * inv_n, acc[4 * k + 1] * inv_n, acc[4 * k + 2] * inv_n, acc[4 * k + 3] * inv_n);
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int e = r * TPB + tid;
    const int64_t j = tile_base + (int64_t)e * 4;
    if (j >= d) continue;
    const float4 a = *reinterpret_cast<const float4 *>(&tile[(e >> 3) * kPitch + (e & 7) * 4]);
    const float av[4] = {a.x, a.y, a.z, a.w};
    if (j + 4 <= d) {
      if (u_avg) *reinterpret_cast<float4 *>(u_avg + j) = a;
      if constexpr (PROX) {
        const float4 m = mu_pre[r];
        float4 w = w_pre[r];
        w.x = prox_scalar(w.x, a.x + m.x, pa.step, pa.thr, pa.shrink);
        w.y = prox_scalar(w.y, a.y + m.y, pa.step, pa.thr, pa.shrink);
        w.z = prox_scalar(w.z, a.z + m.z, pa.step, pa.thr, pa.shrink);
        w.w = prox_scalar(w.w, a.w + m.w, pa.step, pa.thr, pa.shrink);
        *reinterpret_cast<float4 *>(pa.w + j) = w;
      }
    } else {
      for (int t = 0; t < 4 && j + t < d; ++t) {
        if (u_avg) u_avg[j + t] = av[t];
        if constexpr (PROX) pa.w[j + t] = prox_scalar(pa.w[j + t], av[t] + pa.mu[j + t], pa.step, pa.thr, pa.shrink);
      }
    }
  }
}

// The receiver for B in {2, 4}: eight coordinates per thread, which lie in one word of
// each message (8B divides 32).  Four times as many threads as one-segment-per-thread, each with a quarter
// of the arithmetic between its loads and its stores, and a thread's eight results are contiguous, so no
// transposition through LDS.  Accumulation order (worker 0 first) and every operation are those of
// dequantize_kernel.  The threads that share a word sit in one wavefront and load it in one instruction,
// which has returned before the thread at bit 0 sets the word back to zero.
template <int B, bool PROX>
__global__ __launch_bounds__(kQuarterThreads) void dequantize_quarter_kernel(const uint32_t *packed, int64_t W,
                                                                           const float *__restrict__ delta,
                                                                           int32_t N, int64_t d, int64_t d_pad,
                                                                           float *__restrict__ u_avg, ProxArgs pa) {
  touch_kernel_arguments<(int)(56 + sizeof(ProxArgs))>();
  static_assert(32 % (8 * B) == 0, "eight codes in one word");
  const int64_t q = (int64_t)blockIdx.x * kQuarterThreads + threadIdx.x;
  const int64_t j = q * 8;
  if (j >= d_pad) return;
  const bool whole = j + 8 <= d;
  float4 w_pre[2], mu_pre[2];
  if constexpr (PROX) {
    if (whole) {
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        mu_pre[r] = *reinterpret_cast<const float4 *>(pa.mu + j + 4 * r);
        w_pre[r] = *reinterpret_cast<const float4 *>(pa.w + j + 4 * r);
      }
    }
  }
  const int64_t word = (q * B) >> 2;
  const int shift = (int)((q * 8 * B) & 31);
  float acc[8];
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] = 0.0f;
  constexpr int kInFlight = 16;
  uint64_t nonzero = 0;
  for (int32_t i0 = 0; i0 < N; i0 += kInFlight) {
    uint32_t wd[kInFlight];
#pragma unroll
    for (int k = 0; k < kInFlight; ++k) {
      const int32_t i = i0 + k < N ? i0 + k : N - 1;
      wd[k] = packed[(int64_t)i * W + word];
    }
#pragma unroll
    for (int k = 0; k < kInFlight; ++k) {
      if (i0 + k < N) {
        const float dl = delta[i0 + k];
        if (wd[k]) nonzero |= 1ull << ((i0 + k) & 63);
        const uint32_t part = wd[k] >> shift;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
          const int32_t code = (int32_t)(part << (32 - B - c * B)) >> (32 - B);
          acc[c] = __builtin_fmaf(dl, (float)code, acc[c]);
        }
      }
    }
  }
  if constexpr (PROX) {
    if (pa.rezero) {
      if (shift == 0) {
        while (nonzero) {
          const int k = __builtin_ctzll(nonzero);
          nonzero &= nonzero - 1;
          pa.rezero[(int64_t)k * W + word] = 0u;
        }
      }
      if ((q & 127) == 0)
        for (int32_t k = 0; k < N; ++k) pa.touched[(int64_t)k * pa.bitmap_words + (q >> 7)] = 0u;
    }
  }
  const float inv_n = 1.0f / (float)N;
#pragma unroll
  for (int c = 0; c < 8; ++c) acc[c] *= inv_n;
  if (whole) {
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const float4 a = make_float4(acc[4 * r], acc[4 * r + 1], acc[4 * r + 2], acc[4 * r + 3]);
      if (u_avg) *reinterpret_cast<float4 *>(u_avg + j + 4 * r) = a;
      if constexpr (PROX) {
        const float4 m = mu_pre[r];
        float4 w = w_pre[r];
        w.x = prox_scalar(w.x, a.x + m.x, pa.step, pa.thr, pa.shrink);
        w.y = prox_scalar(w.y, a.y + m.y, pa.step, pa.thr, pa.shrink);
        w.z = prox_scalar(w.z, a.z + m.z, pa.step, pa.thr, pa.shrink);
        w.w = prox_scalar(w.w, a.w + m.w, pa.step, pa.thr, pa.shrink);
        *reinterpret_cast<float4 *>(pa.w + j + 4 * r) = w;
      }
    }
  } else {
    for (int t = 0; t < 8 && j + t < d; ++t) {
      if (u_avg) u_avg[j + t] = acc[t];
      if constexpr (PROX) pa.w[j + t] = prox_scalar(pa.w[j + t], acc[t] + pa.mu[j + t], pa.step, pa.thr, pa.shrink);
    }
  }
}

// ---------------------------------------------------------------------------
// Sparse inner iteration (CSR rows): u^i is non-zero only in the always-visited head columns and in the
// 32-coordinate segments marked in the worker's bitmap.  A zero coordinate adds nothing to the statistics,
// quantizes to code 0 without a random draw and is never clipped, so visiting only the marked segments gives
// the results of the dense passes.  One thread per (segment, worker) in all three kernels.
struct SparseArgs {
  float *U;                 // [N][d_pad]
  float *planes;            // [N][parts-1][d_pad]: tail contributions of the worker pass's workgroups 1..parts-1
  const float *head_part;   // [N][parts][head]: partial head rows of the worker pass
  uint32_t *touched;        // [N][bitmap_words]
  uint32_t *touched_parts;  // [N][parts-1][bitmap_words]: segments marked by the worker pass's workgroups 1..parts-1
  int64_t d_pad, W, bitmap_words;
  int32_t head, parts, N;
};

__device__ __forceinline__ bool segment_marked(const uint32_t *bm, int64_t seg) {
  return (bm[seg >> 5] >> (seg & 31)) & 1u;
}

// A wavefront owns kWaveWords words of a worker's bitmap, first_word + k*stride for k < kWaveWords (strided so
// that every wavefront gets its share of the frequent low columns), i.e. kWaveSegs tail segments.  The marked
// ones are compacted into `list` (LDS, kWaveSegs entries per wavefront) so that the lanes share them evenly;
// returns their number.
// A segment is one 128-byte line: it is always moved by eight adjacent lanes with 16 bytes each (one request
// per line); a lane that walks a line of its own costs a request per 16 bytes.
constexpr int kWaveWords = 8;
constexpr int kWaveSegs = kWaveWords * 32;

__device__ __forceinline__ int32_t compact_marked(const uint32_t *__restrict__ bm, int64_t bitmap_words,
                                                  int64_t first_word, int64_t stride, int64_t total_segs, int lane,
                                                  int32_t *__restrict__ list) {
  const int64_t wi = first_word + lane * stride;
  const uint32_t word = (lane < kWaveWords && wi < bitmap_words) ? bm[wi] : 0u;
  int32_t n = 0;
#pragma unroll 4
  for (int c = 0; c < kWaveWords / 2; ++c) {  // chunk c = the 64 segments of words 2c, 2c+1 of this wavefront
    const int k = 2 * c + (lane >> 5);
    const uint32_t w = __shfl(word, k, 64);
    const int64_t seg = (first_word + k * stride) * 32 + (lane & 31);
    const bool marked = ((w >> (lane & 31)) & 1u) && seg < total_segs;
    const uint64_t m = __ballot(marked);
    if (marked) list[n + __popcll(m & ((1ull << lane) - 1ull))] = (int32_t)seg;
    n += __popcll(m);
  }
  return n;
}

// The same over the union of the bitmaps of the worker pass's workgroups ("planes"; plane 0's bitmap is the
// worker's own, which receives the union, the others are cleared): masks[k] has bit p set when plane p holds a
// contribution to listed segment k.  Every bitmap word belongs to exactly one wavefront of the launch.
constexpr int kMaxPlanes = 8;

__device__ __forceinline__ int32_t compact_marked_planes(uint32_t *bm0, uint32_t *bmp, int32_t parts,
                                                         int64_t bitmap_words, int64_t first_word, int64_t stride,
                                                         int64_t total_segs, int lane, int32_t *__restrict__ list,
                                                         uint32_t *__restrict__ masks) {
  const int64_t wi = first_word + lane * stride;
  const bool valid = lane < kWaveWords && wi < bitmap_words;
  uint32_t w[kMaxPlanes];
  w[0] = valid ? bm0[wi] : 0u;
  uint32_t uni = w[0];
#pragma unroll
  for (int p = 1; p < kMaxPlanes; ++p) {
    w[p] = (valid && p < parts) ? bmp[(int64_t)(p - 1) * bitmap_words + wi] : 0u;
    uni |= w[p];
  }
  if (valid && uni != w[0]) bm0[wi] = uni;
#pragma unroll
  for (int p = 1; p < kMaxPlanes; ++p)
    if (w[p]) bmp[(int64_t)(p - 1) * bitmap_words + wi] = 0u;
  int32_t n = 0;
#pragma unroll 4
  for (int c = 0; c < kWaveWords / 2; ++c) {  // chunk c = the 64 segments of words 2c, 2c+1 of this wavefront
    const int k = 2 * c + (lane >> 5);
    const int bit = lane & 31;
    const uint32_t wu = __shfl(uni, k, 64);
    uint32_t mask = 0u;
#pragma unroll
    for (int p = 0; p < kMaxPlanes; ++p) mask |= ((__shfl(w[p], k, 64) >> bit) & 1u) << p;
    const int64_t seg = (first_word + k * stride) * 32 + bit;
    const bool marked = ((wu >> bit) & 1u) && seg < total_segs;
    const uint64_t m = __ballot(marked);
    if (marked) {
      const int32_t at = n + __popcll(m & ((1ull << lane) - 1ull));
      list[at] = (int32_t)seg;
      masks[at] = mask;
    }
    n += __popcll(m);
  }
  return n;
}

// Statistic partials of u^i.  Workgroups [0, head/1024) of a worker fold the head columns from the partial rows
// of the worker pass (fixed order, one float4 per thread, coalesced) into U; in the others every wavefront
// visits the marked ones of its kWaveSegs tail segments.
__global__ __launch_bounds__(kThreads) void sparse_stats_kernel(SparseArgs a, StatSinks sk) {
  touch_kernel_arguments<(int)(sizeof(SparseArgs) + sizeof(StatSinks))>();
  __shared__ double red[4][4];
  __shared__ int32_t list[4][kWaveSegs];
  __shared__ uint32_t masks[4][kWaveSegs];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int32_t worker = blockIdx.y;
  const int32_t head_wgs = a.head / (4 * kThreads);
  float *urow = a.U + (int64_t)worker * a.d_pad;
  double sum = 0.0, sumsq = 0.0, bad = 0.0;
  float fmx = 0.0f;
  auto take = [&](float x) {
    if (isfinite(x)) {
      fmx = fmaxf(fmx, fabsf(x)); sum += (double)x; sumsq += (double)x * (double)x;
    } else {
      bad += 1.0;
    }
  };
  if ((int32_t)blockIdx.x < head_wgs) {
    const int64_t j = ((int64_t)blockIdx.x * kThreads + tid) * 4;
    const float *src = a.head_part + (int64_t)worker * a.parts * a.head + j;
    float4 v = *reinterpret_cast<const float4 *>(src);
    for (int32_t p0 = 1; p0 < a.parts; p0 += 4) {  // four partial rows in flight, added in order
      float4 t[4];
#pragma unroll
      for (int q = 0; q < 4; ++q)
        t[q] = p0 + q < a.parts ? *reinterpret_cast<const float4 *>(src + (int64_t)(p0 + q) * a.head)
                                : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (p0 + q < a.parts) { v.x += t[q].x; v.y += t[q].y; v.z += t[q].z; v.w += t[q].w; }
    }
    *reinterpret_cast<float4 *>(urow + j) = v;
    take(v.x); take(v.y); take(v.z); take(v.w);
  } else {
    const int64_t stride = (int64_t)(gridDim.x - head_wgs) * 4;  // tail wavefronts of this worker
    const int64_t first_word = a.head / (kSegFloats * 32) + ((int64_t)blockIdx.x - head_wgs) * 4 + wv;
    const int32_t n = compact_marked_planes(
        a.touched + (int64_t)worker * a.bitmap_words,
        a.touched_parts + (int64_t)worker * (a.parts - 1) * a.bitmap_words, a.parts, a.bitmap_words, first_word, stride,
        a.d_pad / kSegFloats, lane, list[wv], masks[wv]);
    __builtin_amdgcn_wave_barrier();
    // eight lanes per segment, 32 segments (four independent loads per lane) per step.  A segment's value is the
    // sum of the planes that hold it, in plane order (plane 0 = the row of U, which receives the sum; the other
    // planes are set back to zero).  Nearly every segment lies in one plane only: that plane is read first, the
    // rare further ones in a loop the wavefront enters only when some lane needs it.
    float *pl = a.planes + (int64_t)worker * (a.parts - 1) * a.d_pad;
    for (int32_t i0 = 0; i0 < n; i0 += 32) {
      float4 v[4];
      int64_t at[4];
      uint32_t mk[4], rest_any = 0u;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int32_t i = i0 + q * 8 + (lane >> 3);
        at[q] = -1; mk[q] = 0u;
        v[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < n) {
          at[q] = (int64_t)list[wv][i] * kSegFloats + (lane & 7) * 4;
          mk[q] = masks[wv][i];
          const int first = __builtin_ctz(mk[q]);  // a listed segment lies in at least one plane
          const float *src = first == 0 ? urow + at[q] : pl + (int64_t)(first - 1) * a.d_pad + at[q];
          v[q] = *reinterpret_cast<const float4 *>(src);
          rest_any |= mk[q] & (mk[q] - 1u);
        }
      }
      if (__ballot(rest_any != 0u) != 0ull) {
        // every further plane's copy is requested before the first is added (one trip to memory, not one per plane:
        // the segments of the frequent low columns lie in most planes); the additions keep plane order
        float4 t[kMaxPlanes - 1][4];
#pragma unroll
        for (int p = 1; p < kMaxPlanes; ++p) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const uint32_t rest = mk[q] & (mk[q] - 1u);
            t[p - 1][q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (p < a.parts && ((rest >> p) & 1u))
              t[p - 1][q] = *reinterpret_cast<const float4 *>(pl + (int64_t)(p - 1) * a.d_pad + at[q]);
          }
        }
#pragma unroll
        for (int p = 1; p < kMaxPlanes; ++p) {
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const uint32_t rest = mk[q] & (mk[q] - 1u);
            if (p < a.parts && ((rest >> p) & 1u)) {
              v[q].x += t[p - 1][q].x; v[q].y += t[p - 1][q].y; v[q].z += t[p - 1][q].z; v[q].w += t[p - 1][q].w;
            }
          }
        }
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (mk[q] >> 1) {  // some plane other than the row of U held it: the sum moves there, those planes are cleared
          *reinterpret_cast<float4 *>(urow + at[q]) = v[q];
          for (int32_t p = 1; p < a.parts; ++p)
            if ((mk[q] >> p) & 1u)
              *reinterpret_cast<float4 *>(pl + (int64_t)(p - 1) * a.d_pad + at[q]) = make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) { take(v[q].x); take(v[q].y); take(v[q].z); take(v[q].w); }
    }
  }
  fmx = wave_max(fmx);
  sum = wave_sum(sum); sumsq = wave_sum(sumsq); bad = wave_sum(bad);
  if (lane == 0) { red[wv][0] = (double)fmx; red[wv][1] = sum; red[wv][2] = sumsq; red[wv][3] = bad; }
  __syncthreads();
  if (tid == 0) {
    double amax = 0.0;
    sum = 0.0; sumsq = 0.0; bad = 0.0;
    for (int k = 0; k < 4; ++k) { amax = fmax(amax, red[k][0]); sum += red[k][1]; sumsq += red[k][2]; bad += red[k][3]; }
    double *p = sk.stat_part + ((int64_t)worker * sk.stat_slots + blockIdx.x) * 4;
    p[0] = amax; p[1] = sum; p[2] = sumsq; p[3] = bad;
  }
}

// eq. (3) + quantize + pack over the visited segments; a marked tail segment of U is set back to zero for the
// next iteration.  The launch is bound by latency, not throughput, so the work is spread thin: EIGHT lanes
// share a segment (four coordinates = one Philox block each), the 32 codes of a segment meet in LDS and the
// B words are assembled from there.  Workgroups [0, head/1024) of a worker take 32 head segments each; in
// the others every wavefront visits the marked ones of its kWaveSegs tail segments, up to 32 at a time.
// Every workgroup folds its worker's statistic partials itself (the fixed order of fold_stat_slots, so all of
// them derive the same scale); workgroup 0 of a worker records the results.
template <int B>
__global__ __launch_bounds__(kThreads) void sparse_quantize_kernel(SparseArgs a, StatSinks sk, QuantSpec qs,
                                                                   int32_t nslots, int64_t d, StreamKey key,
                                                                   int32_t share, uint32_t *__restrict__ packed,
                                                                   float *__restrict__ delta_out) {
  touch_kernel_arguments<(int)(sizeof(SparseArgs) + sizeof(StatSinks) + sizeof(QuantSpec) + 48)>();
  __shared__ int32_t codes[4][32][32];  // per wavefront: 32 segments x 32 codes
  __shared__ int32_t lists[4][kWaveSegs];
  __shared__ QParams q_sh;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int sub = lane >> 3, part = lane & 7;  // this lane moves coordinates 4*part..+3 of segment slot `sub` (+8q)
  const uint32_t worker = blockIdx.y;
  const int32_t head_wgs = a.head / (32 * kSegFloats);
  const bool head = (int32_t)blockIdx.x < head_wgs;
  float *urow = a.U + (int64_t)worker * a.d_pad;
  uint32_t *out = packed + (int64_t)worker * a.W;
  int32_t *list = lists[wv];
  int32_t n = 0;
  float4 v[4], vn[4];
  // a batch = up to 32 listed segments of this wavefront: slot 8q + sub for q < 4; the tail's are zeroed as read
  auto load_batch = [&](int32_t i0, float4 (&dst)[4]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int32_t i = i0 + 8 * q + sub;
      dst[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i < n) {
        float *u = urow + (int64_t)list[i] * kSegFloats + part * 4;
        dst[q] = *reinterpret_cast<const float4 *>(u);
        *reinterpret_cast<float4 *>(u) = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
  };
  const int64_t head_seg = (int64_t)blockIdx.x * 32 + wv * 8 + sub;  // head: one segment per eight lanes
  if (head) {
    v[0] = *reinterpret_cast<const float4 *>(urow + head_seg * kSegFloats + part * 4);
  } else {
    const int64_t stride = (int64_t)(gridDim.x - head_wgs) * 4;  // tail wavefronts of this worker
    const int64_t first_word = a.head / (kSegFloats * 32) + ((int64_t)blockIdx.x - head_wgs) * 4 + wv;
    n = compact_marked(a.touched + (int64_t)worker * a.bitmap_words, a.bitmap_words, first_word, stride,
                                    a.d_pad / kSegFloats, lane, list);
    __builtin_amdgcn_wave_barrier();
    load_batch(0, v);  // on its way while the statistics are folded
  }
  if (tid < 64) {
    double amax, sum, sumsq, bad;
    fold_stat_slots(sk.stat_part + (int64_t)worker * sk.stat_slots * 4, nslots, tid, amax, sum, sumsq, bad);
    // schemes (b), (c) of Sec. 4.2: every worker quantizes with the largest of the N scale factors; each workgroup
    // derives it from all the workers' statistic partials (the same folds in the same order everywhere)
    float dmax = 0.0f;
    if (share) {
      for (int32_t i = 0; i < a.N; ++i) {
        double am_i, s_i, s2_i, b_i;
        fold_stat_slots(sk.stat_part + (int64_t)i * sk.stat_slots * 4, nslots, tid, am_i, s_i, s2_i, b_i);
        dmax = fmaxf(dmax, make_qparams(qs, am_i, s_i, s2_i, d).delta);
      }
    }
    if (tid == 0) {
      const QParams q = share ? qparams_from_delta(qs, dmax) : make_qparams(qs, amax, sum, sumsq, d);
      q_sh = q;
      if (blockIdx.x == 0) {
        double *o = sk.stats + (int64_t)worker * 4;
        o[0] = amax; o[1] = sum; o[2] = sumsq; o[3] = bad;
        sk.qparams[worker] = q;
        delta_out[worker] = q.delta;
        if (bad > 0.0) atomicOr(&sk.flags[0], 1u);
      }
    }
  }
  __syncthreads();
  const QParams q = q_sh;
  if (head) {
    int32_t code[4];
    quantize_four<B, false>(v[0], q, key, worker, (uint32_t)(head_seg * 8 + part), code);
    *reinterpret_cast<int4 *>(&codes[wv][sub][4 * part]) = make_int4(code[0], code[1], code[2], code[3]);
    __builtin_amdgcn_wave_barrier();
    const int64_t seg0 = (int64_t)blockIdx.x * 32 + wv * 8;  // the wavefront's eight segments are consecutive
    for (int t = lane; t < 8 * B; t += 64) out[seg0 * B + t] = assemble_word<B>(codes[wv][t / B], t % B);
  } else {
    for (int32_t i0 = 0; i0 < n; i0 += 32) {
      if (i0 + 32 < n) load_batch(i0 + 32, vn);  // the next batch is on its way while this one is quantized
#pragma unroll
      for (int qi = 0; qi < 4; ++qi) {
        const int32_t i = i0 + 8 * qi + sub;
        if (i < n) {
          int32_t code[4];
          quantize_four<B, false>(v[qi], q, key, worker, (uint32_t)list[i] * 8u + (uint32_t)part, code);
          *reinterpret_cast<int4 *>(&codes[wv][8 * qi + sub][4 * part]) = make_int4(code[0], code[1], code[2], code[3]);
        }
      }
      __builtin_amdgcn_wave_barrier();
      const int32_t cnt = n - i0 < 32 ? n - i0 : 32;
      for (int t = lane; t < cnt * B; t += 64) {
        const int sl = t / B, w = t % B;
        out[(int64_t)list[i0 + sl] * B + w] = assemble_word<B>(codes[wv][sl], w);
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int q = 0; q < 4; ++q) v[q] = vn[q];
    }
  }
}

// ---------------------------------------------------------------------------
// Small-d inner iteration: statistics fold -> eq. (3) -> quantize -> pack -> eq. (4) -> prox in ONE
// launch.  When d is a few thousand the whole exchange moves a few hundred KB and is bound by
// launch and dependency latency, not by HBM, so the work is spread as wide as possible: a
// workgroup owns 128 coordinates (4 segments) of ALL workers, thread (g, l) quantizes the four
// coordinates 4l..4l+3 of worker g, g+8, ..., codes meet in LDS, then words are assembled and the
// average and proximal step are taken for the 128 coordinates.  Every workgroup folds the
// statistic partials itself (same fixed order as the stand-alone fold), so no grid-wide
// synchronisation is needed inside the launch.
constexpr int kFusedCoords = 128;
// threads per workgroup; measured back to back on one machine against 512: 256 threads -1.0 % inner
// iterations/s on the d = 4096, N = 8 workload and -1.9 % on d = 8192, N = 16; 1024 threads -3.3 % and -1.0 %
constexpr int kFusedThreads = 512;
constexpr int kFusedMaxN = 64;

struct FusedArgs {
  const float *U;
  int64_t d, d_pad, W;
  int32_t N, bits, nslots, stat_slots;
  const double *stat_part;
  QuantSpec qs;
  StreamKey key;
  uint32_t *packed;
  float *delta_out;
  double *stats;
  uint32_t *flags;
  const float *mu;
  float *w;
  float *u_avg_out;
  float step, thr, shrink;
  int32_t do_prox;
  // ALPC-SVRG epilogue (Alg. 2 steps 13-15 and the next step 6) instead of the plain proximal step
  int32_t do_alpc;
  const float *x, *u_hat, *w_snap;
  float *y, *z, *ysum, *x_next;
  float step_y, thr_y, shrink_y, alpha, thr_z, shrink_z, weight, t1, t2, t3;
  int32_t first;
  // Rows the NEXT worker pass will read (dense data, small batches): workgroups past the tiles draw them from
  // the next iteration's random stream and request them, so that they wait in the last-level cache instead of
  // in HBM.  warm_groups = 0: nothing to warm.
  // Column-tile iteration (dots_R > 0): the launch has dots_R workgroups per tile.  Each repeats the tile's
  // exchange and update (reading the old iterate from w_in / x / z_in, so that the one workgroup per tile that
  // stores results, into w / x_next / z, disturbs nobody) and then leaves the partial dot products of its share of
  // the NEXT iteration's sampled rows with the tile's new iterate (dots.pd).  dots_R = 0: one workgroup per tile,
  // w_in = w, z_in = z, plus the warming workgroups below.
  int32_t dots_R;
  const float *w_in, *z_in;
  DotsArgs dots;
  const float *warm_X, *warm_y, *warm_z;
  int64_t warm_ldx, warm_n;
  StreamKey warm_key;   // of the next iteration
  int32_t warm_groups, warm_parts, warm_rows_per_part, warm_B, warm_shared;  // warm_shared: worker index of batch J, or -1
  float *warm_sink;
};

// Workgroup ntiles + w of the launch touches every 128-byte line of the rows that workgroup w of the next worker
// pass will read.  (The counters show that pass still fetching its rows through the fabric -- the L2s do not
// keep lines from one kernel to the next -- but from the memory-side cache: 6.8 -> 5.7 us.)  Plain loads; the
// sum is stored only if it equals a value it cannot take.
__device__ __forceinline__ void warm_next_rows(const FusedArgs &a, int ntiles) {
  const int w = (int)blockIdx.x - ntiles;
  if (w >= a.warm_groups) return;
  const int wrel = w / a.warm_parts, part = w % a.warm_parts;
  const int pos0 = part * a.warm_rows_per_part;
  const int pos1 = pos0 + a.warm_rows_per_part < a.warm_B ? pos0 + a.warm_rows_per_part : a.warm_B;
  const bool shared = wrel == a.warm_shared;
  const int64_t lines = (a.d + 31) / 32;  // 32 floats per line; line l of a row starts at float 32*l < d
  float sink = 0.0f;
  if (a.warm_rows_per_part <= 2) {
    // one or two rows: one after the other (requested together they get in the way of the tile workgroups' own
    // operands: measured 5 % slower on d = 4096, N = 8, B = 64)
    for (int pos = pos0; pos < pos1; ++pos) {
      const int64_t r = shared ? sample_row(a.warm_key, kTagShared, kSharedWorkerField, (uint32_t)pos, a.warm_n)
                               : sample_row(a.warm_key, kTagBatch, (uint32_t)wrel, (uint32_t)pos, a.warm_n);
      const float *xr = a.warm_X + r * a.warm_ldx;
      for (int64_t l = threadIdx.x; l < lines; l += blockDim.x) sink += xr[l * 32];
      if (threadIdx.x == 0) sink += a.warm_y[r] + (a.warm_z ? a.warm_z[r] : 0.0f);
    }
  } else {
    // more rows: four at a time, their draws first, then all their requests, and only then the additions, so that
    // the workgroup waits for memory once per four rows and not once per row
    for (int p0 = pos0; p0 < pos1; p0 += 4) {
      const float *xr[4];
      int64_t row[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        row[q] = 0;
        if (p0 + q < pos1)  // uniform
          row[q] = shared ? sample_row(a.warm_key, kTagShared, kSharedWorkerField, (uint32_t)(p0 + q), a.warm_n)
                          : sample_row(a.warm_key, kTagBatch, (uint32_t)wrel, (uint32_t)(p0 + q), a.warm_n);
        xr[q] = a.warm_X + row[q] * a.warm_ldx;
      }
      for (int64_t l = threadIdx.x; l < lines; l += blockDim.x) {
        float t[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) t[q] = p0 + q < pos1 ? xr[q][l * 32] : 0.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) sink += t[q];
      }
      if (threadIdx.x < 8) {  // lanes 0-3: the labels, lanes 4-7: the cached margins
        const int q = threadIdx.x & 3;
        const int64_t r = q == 0 ? row[0] : (q == 1 ? row[1] : (q == 2 ? row[2] : row[3]));
        if (p0 + q < pos1) sink += threadIdx.x < 4 ? a.warm_y[r] : (a.warm_z ? a.warm_z[r] : 0.0f);
      }
    }
  }
  if (sink == -1.2345678e-38f) *a.warm_sink = sink;
}

__global__ __launch_bounds__(kFusedThreads) void fused_exchange_kernel(FusedArgs a) {
  touch_kernel_arguments<(int)(sizeof(FusedArgs))>();
  constexpr int GROUPS = kFusedThreads / 32, NW = kFusedThreads / 64;  // 32-lane groups (a worker each per round), wavefronts
  __shared__ QParams qp[kFusedMaxN];
  __shared__ int32_t codes[kFusedMaxN][kFusedCoords];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  __shared__ __attribute__((aligned(16))) float next_sh[kFusedCoords];  // the tile of the new iterate (dots_R > 0)
  const int ntiles = (int)((a.d_pad + kFusedCoords - 1) / kFusedCoords);
  if (a.dots_R == 0 && (int)blockIdx.x >= ntiles) {  // whole workgroups: no barrier below is skipped by part of one
    warm_next_rows(a, ntiles);
    return;
  }
  const int tile = a.dots_R > 0 ? (int)blockIdx.x % ntiles : (int)blockIdx.x;
  const int share = a.dots_R > 0 ? (int)blockIdx.x / ntiles : 0;
  const bool writer = share == 0;  // the one workgroup of the tile that stores the exchange's results
  const int64_t tile0 = (int64_t)tile * kFusedCoords;
  // the next iteration's rows are requested first of all: they come from HBM
  float4 xpre[8];
  if (a.dots_R > 0) tile_dots_load(a.dots, tile, share * a.dots.rows_per_wg, a.dots.rows_per_wg, tid, xpre);
  // everything this thread will need from memory is requested before the statistics fold, so the three
  // dependent round trips (statistics, U, w/mu) overlap
  float4 v_all[kFusedMaxN / GROUPS];  // this thread's four coordinates of workers g, g+GROUPS, ...
#pragma unroll
  for (int q = 0; q < kFusedMaxN / GROUPS; ++q) {
    const int32_t i = (tid >> 5) + GROUPS * q;
    v_all[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (i < a.N && tile0 + 4 * (tid & 31) < a.d_pad)
      v_all[q] = *reinterpret_cast<const float4 *>(a.U + (int64_t)i * a.d_pad + tile0 + 4 * (tid & 31));
  }
  float w_old = 0.0f, mu_j = 0.0f, x_j = 0.0f, z_j = 0.0f, uhat_j = 0.0f, ysum_j = 0.0f, snap_j = 0.0f;
  if (tid < kFusedCoords && tile0 + tid < a.d) {
    const int64_t j = tile0 + tid;
    if (a.do_prox) {
      w_old = a.w_in[j];
      mu_j = a.mu[j];
    }
    if (a.do_alpc) {
      mu_j = a.mu[j]; x_j = a.x[j]; z_j = a.z_in[j]; uhat_j = a.u_hat[j]; snap_j = a.w_snap[j];
      ysum_j = (a.first || !writer) ? 0.0f : a.ysum[j];
    }
  }
  // wavefront wv folds the statistics of vectors wv, wv+NW, ...; four vectors at a time so that their partials
  // are requested together (the lane-wise sums and the butterflies keep fold_stat_slots' order)
  for (int32_t i0 = wv; i0 < a.N; i0 += 4 * NW) {
    double am[4], s[4], s2[4], b[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) { am[q] = 0.0; s[q] = 0.0; s2[q] = 0.0; b[q] = 0.0; }
    for (int32_t k = lane; k < a.nslots; k += 64) {
      double2 lo[4], hi[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int32_t i = i0 + NW * q < a.N ? i0 + NW * q : i0;
        const double *p = a.stat_part + ((int64_t)i * a.stat_slots + k) * 4;
        lo[q] = *reinterpret_cast<const double2 *>(p);
        hi[q] = *reinterpret_cast<const double2 *>(p + 2);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) { am[q] = fmax(am[q], lo[q].x); s[q] += lo[q].y; s2[q] += hi[q].x; b[q] += hi[q].y; }
    }
    // every lane ends with the four vectors' statistics; lane q then derives the quantizer's parameters of vector q
    // of this wavefront, so the (double-precision) derivation runs once for the four and not once after another
    double am_m = 0.0, s_m = 0.0, s2_m = 0.0, b_m = 0.0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      if (i0 + NW * q >= a.N) break;  // uniform over the wavefront
      const double am_w = wave_max(am[q]), s_w = wave_sum(s[q]), s2_w = wave_sum(s2[q]), b_w = wave_sum(b[q]);
      if (lane == q) { am_m = am_w; s_m = s_w; s2_m = s2_w; b_m = b_w; }
    }
    if (lane < 4 && i0 + NW * lane < a.N) {
      const int32_t i = i0 + NW * lane;
      const QParams q_i = make_qparams(a.qs, am_m, s_m, s2_m, a.d);
      qp[i] = q_i;
      if (blockIdx.x == 0) {  // tile 0's writer
        a.delta_out[i] = q_i.delta;
        double *o = a.stats + (int64_t)i * 4;
        o[0] = am_m; o[1] = s_m; o[2] = s2_m; o[3] = b_m;
        if (b_m > 0.0) atomicOr(&a.flags[0], 1u);
      }
    }
  }
  __syncthreads();
  {
    const int g = tid >> 5, l = tid & 31;
    const int64_t j = tile0 + 4 * l;
    const float hi = (float)((1 << (a.bits - 1)) - 1);
    const float lo = -(float)(1 << (a.bits - 1));
#pragma unroll
    for (int qi = 0; qi < kFusedMaxN / GROUPS; ++qi) {
      const int32_t i = g + GROUPS * qi;
      if (i >= a.N) break;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j < a.d_pad) {
        v = v_all[qi];
        if (j + 3 >= a.d) {
          if (j + 0 >= a.d) v.x = 0.f;
          if (j + 1 >= a.d) v.y = 0.f;
          if (j + 2 >= a.d) v.z = 0.f;
          v.w = 0.f;
        }
      }
      const QParams q = qp[i];
      const float vals[4] = {v.x, v.y, v.z, v.w};
      float base[4], frac[4];
      bool any = false;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        float s = vals[t] * q.rdelta;
        s = fminf(fmaxf(s, lo), hi);
        base[t] = floorf(s);
        frac[t] = s - base[t];
        any = any || (frac[t] != 0.0f);
      }
      uint32_t rnd[4] = {0u, 0u, 0u, 0u};
      if (any) {
        const Philox4 blk = stream_block(a.key, kTagQuant, (uint32_t)i, (uint32_t)(j >> 2));
        rnd[0] = blk.x; rnd[1] = blk.y; rnd[2] = blk.z; rnd[3] = blk.w;
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float unif = (float)(rnd[t] >> 8) * 0x1.0p-24f;
        codes[i][4 * l + t] = q.delta > 0.0f ? (int32_t)base[t] + ((unif < frac[t]) ? 1 : 0) : 0;
      }
    }
  }
  __syncthreads();
  // pack: one thread per output word of the tile.  The wavefronts past the first two take the words, so that they
  // run beside the update below (threads 0-127) and not ahead of it on the same threads; index / bits is taken with
  // a 16.16 reciprocal (exact below 4096; the indices here stay below 1024).
  if (tid >= kFusedCoords) {
    const int32_t bits = a.bits;
    const uint32_t mask = (1u << bits) - 1u;
    const uint32_t inv = (65536u + (uint32_t)bits - 1u) / (uint32_t)bits;
    const int32_t words_per_worker = 4 * bits;
    const int64_t seg0 = tile0 / kSegFloats;
    for (int32_t idx = tid - kFusedCoords; idx < a.N * words_per_worker; idx += kFusedThreads - kFusedCoords) {
      const int32_t i = (int32_t)((((uint32_t)idx >> 2) * inv) >> 16), rem = idx - i * words_per_worker;
      const int32_t sgm = (int32_t)(((uint32_t)rem * inv) >> 16), wd = rem - sgm * bits;
      if ((seg0 + sgm) * kSegFloats >= a.d_pad || !writer) continue;
      const int32_t bit0 = 32 * wd;
      uint32_t word = 0u;
      for (int32_t c = (int32_t)(((uint32_t)bit0 * inv) >> 16); c < 32 && c * bits < bit0 + 32; ++c) {
        const uint32_t field = (uint32_t)codes[i][32 * sgm + c] & mask;
        const int32_t sh = c * bits - bit0;
        word |= sh >= 0 ? (field << sh) : (field >> (-sh));
      }
      a.packed[(int64_t)i * a.W + (seg0 + sgm) * bits + wd] = word;
    }
  }
  // eq. (4) in worker order, then Alg. 1 steps 9-10
  if (tid < kFusedCoords) {
    const int64_t j = tile0 + tid;
    float next = 0.0f;
    if (j < a.d) {
      float acc = 0.0f;
      for (int32_t i0 = 0; i0 < a.N; i0 += 8) {  // eight workers' operands are read from LDS before the first is used
        float dl[8];
        int32_t cd[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
          const int32_t i = i0 + k < a.N ? i0 + k : a.N - 1;
          dl[k] = qp[i].delta;
          cd[k] = codes[i][tid];
        }
#pragma unroll
        for (int k = 0; k < 8; ++k)
          if (i0 + k < a.N) acc = __builtin_fmaf(dl[k], (float)cd[k], acc);
      }
      const float avg = acc * (1.0f / (float)a.N);
      if (a.u_avg_out && writer) a.u_avg_out[j] = avg;
      if (a.do_prox) {
        next = prox_scalar(w_old, avg + mu_j, a.step, a.thr, a.shrink);
        if (writer) a.w[j] = next;
      }
      if (a.do_alpc) {
        const float yn = prox_scalar(x_j, avg + mu_j, a.step_y, a.thr_y, a.shrink_y);   // low-precision gradient
        const float zn = prox_scalar(z_j, uhat_j + mu_j, a.alpha, a.thr_z, a.shrink_z);  // full precision
        next = (a.t1 * zn + a.t2 * snap_j) + a.t3 * yn;
        if (writer) {
          a.y[j] = yn;
          a.z[j] = zn;
          a.ysum[j] = a.first ? a.weight * yn : ysum_j + a.weight * yn;
          a.x_next[j] = next;
        }
      }
    }
    next_sh[tid] = next;
  }
  if (a.dots_R > 0) {
    __syncthreads();
    tile_dots_finish(a.dots, next_sh, tile, share * a.dots.rows_per_wg, a.dots.rows_per_wg, tid, xpre);
  }
}

// ---------------------------------------------------------------------------
// Small-d inner iteration in TWO launches: the workers' rows kernel, then this one, which is the exchange above
// with the fold of the partial rows taken in.  A workgroup owns TILE coordinates of ALL vectors: it folds their
// partial rows itself (same order as reduce_parts_kernel, so u^i has the same bits), keeps u^i in registers,
// and needs from the other workgroups only the statistics of their tiles (eq. (3) wants |u^i|_inf over all d
// coordinates).  Those travel through memory as self-validating words: every workgroup stores the four
// statistics of each of its (tile, vector) pairs as 64-bit device-scope atomic stores into its own slots, and
// reads everyone's slots with device-scope atomic loads until none holds the "empty" pattern (all ones: no
// finite double).  No other data crosses workgroups, so no fence is needed.  Two slot sets alternate between
// consecutive launches: a launch empties its slots of the other set, which nobody reads meanwhile.  The wait
// is bounded: after spin_limit polls a workgroup gives up, raises flag bit 1 and finishes with what it has,
// so every wave exits whatever happens; the host reports the flag as LPC_EDEVICE.  All tile workgroups must
// be resident together for the wait to end quickly: the host launches at most one per CU's worth of them,
// ahead (in dispatch order) of the warming workgroups, which never wait.
constexpr unsigned long long kSlotEmpty = ~0ull;

struct IterArgs {
  FusedArgs f;            // as for fused_exchange_kernel; U, stat_part, nslots are unused
  const float *part;      // [nvec][parts][d] partial rows of the workers' pass
  int32_t parts, nvec;    // nvec = N, or N + 1 with the shared batch's vector last
  int32_t nwf;            // interleaved accumulators of the fold: 2 or 4, as launch_reduce_parts picks
  int32_t vec4;           // partial rows may be read 16 bytes at a time
  float scale;
  unsigned long long *slots_cur, *slots_next;  // [ntiles][N][4]
  uint32_t spin_limit;
};

template <int NWF>
__device__ __forceinline__ float4 fold_partial_rows(const float *__restrict__ src, int32_t parts, int64_t d,
                                                    int64_t room, bool vec4, float scale) {
  // room = coordinates of this chunk inside the vector (4, or fewer at a ragged end)
  float4 acc[NWF];
#pragma unroll
  for (int q = 0; q < NWF; ++q) acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int32_t p0 = 0; p0 < parts; p0 += 16) {  // sixteen partial rows in flight
    float4 t[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      t[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (p0 + k < parts) {
        const float *s = src + (int64_t)(p0 + k) * d;
        if (vec4) {
          t[k] = *reinterpret_cast<const float4 *>(s);
        } else {
          t[k].x = s[0];
          if (room > 1) t[k].y = s[1];
          if (room > 2) t[k].z = s[2];
          if (room > 3) t[k].w = s[3];
        }
      }
    }
#pragma unroll
    for (int k = 0; k < 16; ++k) {  // row p joins accumulator p mod NWF, rows in increasing order
      float4 &c = acc[k % NWF];
      c.x += t[k].x; c.y += t[k].y; c.z += t[k].z; c.w += t[k].w;
    }
  }
  float4 v = acc[0];
#pragma unroll
  for (int q = 1; q < NWF; ++q) { v.x += acc[q].x; v.y += acc[q].y; v.z += acc[q].z; v.w += acc[q].w; }
  v.x *= scale; v.y *= scale; v.z *= scale; v.w *= scale;
  if (room < 4) v.w = 0.f;
  if (room < 3) v.z = 0.f;
  if (room < 2) v.y = 0.f;
  return v;
}

// sum / max over the LPV (16 or 32) adjacent lanes that share a vector; every lane of the wavefront takes part
template <int LPV>
__device__ __forceinline__ double group_sum(double v, int lane) {
  v = row16_sum(v);
  if constexpr (LPV == 32) {
    const double lo = read_lane(v, 0) + read_lane(v, 16), hi = read_lane(v, 32) + read_lane(v, 48);
    v = lane < 32 ? lo : hi;
  }
  return v;
}
template <int LPV>
__device__ __forceinline__ float group_max(float v, int lane) {
  v = row16_max(v);
  if constexpr (LPV == 32) {
    const float lo = fmaxf(read_lane(v, 0), read_lane(v, 16)), hi = fmaxf(read_lane(v, 32), read_lane(v, 48));
    v = lane < 32 ? lo : hi;
  }
  return v;
}

__device__ __forceinline__ unsigned long long slot_load(const unsigned long long *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void slot_store(unsigned long long *p, unsigned long long v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <int THREADS, int TILE>
__global__ __launch_bounds__(THREADS) void fused_iter_kernel(IterArgs ia) {
  const FusedArgs &a = ia.f;
  constexpr int LPV = TILE / 4;          // lanes per vector: four coordinates (one Philox block) each
  constexpr int GROUPS = THREADS / LPV;  // vectors served per round
  constexpr int NW = THREADS / 64;
  constexpr int ROUNDS = (kFusedMaxN + GROUPS) / GROUPS;  // rounds over up to kFusedMaxN + 1 vectors
  __shared__ QParams qp[kFusedMaxN];
  __shared__ int32_t codes[kFusedMaxN][TILE];
  __shared__ double st[kFusedMaxN][4];
  __shared__ float uhat_sh[TILE];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int ntiles = (int)((a.d_pad + TILE - 1) / TILE);
  if ((int)blockIdx.x >= ntiles) {  // whole workgroups: no barrier below is skipped by part of one
    warm_next_rows(a, ntiles);
    return;
  }
  const int64_t tile0 = (int64_t)blockIdx.x * TILE;
  const int g = tid / LPV, l = tid % LPV;
  const int64_t j = tile0 + 4 * l;
  // the epilogue's operands are requested first, the partial rows right behind them
  float w_old = 0.0f, mu_j = 0.0f, x_j = 0.0f, z_j = 0.0f, ysum_j = 0.0f, snap_j = 0.0f;
  if (tid < TILE && tile0 + tid < a.d) {
    const int64_t jj = tile0 + tid;
    if (a.do_prox) {
      w_old = a.w[jj];
      mu_j = a.mu[jj];
    }
    if (a.do_alpc) {
      mu_j = a.mu[jj]; x_j = a.x[jj]; z_j = a.z[jj]; snap_j = a.w_snap[jj];
      ysum_j = a.first ? 0.0f : a.ysum[jj];
    }
  }
  float4 v_all[ROUNDS];
#pragma unroll
  for (int q = 0; q < ROUNDS; ++q) {
    v_all[q] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (q * GROUPS >= ia.nvec) break;  // uniform
    const int32_t i = g + GROUPS * q;
    if (i < ia.nvec && j < a.d) {
      const float *src = ia.part + (int64_t)i * ia.parts * a.d + j;
      const int64_t room = a.d - j < 4 ? a.d - j : 4;
      v_all[q] = ia.nwf == 2 ? fold_partial_rows<2>(src, ia.parts, a.d, room, ia.vec4 != 0, ia.scale)
                             : fold_partial_rows<4>(src, ia.parts, a.d, room, ia.vec4 != 0, ia.scale);
    }
  }
  // statistics of this tile of every worker's vector
#pragma unroll
  for (int q = 0; q < ROUNDS; ++q) {
    if (q * GROUPS >= a.N) break;  // uniform
    const int32_t i = g + GROUPS * q;
    const float vals[4] = {v_all[q].x, v_all[q].y, v_all[q].z, v_all[q].w};
    float fmx = 0.0f;
    double sum = 0.0, sumsq = 0.0, bad = 0.0;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      if (isfinite(vals[t])) {
        fmx = fmaxf(fmx, fabsf(vals[t])); sum += (double)vals[t]; sumsq += (double)vals[t] * (double)vals[t];
      } else {
        bad += 1.0;
      }
    }
    fmx = group_max<LPV>(fmx, lane);
    sum = group_sum<LPV>(sum, lane); sumsq = group_sum<LPV>(sumsq, lane); bad = group_sum<LPV>(bad, lane);
    if (l == 0 && i < a.N) { st[i][0] = (double)fmx; st[i][1] = sum; st[i][2] = sumsq; st[i][3] = bad; }
  }
  __syncthreads();
  if (tid < 4 * a.N) {
    const int64_t at = ((int64_t)blockIdx.x * a.N + (tid >> 2)) * 4 + (tid & 3);
    slot_store(ia.slots_cur + at, __builtin_bit_cast(unsigned long long, st[tid >> 2][tid & 3]));
    slot_store(ia.slots_next + at, kSlotEmpty);
  }
  // the random draws do not depend on the scale: they are taken while the statistics travel
  uint32_t rnd[ROUNDS][4];
#pragma unroll
  for (int q = 0; q < ROUNDS; ++q) {
    rnd[q][0] = rnd[q][1] = rnd[q][2] = rnd[q][3] = 0u;
    if (q * GROUPS >= a.N) break;  // uniform
    const int32_t i = g + GROUPS * q;
    if (i < a.N && j < a.d_pad) {
      const Philox4 blk = stream_block(a.key, kTagQuant, (uint32_t)i, (uint32_t)(j >> 2));
      rnd[q][0] = blk.x; rnd[q][1] = blk.y; rnd[q][2] = blk.z; rnd[q][3] = blk.w;
    }
  }
  // wavefront wv gathers the statistics of vectors wv, wv+NW, ... from all tiles, four vectors at a time; lane k
  // takes tiles k, k+64, ..., then the butterflies: a fixed order, the same in every workgroup
  bool gave_up = false;
  for (int32_t i0 = wv; i0 < a.N; i0 += 4 * NW) {
    double am[4], s[4], s2[4], b[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) { am[q] = 0.0; s[q] = 0.0; s2[q] = 0.0; b[q] = 0.0; }
    for (int32_t k0 = 0; k0 < ntiles; k0 += 64) {
      const int32_t k = k0 + lane;
      const bool mine = k < ntiles;
      unsigned long long wd[4][4];
      bool ok[4];
      uint32_t polls = 0;
      for (;;) {
        bool all_ok = true;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int32_t i = i0 + NW * q < a.N ? i0 + NW * q : i0;
          const unsigned long long *p = ia.slots_cur + ((int64_t)(mine ? k : 0) * a.N + i) * 4;
#pragma unroll
          for (int t = 0; t < 4; ++t) wd[q][t] = slot_load(p + t);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          ok[q] = wd[q][0] != kSlotEmpty && wd[q][1] != kSlotEmpty && wd[q][2] != kSlotEmpty && wd[q][3] != kSlotEmpty;
          all_ok = all_ok && (ok[q] || !mine);
        }
        if (__ballot(!all_ok) == 0ull) break;
        if (++polls > ia.spin_limit) { gave_up = true; break; }
        __builtin_amdgcn_s_sleep(1);
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        if (mine && ok[q]) {
          am[q] = fmax(am[q], __builtin_bit_cast(double, wd[q][0]));
          s[q] += __builtin_bit_cast(double, wd[q][1]);
          s2[q] += __builtin_bit_cast(double, wd[q][2]);
          b[q] += __builtin_bit_cast(double, wd[q][3]);
        }
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int32_t i = i0 + NW * q;
      if (i >= a.N) break;  // uniform over the wavefront
      const double am_w = wave_max(am[q]), s_w = wave_sum(s[q]), s2_w = wave_sum(s2[q]), b_w = wave_sum(b[q]);
      if (lane == 0) {
        const QParams q_i = make_qparams(a.qs, am_w, s_w, s2_w, a.d);
        qp[i] = q_i;
        if (blockIdx.x == 0) {
          a.delta_out[i] = q_i.delta;
          double *o = a.stats + (int64_t)i * 4;
          o[0] = am_w; o[1] = s_w; o[2] = s2_w; o[3] = b_w;
          if (b_w > 0.0) atomicOr(&a.flags[0], 1u);
        }
      }
    }
  }
  if (gave_up && lane == 0) atomicOr(&a.flags[0], 2u);
  __syncthreads();
  {
    const float hi = (float)((1 << (a.bits - 1)) - 1);
    const float lo = -(float)(1 << (a.bits - 1));
#pragma unroll
    for (int qi = 0; qi < ROUNDS; ++qi) {
      if (qi * GROUPS >= ia.nvec) break;  // uniform
      const int32_t i = g + GROUPS * qi;
      const float vals[4] = {v_all[qi].x, v_all[qi].y, v_all[qi].z, v_all[qi].w};
      if (i < a.N) {
        const QParams q = qp[i];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          float s = vals[t] * q.rdelta;
          s = fminf(fmaxf(s, lo), hi);
          const float base = floorf(s);
          const float frac = s - base;
          const float unif = (float)(rnd[qi][t] >> 8) * 0x1.0p-24f;
          codes[i][4 * l + t] = q.delta > 0.0f ? (int32_t)base + ((unif < frac) ? 1 : 0) : 0;
        }
      } else if (i == a.N && ia.nvec > a.N) {
#pragma unroll
        for (int t = 0; t < 4; ++t) uhat_sh[4 * l + t] = vals[t];  // the shared batch's difference, full precision
      }
    }
  }
  __syncthreads();
  // pack: one thread per output word of the tile
  {
    const int32_t bits = a.bits;
    const uint32_t mask = (1u << bits) - 1u;
    const int32_t words_per_worker = (TILE / kSegFloats) * bits;
    const int64_t seg0 = tile0 / kSegFloats;
    for (int32_t idx = tid; idx < a.N * words_per_worker; idx += THREADS) {
      const int32_t i = idx / words_per_worker, rem = idx % words_per_worker;
      const int32_t sgm = rem / bits, wd = rem % bits;
      if ((seg0 + sgm) * kSegFloats >= a.d_pad) continue;
      const int32_t bit0 = 32 * wd;
      uint32_t word = 0u;
      for (int32_t c = bit0 / bits; c < 32 && c * bits < bit0 + 32; ++c) {
        const uint32_t field = (uint32_t)codes[i][32 * sgm + c] & mask;
        const int32_t sh = c * bits - bit0;
        word |= sh >= 0 ? (field << sh) : (field >> (-sh));
      }
      a.packed[(int64_t)i * a.W + (seg0 + sgm) * bits + wd] = word;
    }
  }
  // eq. (4) in worker order, then Alg. 1 steps 9-10 (or Alg. 2 steps 13-15 and the next step 6)
  if (tid < TILE) {
    const int64_t jj = tile0 + tid;
    if (jj < a.d) {
      float acc = 0.0f;
      for (int32_t i = 0; i < a.N; ++i) acc = __builtin_fmaf(qp[i].delta, (float)codes[i][tid], acc);
      const float avg = acc * (1.0f / (float)a.N);
      if (a.u_avg_out) a.u_avg_out[jj] = avg;
      if (a.do_prox) a.w[jj] = prox_scalar(w_old, avg + mu_j, a.step, a.thr, a.shrink);
      if (a.do_alpc) {
        const float yn = prox_scalar(x_j, avg + mu_j, a.step_y, a.thr_y, a.shrink_y);          // low-precision gradient
        const float zn = prox_scalar(z_j, uhat_sh[tid] + mu_j, a.alpha, a.thr_z, a.shrink_z);  // full precision
        a.y[jj] = yn;
        a.z[jj] = zn;
        a.ysum[jj] = a.first ? a.weight * yn : ysum_j + a.weight * yn;
        a.x_next[jj] = (a.t1 * zn + a.t2 * snap_j) + a.t3 * yn;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// Schemes (b) and (c) of Sec. 4.2: every worker quantized with the same delta = max_i delta_i, so the
// codes add as integers (ceil(log2 N) overflow bits) and one scaling recovers the average.  With
// REQUANT the average is stochastically rounded once more onto dom(delta, b) (eq. (5)); it lies inside
// the hull, so this second rounding is unbiased.

// all vectors take the largest delta among them
__global__ void share_delta_kernel(QParams *qp, int32_t nvec, QuantSpec qs, float *delta_out) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  float dmax = 0.0f;
  for (int32_t i = 0; i < nvec; ++i) dmax = fmaxf(dmax, qp[i].delta);
  const QParams q = qparams_from_delta(qs, dmax);
  for (int32_t i = 0; i < nvec; ++i) qp[i] = q;
  if (delta_out) delta_out[0] = q.delta;
}

template <int B>
__device__ __forceinline__ void unpack_add(const uint32_t *__restrict__ src, int32_t (&acc)[32]) {
  uint32_t words[B];
#pragma unroll
  for (int i = 0; i < B; ++i) words[i] = src[i];
#pragma unroll
  for (int c = 0; c < 32; ++c) {
    const int p = c * B, wi = p >> 5, sh = p & 31;
    uint32_t field = words[wi] >> sh;
    if (sh + B > 32) field |= words[wi + 1] << (32 - sh);
    acc[c] += (int32_t)(field << (32 - B)) >> (32 - B);
  }
}

template <int B, bool REQUANT>
__global__ __launch_bounds__(kThreads) void dequantize_shared_kernel(const uint32_t *__restrict__ packed, int64_t W,
                                                                     const float *__restrict__ delta, int32_t N,
                                                                     int64_t d, int64_t d_pad, StreamKey key,
                                                                     float *__restrict__ u_avg) {
  __shared__ __attribute__((aligned(16))) float tile[kThreads * kPitch];
  const int tid = threadIdx.x;
  const int64_t tile_base = (int64_t)blockIdx.x * kTileFloats;
  const int64_t seg = tile_base / kSegFloats + tid;
  if (seg * kSegFloats < d_pad) {
    int32_t acc[32];
#pragma unroll
    for (int c = 0; c < 32; ++c) acc[c] = 0;
    for (int32_t i = 0; i < N; ++i) unpack_add<B>(packed + (int64_t)i * W + seg * B, acc);
    const float dl = delta[0];
    const float inv_n = 1.0f / (float)N;
    const float hi = (float)((1 << (B - 1)) - 1), lo = -(float)(1 << (B - 1));
#pragma unroll
    for (int k = 0; k < 8; ++k) {
      float out[4];
      uint32_t rnd[4] = {0u, 0u, 0u, 0u};
      if (REQUANT) {
        const Philox4 blk = stream_block(key, kTagRequant, 0u, (uint32_t)(seg * 8 + k));
        rnd[0] = blk.x; rnd[1] = blk.y; rnd[2] = blk.z; rnd[3] = blk.w;
      }
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float mean_code = (float)acc[4 * k + t] * inv_n;  // position of the average on the grid
        if (!REQUANT) {
          out[t] = dl * mean_code;
        } else {
          float s = mean_code * 1.0f;
          s = fminf(fmaxf(s, lo), hi);
          const float base = floorf(s);
          const float frac = s - base;
          const float unif = (float)(rnd[t] >> 8) * 0x1.0p-24f;
          out[t] = dl * (float)((int32_t)base + ((unif < frac) ? 1 : 0));
        }
      }
      *reinterpret_cast<float4 *>(&tile[tid * kPitch + k * 4]) = make_float4(out[0], out[1], out[2], out[3]);
    }
  }
  __syncthreads();
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    const int e = r * kThreads + tid;
    const int64_t j = tile_base + (int64_t)e * 4;
    if (j >= d) continue;
    const float4 a = *reinterpret_cast<const float4 *>(&tile[(e >> 3) * kPitch + (e & 7) * 4]);
    if (j + 4 <= d) {
      *reinterpret_cast<float4 *>(u_avg + j) = a;
    } else {
      const float av[4] = {a.x, a.y, a.z, a.w};
      for (int t = 0; t < 4 && j + t < d; ++t) u_avg[j + t] = av[t];
    }
  }
}

// quantization off: u_avg = (1/N) sum_i u^i, float adds in worker order
__global__ void plain_avg_kernel(const float *__restrict__ U, int64_t d, int64_t d_pad, int32_t N,
                                 float *__restrict__ u_avg) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= d) return;
  float acc = 0.0f;
  for (int32_t i = 0; i < N; ++i) acc = acc + U[(int64_t)i * d_pad + j];
  u_avg[j] = acc * (1.0f / (float)N);
}

__global__ void prox_kernel(float *__restrict__ w, const float *__restrict__ u_avg, const float *__restrict__ mu,
                            int64_t d, float step, float thr, float shrink) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= d) return;
  w[j] = prox_scalar(w[j], u_avg[j] + mu[j], step, thr, shrink);
}

__global__ void copy_kernel(float *__restrict__ dst, const float *__restrict__ src, int64_t n) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n) dst[j] = src[j];
}

__global__ void fill_u32_kernel(uint32_t *dst, uint32_t v, int64_t n) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n) dst[j] = v;
}

__global__ void scale_to_kernel(const float *__restrict__ src, float scale, float *__restrict__ dst, int64_t n) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j < n) dst[j] = src[j] * scale;
}

// Alg. 2 step 6: x = tau1*z + tau2*x~ + (1 - tau1 - tau2)*y
__global__ void alpc_couple_kernel(const float *__restrict__ z, const float *__restrict__ ws,
                                   const float *__restrict__ y, float t1, float t2, float t3, float *__restrict__ x,
                                   int64_t d) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j < d) x[j] = (t1 * z[j] + t2 * ws[j]) + t3 * y[j];
}

// Alg. 2 steps 13-15: y <- prox_{h/(4L)}(x - v/(4L)), z <- prox_{alpha h}(z - alpha v^),
// ysum <- ysum + theta^t * y
__global__ void alpc_update_kernel(const float *__restrict__ x, const float *__restrict__ u_avg,
                                   const float *__restrict__ u_hat, const float *__restrict__ mu, float step_y,
                                   float thr_y, float shrink_y, float alpha, float thr_z, float shrink_z,
                                   float weight, int first, float *__restrict__ y, float *__restrict__ z,
                                   float *__restrict__ ysum, int64_t d) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= d) return;
  const float m = mu[j];
  const float yn = prox_scalar(x[j], u_avg[j] + m, step_y, thr_y, shrink_y);
  const float zn = prox_scalar(z[j], u_hat[j] + m, alpha, thr_z, shrink_z);
  y[j] = yn;
  z[j] = zn;
  ysum[j] = first ? weight * yn : ysum[j] + weight * yn;
}

// Alg. 2 steps 13-15 and the next step 6 for the sparse inner iteration: as alpc_update_kernel followed by
// alpc_couple_kernel, and the shared batch's difference u_hat (dense storage, non-zero in the head columns and the
// touched tail segments only) is set back to zero where it was not, ready for the next iteration's scatter.
__global__ void alpc_update_couple_kernel(const float *__restrict__ x, const float *__restrict__ u_avg,
                                          float *__restrict__ u_hat, const float *__restrict__ mu,
                                          const float *__restrict__ ws, float step_y, float thr_y, float shrink_y,
                                          float alpha, float thr_z, float shrink_z, float weight, int first, float t1,
                                          float t2, float t3, float *__restrict__ y, float *__restrict__ z,
                                          float *__restrict__ ysum, float *__restrict__ x_next, int64_t d) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= d) return;
  const float m = mu[j], uh = u_hat[j];
  const float yn = prox_scalar(x[j], u_avg[j] + m, step_y, thr_y, shrink_y);
  const float zn = prox_scalar(z[j], uh + m, alpha, thr_z, shrink_z);
  if (uh != 0.0f) u_hat[j] = 0.0f;
  y[j] = yn;
  z[j] = zn;
  ysum[j] = first ? weight * yn : ysum[j] + weight * yn;
  x_next[j] = (t1 * zn + t2 * ws[j]) + t3 * yn;
}

// f_out = scale * sum of the loss partials (one workgroup, fixed order)
__global__ __launch_bounds__(kThreads) void sum_loss_kernel(const double *__restrict__ part, int32_t n, double scale,
                                                            double *__restrict__ f_out) {
  __shared__ double red[4];
  const int tid = threadIdx.x;
  double acc = 0.0;
  for (int32_t k = tid; k < n; k += kThreads) acc += part[k];
  acc = wave_sum(acc);
  if ((tid & 63) == 0) red[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) *f_out = (((red[0] + red[1]) + red[2]) + red[3]) * scale;
}

// partial[g] = lambda1*|w|_1 + (lambda2/2)*|w|^2 over workgroup g's share of w (coordinates g*1024 + tid, then in
// steps of 1024*gridDim.x; eight loads in flight per thread); fixed order, fp64
__global__ __launch_bounds__(1024) void objective_reg_kernel(const float *__restrict__ w, int64_t d, double l1,
                                                             double l2, double *__restrict__ partial) {
  __shared__ double red[16];
  const int tid = threadIdx.x;
  const int64_t stride = (int64_t)gridDim.x * 1024;
  double a = 0.0;
  for (int64_t j = (int64_t)blockIdx.x * 1024 + tid; j < d; j += 8 * stride) {
    float v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = j + q * stride < d ? w[j + q * stride] : 0.0f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const double x = (double)v[q];
      a += l1 * fabs(x) + 0.5 * l2 * x * x;
    }
  }
  a = wave_sum(a);
  if ((tid & 63) == 0) red[tid >> 6] = a;
  __syncthreads();
  if (tid == 0) {
    double t = 0.0;
    for (int k = 0; k < 16; ++k) t += red[k];
    partial[blockIdx.x] = t;
  }
}

// acc += the n <= 256 partials: lane l takes partial[l], [l+64], [l+128], [l+192], then the wavefront sum (one
// wavefront; a fixed order)
__global__ __launch_bounds__(64) void objective_reg_fold_kernel(const double *__restrict__ partial, int32_t n,
                                                               double *__restrict__ acc) {
  const int lane = threadIdx.x;
  double v[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) v[q] = lane + 64 * q < n ? partial[lane + 64 * q] : 0.0;
  const double t = wave_sum((v[0] + v[1]) + (v[2] + v[3]));
  if (lane == 0) *acc += t;
}

QuantSpec spec_of(const lpc_ctx *c) {
  QuantSpec qs;
  qs.bits = c->cfg.bits;
  qs.clip_mode = c->cfg.clip_mode;
  qs.clip = c->cfg.clip;
  qs.enabled = c->quant ? 1 : 0;
  return qs;
}

StatSinks sinks_of(const lpc_ctx *c, double *stats_out) {
  StatSinks sk;
  sk.stat_part = c->s.stat_part;
  sk.stats = c->s.stats;
  sk.qparams = c->s.qparams;
  sk.flags = c->s.flags;
  sk.n_clipped = c->s.n_clipped;
  sk.stats_out = stats_out;
  sk.stat_slots = c->stat_slots;
  return sk;
}

inline dim3 grid1d(int64_t n, int threads) { return dim3((unsigned)((n + threads - 1) / threads)); }

}  // namespace

// Wavefronts per workgroup of the fold of `parts` partial rows into nvec vectors (they take interleaved rows, which
// fixes the order of the sum).  A wavefront takes eight partial rows per step: two wavefronts for up to 16 rows
// when the launch has workgroups to spare, four otherwise (measured back to back on one machine: 16 rows and 2176
// workgroups, two against four wavefronts +0.9 % inner iterations/s, eight -3.9 %; 16 rows and 4 workgroups,
// two -2 %; 32 rows, two -2.3 %, eight +0.2 %)
int reduce_parts_waves(const lpc_ctx *c, int32_t parts, int32_t nvec) {
  const int64_t wgs = ((c->d_pad + 63) / 64) * (int64_t)nvec;
  return (parts <= 16 && wgs >= 2 * c->cus) ? 2 : 4;
}

hipError_t launch_reduce_parts(const lpc_ctx *c, const float *part, int32_t parts, float scale, float *out,
                               int64_t ld_out, int32_t vec_begin, int32_t nvec, int stats_mode, double *stats_out,
                               hipStream_t st) {
  // `out` and `stats_out` point at the row of the first vector of this launch; vec_begin only selects
  // the scratch slots (statistics, quantizer parameters).
  const dim3 grid((unsigned)((c->d_pad + 63) / 64), (unsigned)nvec);
  if (reduce_parts_waves(c, parts, nvec) == 2)
    LPC_LAUNCH_TIMED(reduce_parts_kernel<2>, grid, dim3(128), st, part, parts, c->d, c->d_pad, scale, out, ld_out,
                     vec_begin, (int32_t)stats_mode, sinks_of(c, stats_out));
  else
    LPC_LAUNCH_TIMED(reduce_parts_kernel<4>, grid, dim3(256), st, part, parts, c->d, c->d_pad, scale, out, ld_out,
                     vec_begin, (int32_t)stats_mode, sinks_of(c, stats_out));
  if (stats_mode == kStatsFinal)
    hipLaunchKernelGGL(finalize_stats_kernel, dim3((unsigned)nvec), dim3(64), 0, st, sinks_of(c, stats_out),
                       spec_of(c), vec_begin, (int32_t)grid.x, c->d);
  return hipGetLastError();
}

hipError_t launch_range_stats(const lpc_ctx *c, const float *U, int64_t ld, int32_t vec_begin, int32_t nvec,
                              const StatRange &ranges, int32_t slot0, hipStream_t st) {
  if (ranges.n <= 0) return hipSuccess;
  hipLaunchKernelGGL(range_stats_kernel, dim3((unsigned)ranges.n, (unsigned)nvec), dim3(kThreads), 0, st, U, ld, ranges,
                     vec_begin, slot0, sinks_of(c, nullptr));
  return hipGetLastError();
}

hipError_t launch_finalize_stats(const lpc_ctx *c, int32_t vec_begin, int32_t nvec, int32_t nslots, double *stats_out,
                                 hipStream_t st) {
  hipLaunchKernelGGL(finalize_stats_kernel, dim3((unsigned)nvec), dim3(64), 0, st, sinks_of(c, stats_out), spec_of(c),
                     vec_begin, nslots, c->d);
  return hipGetLastError();
}

hipError_t launch_vector_stats(const lpc_ctx *c, const float *U, int64_t ld, int32_t vec_begin, int32_t nvec,
                               double *stats_out, int stats_mode, int32_t *slots_used, hipStream_t st) {
  // 1K..32K coordinates per workgroup: short vectors spread wide (latency), long ones keep the number of
  // statistic partials (and of fenced arrivals) small
  int64_t chunk = ((c->d / 64 + 1023) / 1024) * 1024;
  chunk = chunk < 1024 ? 1024 : (chunk > 32768 ? 32768 : chunk);
  int64_t slots = (c->d + chunk - 1) / chunk;
  if (slots > c->stat_slots) {  // cannot happen for chunk >= 64, kept as a guard for the scratch layout
    slots = c->stat_slots;
    chunk = (((c->d + slots - 1) / slots) + 3) / 4 * 4;
    slots = (c->d + chunk - 1) / chunk;
  }
  const dim3 grid((unsigned)slots, (unsigned)nvec);
  hipLaunchKernelGGL(vector_stats_kernel, grid, dim3(kThreads), 0, st, U, ld, c->d, chunk, vec_begin,
                     sinks_of(c, stats_out));
  if (stats_mode == kStatsFinal)
    hipLaunchKernelGGL(finalize_stats_kernel, dim3((unsigned)nvec), dim3(64), 0, st, sinks_of(c, stats_out),
                       spec_of(c), vec_begin, (int32_t)slots, c->d);
  if (slots_used) *slots_used = (int32_t)slots;
  return hipGetLastError();
}

hipError_t launch_prepare_qparams(const lpc_ctx *c, const double *stats, const float *delta_in, int32_t nvec,
                                  hipStream_t st) {
  hipLaunchKernelGGL(prepare_qparams_kernel, grid1d(nvec, 64), dim3(64), 0, st, stats, delta_in, nvec, c->d,
                     spec_of(c), c->s.qparams, c->s.n_clipped, c->s.flags);
  return hipGetLastError();
}

namespace {
template <int B>
void quantize_launch(const lpc_ctx *c, const float *U, StreamKey key, uint32_t *packed, float *delta_out,
                     uint32_t *n_clipped, hipStream_t st) {
  // evaluation runs and callers of lpc_quantize_clip want the clip counts; the epoch's own launches do not, and
  // on dense vectors they also draw unconditionally
  if constexpr (B == 2 || B == 4 || B == 8) {
    const dim3 grid((unsigned)((c->W + kThreads - 1) / kThreads), (unsigned)c->cfg.N);
    if (n_clipped)
      hipLaunchKernelGGL((quantize_word_kernel<B, true, true>), grid, dim3(kThreads), 0, st, U, c->d, c->d_pad,
                         c->s.qparams, key, packed, c->W, delta_out, n_clipped);
    else if (c->csr)
      hipLaunchKernelGGL((quantize_word_kernel<B, false, true>), grid, dim3(kThreads), 0, st, U, c->d, c->d_pad,
                         c->s.qparams, key, packed, c->W, delta_out, n_clipped);
    else
      hipLaunchKernelGGL((quantize_word_kernel<B, false, false>), grid, dim3(kThreads), 0, st, U, c->d, c->d_pad,
                         c->s.qparams, key, packed, c->W, delta_out, n_clipped);
  } else {
    const dim3 grid((unsigned)((c->d_pad + kTileFloats - 1) / kTileFloats), (unsigned)c->cfg.N);
    if (n_clipped)
      hipLaunchKernelGGL((quantize_kernel<B, true, true>), grid, dim3(kThreads), 0, st, U, c->d, c->d_pad,
                         c->s.qparams, key, packed, c->W, delta_out, n_clipped);
    else if (c->csr)
      hipLaunchKernelGGL((quantize_kernel<B, false, true>), grid, dim3(kThreads), 0, st, U, c->d, c->d_pad,
                         c->s.qparams, key, packed, c->W, delta_out, n_clipped);
    else
      hipLaunchKernelGGL((quantize_kernel<B, false, false>), grid, dim3(kThreads), 0, st, U, c->d, c->d_pad,
                         c->s.qparams, key, packed, c->W, delta_out, n_clipped);
  }
}

template <int B, bool PROX>
void dequantize_launch(const lpc_ctx *c, const uint32_t *packed, const float *delta, float *u_avg, ProxArgs pa,
                       hipStream_t st) {
  if constexpr (32 % (8 * B) == 0) {
    const int64_t threads = c->d_pad / 8;
    hipLaunchKernelGGL((dequantize_quarter_kernel<B, PROX>),
                       dim3((unsigned)((threads + kQuarterThreads - 1) / kQuarterThreads)), dim3(kQuarterThreads), 0, st,
                       packed, c->W, delta, c->cfg.N, c->d, c->d_pad, u_avg, pa);
  } else {
    const int64_t wide = (c->d_pad + kTileFloats - 1) / kTileFloats;
    if (wide >= 2 * c->cus) {
      hipLaunchKernelGGL((dequantize_kernel<B, PROX, kThreads>), dim3((unsigned)wide), dim3(kThreads), 0, st, packed,
                         c->W, delta, c->cfg.N, c->d, c->d_pad, u_avg, pa);
    } else {
      const int64_t tile = 64 * kSegFloats;
      hipLaunchKernelGGL((dequantize_kernel<B, PROX, 64>), dim3((unsigned)((c->d_pad + tile - 1) / tile)), dim3(64), 0,
                         st, packed, c->W, delta, c->cfg.N, c->d, c->d_pad, u_avg, pa);
    }
  }
}

#define LPC_DISPATCH_BITS(bits, CALL)                                                                     \
  switch (bits) {                                                                                         \
    case 2: CALL(2); break;   case 3: CALL(3); break;   case 4: CALL(4); break;   case 5: CALL(5); break;   \
    case 6: CALL(6); break;   case 7: CALL(7); break;   case 8: CALL(8); break;   case 9: CALL(9); break;   \
    case 10: CALL(10); break; case 11: CALL(11); break; case 12: CALL(12); break; case 13: CALL(13); break; \
    case 14: CALL(14); break; case 15: CALL(15); break; case 16: CALL(16); break;                          \
    default: return hipErrorInvalidValue;                                                                 \
  }
}  // namespace

hipError_t launch_quantize(const lpc_ctx *c, const float *U, StreamKey key, uint32_t *packed, float *delta_out,
                           uint32_t *n_clipped, hipStream_t st) {
#define CALL(BITS) quantize_launch<BITS>(c, U, key, packed, delta_out, n_clipped, st)
  LPC_DISPATCH_BITS(c->cfg.bits, CALL)
#undef CALL
  return hipGetLastError();
}

hipError_t launch_dequantize_avg(const lpc_ctx *c, const uint32_t *packed, const float *delta, float *u_avg,
                                 hipStream_t st) {
  ProxArgs pa{nullptr, nullptr, 0.f, 0.f, 0.f, nullptr, nullptr, 0};
#define CALL(BITS) dequantize_launch<BITS, false>(c, packed, delta, u_avg, pa, st)
  LPC_DISPATCH_BITS(c->cfg.bits, CALL)
#undef CALL
  return hipGetLastError();
}

namespace {
inline void prox_consts(const lpc_ctx *c, float step, float *thr, float *shrink) {
  *thr = (float)((double)step * (double)c->prob.lambda1);
  *shrink = (float)(1.0 / (1.0 + (double)step * (double)c->prob.lambda2));
}
}  // namespace

hipError_t launch_dequantize_prox(const lpc_ctx *c, const uint32_t *packed, const float *delta, const float *mu,
                                  float step, float *w, float *u_avg_out, hipStream_t st) {
  ProxArgs pa{mu, w, step, 0.f, 0.f, nullptr, nullptr, 0};
  prox_consts(c, step, &pa.thr, &pa.shrink);
#define CALL(BITS) dequantize_launch<BITS, true>(c, packed, delta, u_avg_out, pa, st)
  LPC_DISPATCH_BITS(c->cfg.bits, CALL)
#undef CALL
  return hipGetLastError();
}

namespace {
SparseArgs sparse_args_of(const lpc_ctx *c) {
  SparseArgs a{};
  a.U = c->s.U; a.planes = c->s.sparse_planes; a.head_part = c->s.part; a.touched = c->s.touched;
  a.touched_parts = c->s.touched_parts;
  a.d_pad = c->d_pad; a.W = c->W; a.bitmap_words = c->bitmap_words;
  a.head = c->sparse_head; a.parts = csr_sparse_parts(c->cfg.B); a.N = c->cfg.N;
  return a;
}
}  // namespace

namespace {
// workgroups per worker that cover the tail: four wavefronts of kWaveSegs segments each
int32_t sparse_tail_wgs(const lpc_ctx *c) {
  const int64_t tail_segs = (c->d_pad - c->sparse_head) / kSegFloats;
  return (int32_t)((tail_segs + 4 * kWaveSegs - 1) / (4 * kWaveSegs));  // four wavefronts per workgroup
}
int32_t sparse_stat_slots(const lpc_ctx *c) { return c->sparse_head / (4 * kThreads) + sparse_tail_wgs(c); }
}  // namespace

// statistic partials of the N sparse vectors left by launch_csr_vr_sparse
hipError_t launch_sparse_stats(const lpc_ctx *c, int32_t nvec, hipStream_t st) {
  hipLaunchKernelGGL(sparse_stats_kernel, dim3((unsigned)sparse_stat_slots(c), (unsigned)nvec), dim3(kThreads), 0,
                     st, sparse_args_of(c), sinks_of(c, nullptr));
  return hipGetLastError();
}

hipError_t launch_sparse_quantize(const lpc_ctx *c, StreamKey key, bool share_delta, hipStream_t st) {
  // 32 head segments per workgroup, then the tail workgroups
  const dim3 grid((unsigned)(c->sparse_head / (32 * kSegFloats) + sparse_tail_wgs(c)), (unsigned)c->cfg.N);
  const int32_t slots = sparse_stat_slots(c);
#define CALL(BITS)                                                                                             \
  hipLaunchKernelGGL(sparse_quantize_kernel<BITS>, grid, dim3(kThreads), 0, st, sparse_args_of(c), sinks_of(c, nullptr), \
                     spec_of(c), slots, c->d, key, share_delta ? 1 : 0, c->s.packed, c->s.delta)
  LPC_DISPATCH_BITS(c->cfg.bits, CALL)
#undef CALL
  return hipGetLastError();
}

hipError_t launch_sparse_receive_prox(const lpc_ctx *c, const float *mu, float step, float *w, hipStream_t st) {
  ProxArgs pa{mu, w, step, 0.f, 0.f, c->s.packed, c->s.touched, c->bitmap_words};
  prox_consts(c, step, &pa.thr, &pa.shrink);
#define CALL(BITS) dequantize_launch<BITS, true>(c, c->s.packed, c->s.delta, nullptr, pa, st)
  LPC_DISPATCH_BITS(c->cfg.bits, CALL)
#undef CALL
  return hipGetLastError();
}

namespace {
// Fills the warming fields and returns the number of extra workgroups (0 when there is nothing to warm: no
// next iteration in this epoch, other data kinds).  `shared`: the
// next worker pass also reads the shared batch J as worker index N.
int warm_setup(const lpc_ctx *c, StreamKey key, bool shared, FusedArgs *a) {
  a->warm_groups = 0;
  if (key.iter + 1 >= (uint32_t)c->cfg.m || c->csr || c->mlp || !c->grad_ok) return 0;
  const int32_t workers = c->cfg.N + (shared ? 1 : 0);
  const int32_t parts = c->vr_parts, B = c->cfg.B;
  const int32_t rows_per_part = (B + parts - 1) / parts;
  // measured: 8.5 MB arrive within the exchange's own 6 us; with 16 MB or more the requests outlast it and the
  // launch grows by what the next worker pass saves.  Larger batches are warmed in part (their first workgroups):
  // with more than two rows per workgroup the rows are requested four at a time and 18 MB pay (d = 8192, N = 16 + the
  // shared batch, B = 64: 9 MB +1.8 %, 14 MB +2.9 %, 18 MB +3.6 %, 24 MB +3.1 % inner iterations/s over rows requested
  // one after the other with a 9 MB cap).
  const int64_t cap = (int64_t)(rows_per_part > 2 ? 18 : 9) << 20;
  const int64_t bytes_per_group = (int64_t)rows_per_part * c->d * 4;
  const int64_t groups_cap = cap / bytes_per_group;
  if (groups_cap < 1) return 0;
  a->warm_X = c->prob.X; a->warm_ldx = c->prob.ldx; a->warm_y = c->prob.y;
  a->warm_z = (c->n_full == c->n) ? c->s.z_snap : nullptr;
  a->warm_n = c->n;
  a->warm_key = key;
  a->warm_key.iter = key.iter + 1;
  a->warm_shared = shared ? c->cfg.N : -1;
  a->warm_groups = (int32_t)(groups_cap < (int64_t)workers * parts ? groups_cap : (int64_t)workers * parts); a->warm_parts = parts; a->warm_rows_per_part = rows_per_part; a->warm_B = B;
  a->warm_sink = c->s.warm_sink;
  return a->warm_groups;
}
}  // namespace

bool fused_exchange_supported(const lpc_ctx *c) {
  return c->quant && c->cfg.N <= kFusedMaxN && c->stat_slots <= 256 && c->d_pad <= 16384;
}

// One launch for eq. (3), quantize, pack, eq. (4) and (optionally) the proximal step; reads the statistic
// partials left by launch_reduce_parts(..., kStatsPartial, ...) for vectors 0..N-1.
hipError_t launch_fused_exchange(const lpc_ctx *c, const float *U, int32_t nslots, StreamKey key, uint32_t *packed,
                                 float *delta_out, const float *mu, float step, float *w, float *u_avg_out,
                                 hipStream_t st) {
  FusedArgs a{};
  a.U = U; a.d = c->d; a.d_pad = c->d_pad; a.W = c->W;
  a.N = c->cfg.N; a.bits = c->cfg.bits; a.nslots = nslots; a.stat_slots = c->stat_slots;
  a.stat_part = c->s.stat_part; a.qs = spec_of(c); a.key = key;
  a.packed = packed; a.delta_out = delta_out; a.stats = c->s.stats; a.flags = c->s.flags;
  a.mu = mu; a.w = w; a.w_in = w; a.u_avg_out = u_avg_out; a.step = step; a.do_prox = w != nullptr ? 1 : 0;
  prox_consts(c, step > 0.0f ? step : 1.0f, &a.thr, &a.shrink);
  const int extra = w != nullptr ? warm_setup(c, key, false, &a) : 0;
  const dim3 grid((unsigned)((c->d_pad + kFusedCoords - 1) / kFusedCoords + extra));
  LPC_LAUNCH_TIMED(fused_exchange_kernel, grid, dim3(kFusedThreads), st, a);
  return hipGetLastError();
}

hipError_t launch_fused_exchange_alpc(const lpc_ctx *c, const float *U, int32_t nslots, StreamKey key,
                                      uint32_t *packed, float *delta_out, const AlpcStep &al, hipStream_t st) {
  FusedArgs a{};
  a.U = U; a.d = c->d; a.d_pad = c->d_pad; a.W = c->W;
  a.N = c->cfg.N; a.bits = c->cfg.bits; a.nslots = nslots; a.stat_slots = c->stat_slots;
  a.stat_part = c->s.stat_part; a.qs = spec_of(c); a.key = key;
  a.packed = packed; a.delta_out = delta_out; a.stats = c->s.stats; a.flags = c->s.flags;
  a.mu = al.mu; a.do_alpc = 1;
  a.x = al.x; a.u_hat = al.u_hat; a.w_snap = al.w_snap; a.y = al.y; a.z = al.z; a.z_in = al.z; a.ysum = al.ysum;
  a.x_next = al.x_next;
  a.step_y = al.step_y; a.alpha = al.alpha; a.weight = al.weight; a.first = al.first;
  a.t1 = al.tau1; a.t2 = al.tau2; a.t3 = (float)(1.0 - (double)al.tau1 - (double)al.tau2);
  prox_consts(c, al.step_y, &a.thr_y, &a.shrink_y);
  prox_consts(c, al.alpha, &a.thr_z, &a.shrink_z);
  const int extra = warm_setup(c, key, true, &a);
  const dim3 grid((unsigned)((c->d_pad + kFusedCoords - 1) / kFusedCoords + extra));
  LPC_LAUNCH_TIMED(fused_exchange_kernel, grid, dim3(kFusedThreads), st, a);
  return hipGetLastError();
}

// The exchange of the column-tile iteration: reads U and the statistic partials the column-tile worker pass left
// (one slot per tile), updates the iterate (Alg. 1: w_in -> w_out; Alg. 2/3: al->x -> al->x_next, z_in -> al->z),
// and, when next_pd is given, leaves the partial dots of the rows iteration key.iter + 1 samples (nvec_next
// vectors, the last one the shared batch for Alg. 2/3) with the new iterate.
hipError_t launch_cols_exchange(const lpc_ctx *c, const float *U, StreamKey key, uint32_t *packed, float *delta_out,
                                const float *mu, float step, const float *w_in, float *w_out, const AlpcStep *al,
                                const float *z_in, float *next_pd, hipStream_t st) {
  FusedArgs a{};
  a.U = U; a.d = c->d; a.d_pad = c->d_pad; a.W = c->W;
  a.N = c->cfg.N; a.bits = c->cfg.bits; a.nslots = dense_cols_tiles(c); a.stat_slots = c->stat_slots;
  a.stat_part = c->s.stat_part; a.qs = spec_of(c); a.key = key;
  a.packed = packed; a.delta_out = delta_out; a.stats = c->s.stats; a.flags = c->s.flags;
  if (al) {
    a.mu = al->mu; a.do_alpc = 1;
    a.x = al->x; a.u_hat = al->u_hat; a.w_snap = al->w_snap; a.y = al->y; a.z = al->z; a.z_in = z_in;
    a.ysum = al->ysum; a.x_next = al->x_next;
    a.step_y = al->step_y; a.alpha = al->alpha; a.weight = al->weight; a.first = al->first;
    a.t1 = al->tau1; a.t2 = al->tau2; a.t3 = (float)(1.0 - (double)al->tau1 - (double)al->tau2);
    prox_consts(c, al->step_y, &a.thr_y, &a.shrink_y);
    prox_consts(c, al->alpha, &a.thr_z, &a.shrink_z);
  } else {
    a.mu = mu; a.w = w_out; a.w_in = w_in; a.step = step; a.do_prox = 1;
    prox_consts(c, step, &a.thr, &a.shrink);
  }
  const int tiles = dense_cols_tiles(c);
  a.dots_R = 1;
  if (next_pd) {
    DotsArgs &dd = a.dots;
    dd.X = c->prob.X; dd.ldx = c->prob.ldx; dd.d = c->d; dd.n = c->n; dd.w = nullptr; dd.pd = next_pd;
    dd.C = tiles; dd.B = c->cfg.B; dd.nvec = c->cfg.N + (al ? 1 : 0); dd.worker_begin = 0;
    dd.shared_rel = al ? c->cfg.N : -1;
    dd.vec4 = (c->d % 4 == 0 && c->prob.ldx % 4 == 0 && (((uintptr_t)c->prob.X) & 15u) == 0) ? 1 : 0;
    dd.key = key; dd.key.iter = key.iter + 1; dd.tag = kTagBatch;
    const int32_t rows = dd.nvec * dd.B;
    int groups = dense_dots_groups(c, rows);
    const int least = (rows + kDotRows - 1) / kDotRows;  // a workgroup holds at most kDotRows rows in registers
    if (groups < least) groups = least;
    dd.rows_per_wg = (rows + groups - 1) / groups;
    a.dots_R = groups;
  } else {
    a.dots.rows_per_wg = 0; a.dots.nvec = 0; a.dots.B = 1; a.dots.C = tiles;
  }
  LPC_LAUNCH_TIMED(fused_exchange_kernel, dim3((unsigned)(tiles * a.dots_R)), dim3(kFusedThreads), st, a);
  return hipGetLastError();
}

bool fused_iter_supported(const lpc_ctx *c) {
  return fused_exchange_supported(c) && c->grad_ok && !c->csr && !c->mlp;
}

// 64-bit words of the two slot sets the workgroups of launch_fused_iter exchange their statistics through
int64_t fused_iter_slot_words(const lpc_ctx *c) {
  return 2 * ((c->d_pad + 63) / 64) * (int64_t)c->cfg.N * 4;
}

hipError_t launch_fused_iter_reset(const lpc_ctx *c, hipStream_t st) {
  return launch_fill_u32(reinterpret_cast<uint32_t *>(c->s.iter_slots), 0xFFFFFFFFu, 2 * fused_iter_slot_words(c), st);
}

// Fold of the workers' partial rows (and of the shared batch's when `al` is given), eq. (3), quantize, pack, eq. (4)
// and the update in one launch; iteration key.iter uses slot set key.iter & 1.
hipError_t launch_fused_iter(const lpc_ctx *c, StreamKey key, uint32_t *packed, float *delta_out, const float *mu,
                             float step, float *w, const AlpcStep *al, hipStream_t st) {
  IterArgs ia{};
  FusedArgs &a = ia.f;
  a.d = c->d; a.d_pad = c->d_pad; a.W = c->W;
  a.N = c->cfg.N; a.bits = c->cfg.bits; a.stat_slots = c->stat_slots;
  a.qs = spec_of(c); a.key = key;
  a.packed = packed; a.delta_out = delta_out; a.stats = c->s.stats; a.flags = c->s.flags;
  int extra;
  if (al) {
    a.mu = al->mu; a.do_alpc = 1;
    a.x = al->x; a.w_snap = al->w_snap; a.y = al->y; a.z = al->z; a.ysum = al->ysum; a.x_next = al->x_next;
    a.step_y = al->step_y; a.alpha = al->alpha; a.weight = al->weight; a.first = al->first;
    a.t1 = al->tau1; a.t2 = al->tau2; a.t3 = (float)(1.0 - (double)al->tau1 - (double)al->tau2);
    prox_consts(c, al->step_y, &a.thr_y, &a.shrink_y);
    prox_consts(c, al->alpha, &a.thr_z, &a.shrink_z);
    extra = warm_setup(c, key, true, &a);
  } else {
    a.mu = mu; a.w = w; a.w_in = w; a.step = step; a.do_prox = 1;
    prox_consts(c, step, &a.thr, &a.shrink);
    extra = warm_setup(c, key, false, &a);
  }
  ia.part = c->s.part; ia.parts = c->vr_parts; ia.nvec = c->cfg.N + (al ? 1 : 0);
  ia.nwf = reduce_parts_waves(c, c->vr_parts, ia.nvec);
  ia.vec4 = (c->d % 4 == 0) ? 1 : 0;
  ia.scale = (float)(1.0 / (double)c->cfg.B);
  const int64_t set_words = fused_iter_slot_words(c) / 2;
  ia.slots_cur = c->s.iter_slots + (key.iter & 1u) * set_words;
  ia.slots_next = c->s.iter_slots + ((key.iter + 1u) & 1u) * set_words;
  ia.spin_limit = c->spin_limit;
  const int tile = c->iter_tile == 64 ? 64 : 128;
  const dim3 grid((unsigned)((c->d_pad + tile - 1) / tile + extra));
  if (tile == 64 && c->iter_threads == 256)
    LPC_LAUNCH_TIMED((fused_iter_kernel<256, 64>), grid, dim3(256), st, ia);
  else if (tile == 64)
    LPC_LAUNCH_TIMED((fused_iter_kernel<512, 64>), grid, dim3(512), st, ia);
  else if (c->iter_threads == 256)
    LPC_LAUNCH_TIMED((fused_iter_kernel<256, 128>), grid, dim3(256), st, ia);
  else
    LPC_LAUNCH_TIMED((fused_iter_kernel<512, 128>), grid, dim3(512), st, ia);
  return hipGetLastError();
}

hipError_t launch_share_delta(const lpc_ctx *c, int32_t nvec, float *delta_out, hipStream_t st) {
  hipLaunchKernelGGL(share_delta_kernel, dim3(1), dim3(64), 0, st, c->s.qparams, nvec, spec_of(c), delta_out);
  return hipGetLastError();
}

namespace {
template <int B>
void dequantize_shared_launch(const lpc_ctx *c, const uint32_t *packed, const float *delta, bool requant,
                              StreamKey key, float *u_avg, hipStream_t st) {
  const dim3 grid((unsigned)((c->d_pad + kTileFloats - 1) / kTileFloats));
  if (requant)
    hipLaunchKernelGGL((dequantize_shared_kernel<B, true>), grid, dim3(kThreads), 0, st, packed, c->W, delta,
                       c->cfg.N, c->d, c->d_pad, key, u_avg);
  else
    hipLaunchKernelGGL((dequantize_shared_kernel<B, false>), grid, dim3(kThreads), 0, st, packed, c->W, delta,
                       c->cfg.N, c->d, c->d_pad, key, u_avg);
}
}  // namespace

hipError_t launch_dequantize_shared(const lpc_ctx *c, const uint32_t *packed, const float *delta, bool requant,
                                    StreamKey key, float *u_avg, hipStream_t st) {
#define CALL(BITS) dequantize_shared_launch<BITS>(c, packed, delta, requant, key, u_avg, st)
  LPC_DISPATCH_BITS(c->cfg.bits, CALL)
#undef CALL
  return hipGetLastError();
}

hipError_t launch_plain_avg(const lpc_ctx *c, const float *U, float *u_avg, hipStream_t st) {
  hipLaunchKernelGGL(plain_avg_kernel, grid1d(c->d, 256), dim3(256), 0, st, U, c->d, c->d_pad, c->cfg.N, u_avg);
  return hipGetLastError();
}

hipError_t launch_prox(const lpc_ctx *c, float *w, const float *u_avg, const float *mu, float step, hipStream_t st) {
  float thr, shrink;
  prox_consts(c, step, &thr, &shrink);
  hipLaunchKernelGGL(prox_kernel, grid1d(c->d, 256), dim3(256), 0, st, w, u_avg, mu, c->d, step, thr, shrink);
  return hipGetLastError();
}

hipError_t launch_finish_full_grad(const lpc_ctx *c, int32_t parts, int64_t cols, float scale, float *mu,
                                   double *f_out, bool want_loss, hipStream_t st) {
  // the partial rows are `cols` floats long; mu[0..cols) = scale * their sum
  if (mu) {
    const float *src = c->s.part;
    int32_t left = parts;
    const dim3 grid((unsigned)((cols + 63) / 64), 1u);
    if (c->fold_slices > 1 && parts % c->fold_slices == 0) {
      // first level: fold_slices groups of consecutive partial rows, all columns in parallel
      const dim3 grid1(grid.x, (unsigned)c->fold_slices);
      hipLaunchKernelGGL(reduce_parts_kernel<4>, grid1, dim3(kThreads), 0, st, src, parts / c->fold_slices, cols, cols,
                         1.0f, c->s.part2, cols, 0, kStatsNone, sinks_of(c, nullptr));
      src = c->s.part2;
      left = c->fold_slices;
    }
    hipLaunchKernelGGL(reduce_parts_kernel<4>, grid, dim3(kThreads), 0, st, src, left, cols, cols, scale, mu, cols, 0,
                       kStatsNone, sinks_of(c, nullptr));
  }
  if (want_loss && f_out)
    hipLaunchKernelGGL(sum_loss_kernel, dim3(1), dim3(kThreads), 0, st, (const double *)c->s.part_loss, parts,
                       (double)scale, f_out);
  return hipGetLastError();
}

hipError_t launch_copy(float *dst, const float *src, int64_t n, hipStream_t st) {
  hipLaunchKernelGGL(copy_kernel, grid1d(n, 256), dim3(256), 0, st, dst, src, n);
  return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t *dst, uint32_t v, int64_t n, hipStream_t st) {
  hipLaunchKernelGGL(fill_u32_kernel, grid1d(n, 256), dim3(256), 0, st, dst, v, n);
  return hipGetLastError();
}

hipError_t launch_alpc_couple(const lpc_ctx *c, const float *z, const float *w_snap, const float *y, float tau1,
                              float tau2, float *x, hipStream_t st) {
  const float t3 = (float)(1.0 - (double)tau1 - (double)tau2);
  hipLaunchKernelGGL(alpc_couple_kernel, grid1d(c->d, 256), dim3(256), 0, st, z, w_snap, y, tau1, tau2, t3, x, c->d);
  return hipGetLastError();
}

hipError_t launch_alpc_update(const lpc_ctx *c, const float *x, const float *u_avg, const float *u_hat,
                              const float *mu, float step_y, float alpha, float weight, bool first, float *y,
                              float *z, float *ysum, hipStream_t st) {
  float thr_y, shrink_y, thr_z, shrink_z;
  prox_consts(c, step_y, &thr_y, &shrink_y);
  prox_consts(c, alpha, &thr_z, &shrink_z);
  hipLaunchKernelGGL(alpc_update_kernel, grid1d(c->d, 256), dim3(256), 0, st, x, u_avg, u_hat, mu, step_y, thr_y,
                     shrink_y, alpha, thr_z, shrink_z, weight, first ? 1 : 0, y, z, ysum, c->d);
  return hipGetLastError();
}

hipError_t launch_alpc_update_couple(const lpc_ctx *c, const AlpcStep &al, hipStream_t st) {
  float thr_y, shrink_y, thr_z, shrink_z;
  prox_consts(c, al.step_y, &thr_y, &shrink_y);
  prox_consts(c, al.alpha, &thr_z, &shrink_z);
  const float t3 = (float)(1.0 - (double)al.tau1 - (double)al.tau2);
  hipLaunchKernelGGL(alpc_update_couple_kernel, grid1d(c->d, 256), dim3(256), 0, st, al.x, c->s.u_avg,
                     const_cast<float *>(al.u_hat), al.mu, al.w_snap, al.step_y, thr_y, shrink_y, al.alpha, thr_z,
                     shrink_z, al.weight, al.first, al.tau1, al.tau2, t3, al.y, al.z, al.ysum, al.x_next, c->d);
  return hipGetLastError();
}

hipError_t launch_scale_to(const lpc_ctx *c, const float *src, float scale, float *dst, hipStream_t st) {
  hipLaunchKernelGGL(scale_to_kernel, grid1d(c->d, 256), dim3(256), 0, st, src, scale, dst, c->d);
  return hipGetLastError();
}

hipError_t launch_objective_reg(const lpc_ctx *c, const float *w, double *acc, hipStream_t st) {
  // one workgroup per 8192 coordinates, at most as many as the statistic scratch (free outside an epoch) holds
  int64_t groups = (c->d + 8191) / 8192;
  const int64_t room = (int64_t)(c->cfg.N + 1) * c->stat_slots * 4;
  if (groups > room) groups = room;
  if (groups > 256) groups = 256;
  hipLaunchKernelGGL(objective_reg_kernel, dim3((unsigned)groups), dim3(1024), 0, st, w, c->d,
                     (double)c->prob.lambda1, (double)c->prob.lambda2, c->s.stat_part);
  hipLaunchKernelGGL(objective_reg_fold_kernel, dim3(1), dim3(64), 0, st, (const double *)c->s.stat_part,
                     (int32_t)groups, acc);
  return hipGetLastError();
}

}  // namespace lpc
