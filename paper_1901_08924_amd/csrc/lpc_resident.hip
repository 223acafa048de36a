// The inner loop of an epoch (Alg. 1 steps 5-11; Alg. 2 steps 5-15) as ONE resident launch for dense data of
// moderate width (d_pad <= 16384, N <= 64): 256 workgroups of 1024 threads, one per compute unit, stay on the chip
// for all m inner iterations and hand each other what the paper's workers send over the wire.
//
// The chip is used the way the method is distributed.  An MI355X is eight dies (XCDs) of 32 compute units, each
// die with its own L2; workgroup k of a launch runs on die k mod 8, and a workgroup reads its die's number from the
// XCC_ID hardware register.  Worker i lives on die i mod 8:
//
//   rows      the rows that a die's workers sample are dealt to its 32 compute units in contiguous shares; each
//             forms the margins, the slope differences against the cached snapshot margins and slope * row
//             (Alg. 1 step 6) and leaves one partial vector per worker it touched in the die's L2;
//   fold      after a barrier among the die's 32 workgroups, compute unit c adds the partial vectors over its own
//             slice of the coordinates (a fixed order), takes the slice's statistics, and publishes the slice of
//             u^i and the statistics for every die to read;
//   exchange  compute unit c of EVERY die reads slice c of all N vectors and the statistics of all slices, forms
//             delta_i (eq. (3)), quantizes the slice of every worker's vector (Sec. 3.2 rules (1), (2); the random
//             stream is a function of (worker, coordinate, iteration), so all dies get the same codes), averages
//             the codes (eq. (4)) and takes the proximal step (Alg. 1 steps 9-10, or Alg. 2 steps 13-15 with the
//             next step 6) for its slice.  Die 0 also stores the packed messages.  Every die thus holds the new
//             iterate, one slice per compute unit, and every compute unit reads the whole of it from its die's L2
//             for the next margins.
//
// One barrier among 32 workgroups per iteration replaces three kernel launches.  Everything else that crosses
// workgroups travels as self-validating 64-bit words (value, tag): the tag is a number that grows with every
// iteration of every launch of the context, a reader loads the word with one 64-bit atomic load and takes the value
// once the tag is the one it expects, so neither a flag nor an acknowledged store stands between writer and reader.
// The shared batch J of Alg. 2 is spread over the dies; each die publishes its partial sum and the exchange step
// adds the eight.
//
// Memory rules.  Partial vectors (read inside the die, after the barrier) are written with ordinary stores -- the
// vector L1 writes through to the die's L2, and a wave waits for its stores to be acknowledged before its workgroup
// arrives at the barrier -- and read with agent-scope atomic loads, which bypass the reader's L1.  Tagged words
// are written with 64-bit atomic stores (agent scope where they cross dies) and read with agent-scope atomic loads.
// The barrier counter is bumped with atomics that execute in the die's L2.  Every wait is bounded: after
// spin_limit polls a workgroup raises the abort word and flag bit 1, leaves the loop, and every other workgroup
// follows at its next wait, so all waves exit whatever happens; the host then reports LPC_EDEVICE.  The launch is
// cooperative, so all 256 workgroups are resident together.
//
// Which rows an iteration samples does not depend on the iterate.  Wavefronts 0-7 of a workgroup draw the coming
// iteration's rows as soon as this iteration's are consumed, load their labels and cached margins, and touch one
// word per 128-byte line of each row, so that the rows travel from HBM towards the die's L2 while wavefronts 8-15
// fold and exchange; fold and exchange are kept out of wavefronts 0-7 because the loads of a wavefront return in
// order: a wait on a short load there would also wait for the touches.
#include <hip/hip_runtime.h>

#include "lpc_device.h"
#include "lpc_internal.h"

namespace lpc {

namespace {

constexpr int kResThreads = 1024;
constexpr int kRowThreads = 512;  // wavefronts 0-7: they prepare the coming rows; 8-15 fold and exchange
constexpr int kXcds = 8;
constexpr int kCusPerXcd = 32;
constexpr int kResBlocks = 2;     // Philox blocks (four coordinates each) per exchange thread, at most
constexpr int kResRows = 64;      // rows of one iteration per compute unit, at most
constexpr int kTouch = 6;         // words a thread of wavefronts 0-7 touches of the coming iteration's rows, at most
constexpr int kStatWords = 6;     // tagged words per (vector, slice): |u|max, non-finite count, sum and sum of squares
                                  // as two halves of a double each
// control block (32-bit words; every counter on a 128-byte line of its own)
constexpr int kCtlTicket = 0;       // [8][32]: arrival order of the workgroups of a die
constexpr int kCtlBar = 8 * 32;     // [8][32]: barrier counter of a die
constexpr int kCtlAbort = 16 * 32;  // [32]
constexpr int kCtlWords = kCtlAbort + 32;
// dynamic LDS: more than half of a compute unit's, so that no two of these workgroups share one
constexpr size_t kResLds = 84 * 1024;

typedef unsigned long long u64;

struct ResArgs {
  const float *X;
  int64_t ldx, d, d_pad, n, W;
  const float *y, *z_snap, *mu, *w_snap;
  float *w;                 // in: x_0 (Alg. 1) / the coupled x_1 (Alg. 2, 3); out: the last iterate
  float *yv, *zv, *ysum;    // Alg. 2, 3: y and z in and out, the weighted sum of y out
  int32_t N, B, m, bits, loss, alpc;
  QuantSpec qs;
  StreamKey key;            // of iteration 0
  float step, thr, shrink;  // Alg. 1
  float step_y, thr_y, shrink_y, alpha, thr_z, shrink_z, t1, t2, t3, theta;
  float scale;              // 1/B
  float *part;              // [8][S][32][d_pad] partial vectors (die, slot, compute unit)
  u64 *ubuf;                // [2][N][d_pad] u^i as published, tagged
  u64 *jbuf;                // [2][8][d_pad] the dies' partial sums of the shared batch's difference, tagged
  u64 *statbuf;             // [2][N][32][8] slice statistics, tagged
  u64 *wbuf;                // [8][d_pad] the iterate, one tagged copy per die
  uint32_t *ctl;
  uint32_t *packed;
  float *delta_out;
  double *stats_out;
  uint32_t *flags;
  int32_t S, cw, nslices;
  uint32_t spin_limit;
  uint32_t tag0;              // iteration t of this launch writes tag0 + t + 1
  unsigned long long *trace;  // [m][16] time stamps of die 0's first workgroup (100 MHz counter), or nullptr
};

__device__ __forceinline__ uint32_t xcc_id() {
  uint32_t v;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
  return v & 0xFu;
}
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// agent-scope accesses: they bypass the vector L1 (and are what crosses dies)
__device__ __forceinline__ uint32_t ld_agent(const uint32_t *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(uint32_t *p, uint32_t v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ u64 ld_agent(const u64 *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(u64 *p, u64 v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// a 64-bit store that stays in the die's L2: for words only this die reads
__device__ __forceinline__ void st_die(u64 *p, u64 v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ float2 ld_agent2(const float *p) {  // 8-byte aligned
  const u64 v = ld_agent(reinterpret_cast<const u64 *>(p));
  return make_float2(__builtin_bit_cast(float, (uint32_t)v), __builtin_bit_cast(float, (uint32_t)(v >> 32)));
}
// an atomic add that executes in the die's own L2 (no agent scope): counters shared by one die's workgroups only
__device__ __forceinline__ uint32_t die_add(uint32_t *p, uint32_t v) {
  return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
// tagged words
__device__ __forceinline__ u64 tagged(uint32_t bits, uint32_t tag) { return (u64)bits | ((u64)tag << 32); }
__device__ __forceinline__ u64 tagged(float v, uint32_t tag) { return tagged(__builtin_bit_cast(uint32_t, v), tag); }
__device__ __forceinline__ bool tag_is(u64 w, uint32_t tag) { return (uint32_t)(w >> 32) == tag; }
__device__ __forceinline__ float value_of(u64 w) { return __builtin_bit_cast(float, (uint32_t)w); }

// sums / maxima over the 32 adjacent lanes of a half wavefront (a fixed order); the whole wavefront takes part
__device__ __forceinline__ double half_sum(double v, int lane) {
  v = row16_sum(v);
  const double lo = read_lane(v, 0) + read_lane(v, 16), hi = read_lane(v, 32) + read_lane(v, 48);
  return lane < 32 ? lo : hi;
}
__device__ __forceinline__ float half_max(float v, int lane) {
  v = row16_max(v);
  const float lo = fmaxf(read_lane(v, 0), read_lane(v, 16)), hi = fmaxf(read_lane(v, 32), read_lane(v, 48));
  return lane < 32 ? lo : hi;
}

// One thread waits until *p (read at agent scope) has reached `target`; false after `limit` polls or once the
// abort word is set.
__device__ __forceinline__ bool wait_reach(const uint32_t *p, uint32_t target, const uint32_t *abort_word,
                                           uint32_t limit) {
  for (uint32_t k = 0; k < limit; ++k) {
    if ((int32_t)(ld_agent(p) - target) >= 0) return true;
    if ((k & 63u) == 63u && ld_agent(abort_word) != 0u) return false;
    __builtin_amdgcn_s_sleep(1);
  }
  return false;
}

// Rows of one die and of one of its compute units.  Die x hosts workers x, x+8, ... (slots 0, 1, ...), whose
// batches follow each other in the die's row list, then its share of the shared batch J (positions x, x+8, ...;
// slot S-1).  Compute unit c takes rows [c*R/32, (c+1)*R/32) of the list.
struct RowList {
  int32_t nws, B, nJ, R, k0, k1, S;
  uint32_t x;
  __device__ __forceinline__ static int32_t first_of(int32_t cu, int32_t R) { return (int32_t)(((int64_t)cu * R) / kCusPerXcd); }
  __device__ __forceinline__ void slot_pos(int32_t k, int32_t &slot, uint32_t &tag, uint32_t &worker, uint32_t &pos) const {
    const int32_t nw = nws * B;
    if (k < nw) {
      const int32_t s = k / B;
      slot = s; tag = kTagBatch; worker = x + 8u * (uint32_t)s; pos = (uint32_t)(k - s * B);
    } else {
      slot = S - 1; tag = kTagShared; worker = kSharedWorkerField; pos = x + 8u * (uint32_t)(k - nw);
    }
  }
};

// `v` is made opaque to the optimiser: what is derived from it inside the loop is formed there, not ahead of the
// loop and kept in registers (or spilled) across all of it.
__device__ __forceinline__ uint32_t opaque(uint32_t v) {
  asm volatile("" : "+v"(v));
  return v;
}

template <int KR, int RP>
__global__ __launch_bounds__(kResThreads) void resident_epoch_kernel(ResArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float *red = reinterpret_cast<float *>(smem);                                  // [2][16][8]
  QParams *qp = reinterpret_cast<QParams *>(smem + 1024);                        // [64]
  uint32_t *ctl_sh = reinterpret_cast<uint32_t *>(smem + 2048);                  // [4]: rank, alive, exchange counter
  long long *row_sh = reinterpret_cast<long long *>(smem + 2560);                // [64] this iteration's rows
  float2 *yz_sh = reinterpret_cast<float2 *>(smem + 2560 + 512);                 // [64] their labels and margins
  float *u_sh = reinterpret_cast<float *>(smem + 4096);                          // [slots][cw] <= 8 * 512 floats
  int16_t *codes = reinterpret_cast<int16_t *>(smem + 4096 + 16384);             // [N][cw] <= 4096 codes
  float2 *gsum = reinterpret_cast<float2 *>(smem + 4096 + 16384 + 8192);         // [G][items] <= 512 pairs

  const int tid0 = threadIdx.x;
  const int lane = tid0 & 63, wave = tid0 >> 6;
  const bool warm_role = tid0 < kRowThreads;
  const int e = tid0 - kRowThreads;  // index among the exchange threads (>= 0 for them)
  const uint32_t x = xcc_id();
  uint32_t *abort_word = a.ctl + kCtlAbort;
  if (tid0 == 0) {
    uint32_t rank = 0xFFFFu, ok = 0u;
    if (x < (uint32_t)kXcds) {
      rank = die_add(a.ctl + kCtlTicket + 32 * x, 1u);
      ok = rank < (uint32_t)kCusPerXcd ? 1u : 0u;
    }
    if (!ok) {  // a placement this kernel is not written for: nobody computes
      st_agent(abort_word, 1u);
      atomicOr(a.flags, 2u);
    }
    ctl_sh[0] = rank; ctl_sh[1] = ok; ctl_sh[2] = 0u;
  }
  __syncthreads();
  // (read back as scalars: everything derived from the rank is uniform over the workgroup)
  const uint32_t c = (uint32_t)__builtin_amdgcn_readfirstlane((int)ctl_sh[0]);
  bool alive = __builtin_amdgcn_readfirstlane((int)ctl_sh[1]) != 0;
  if (!alive) return;  // whole workgroup

  uint32_t *bar = a.ctl + kCtlBar + 32 * x;
  uint32_t bar_count = 0;  // barriers of the die this workgroup has arrived at (thread kRowThreads keeps it)

  RowList rl;
  rl.x = x; rl.S = a.S; rl.B = a.B;
  rl.nws = x < (uint32_t)a.N ? (a.N - (int32_t)x + 7) / 8 : 0;
  rl.nJ = (a.alpc && x < (uint32_t)a.B) ? (a.B - (int32_t)x + 7) / 8 : 0;
  rl.R = rl.nws * a.B + rl.nJ;
  rl.k0 = RowList::first_of((int32_t)c, rl.R);
  rl.k1 = RowList::first_of((int32_t)c + 1, rl.R);
  const int32_t total = rl.k1 - rl.k0;  // <= kResRows (the host checks)
  const uint32_t dpad = (uint32_t)a.d_pad, dlen = (uint32_t)a.d;

  // ---- this compute unit's slice of the coordinates
  const uint32_t col0 = c * (uint32_t)a.cw;
  const int32_t ncols = (int32_t)c < a.nslices ? (int32_t)((dpad - col0) < (uint32_t)a.cw ? (dpad - col0) : (uint32_t)a.cw) : 0;
  const int32_t npair = ncols / 2, nquad = ncols / 4;

  // ======== per-thread constants of the loop (index arithmetic done once) ========================================
  // rows phase: float offsets of this thread's chunks of a row / of the iterate
  uint32_t p1_off[KR];
#pragma unroll
  for (int k = 0; k < KR; ++k) p1_off[k] = (uint32_t)(k * kResThreads + tid0) * 4u;
  // fold: one (vector, column pair, group of compute units) unit per exchange thread
  const int32_t nfold = rl.nws + (a.alpc ? 1 : 0);  // vectors this die folds
  const int32_t items = nfold * npair;              // <= 512 (the host checks)
  const int32_t G = items > 256 ? 1 : (items > 128 ? 2 : (items > 64 ? 4 : 8));
  const bool gaps = rl.R < kCusPerXcd;              // fewer rows than compute units: some shares are empty
  bool fu_on = false;
  uint32_t fu_src = 0, fu_slot = 0;  // float offset of the unit's columns in compute unit 0's partial vector; LDS slot
  int32_t fu_lo = 0, fu_hi = -1;     // compute units of the group
  bool fc_on = false, fc_shared = false, fc_zero = false;
  uint32_t fc_dst = 0, fc_ush = 0;   // word offset in ubuf / jbuf (without the parity part); index in u_sh
  if (!warm_role && items > 0) {
    if (e < items * G) {
      const uint32_t g = G == 1 ? 0u : (uint32_t)e / (uint32_t)items, idx = (uint32_t)e - g * (uint32_t)items;
      const uint32_t si = idx / (uint32_t)npair, pr = idx - si * (uint32_t)npair;
      const bool shared = (int32_t)si >= rl.nws;
      const uint32_t slot = shared ? (uint32_t)a.S - 1u : si;
      // rows [ra, rb) of the die's list belong to this vector: the compute units clo .. chi hold them
      const uint32_t ra = shared ? (uint32_t)(rl.nws * a.B) : si * (uint32_t)a.B;
      const uint32_t rb = shared ? (uint32_t)rl.R : ra + (uint32_t)a.B;
      if (rb > ra) {
        const int32_t clo = (int32_t)((32u * (ra + 1u) - 1u) / (uint32_t)rl.R), chi = (int32_t)((32u * rb - 1u) / (uint32_t)rl.R);
        const int32_t len = (chi - clo + G) / G;
        fu_lo = clo + (int32_t)g * len;
        fu_hi = fu_lo + len - 1 < chi ? fu_lo + len - 1 : chi;
      }
      fu_on = true;
      fu_src = ((x * (uint32_t)a.S + slot) * kCusPerXcd) * dpad + col0 + 2u * pr;
      fu_slot = g * (uint32_t)items + idx;
    }
    if (e < items) {
      const uint32_t si = (uint32_t)e / (uint32_t)npair, pr = (uint32_t)e - si * (uint32_t)npair;
      const uint32_t col = col0 + 2u * pr;
      fc_on = true;
      fc_shared = (int32_t)si >= rl.nws;
      fc_zero = col >= dlen;
      fc_dst = (fc_shared ? x : x + 8u * si) * dpad + col;
      fc_ush = si * (uint32_t)a.cw + 2u * pr;
    }
  }
  // exchange: this thread's blocks of four coordinates (vector i, columns col0 + 4l ..)
  bool qb_on[kResBlocks];
  uint32_t qb_src[kResBlocks], qb_code[kResBlocks], qb_i[kResBlocks], qb_blk[kResBlocks];
#pragma unroll
  for (int q = 0; q < kResBlocks; ++q) {
    const int32_t b = e + kRowThreads * q;
    qb_on[q] = !warm_role && nquad > 0 && b < a.N * nquad;
    const uint32_t i = qb_on[q] ? (uint32_t)b / (uint32_t)nquad : 0u, l = qb_on[q] ? (uint32_t)b - i * (uint32_t)nquad : 0u;
    qb_i[q] = i;
    qb_src[q] = i * dpad + col0 + 4u * l;
    qb_code[q] = i * (uint32_t)a.cw + 4u * l;
    qb_blk[q] = (col0 + 4u * l) >> 2;
  }
  // per-coordinate state of the update, held by exchange thread e for column col0 + e
  float w_j = 0.f, mu_j = 0.f, z_j = 0.f, ysum_j = 0.f, snap_j = 0.f, y_j = 0.f;
  const bool mine = !warm_role && e < ncols;
  const bool own = mine && col0 + (uint32_t)e < dlen;
  if (own) {
    const int64_t j = col0 + e;
    w_j = a.w[j]; mu_j = a.mu[j];
    if (a.alpc) { z_j = a.zv[j]; snap_j = a.w_snap[j]; }
  }
  double weight = 1.0;
  // the vectors this die packs (Sec. 4.2's messages): i = x, x+8, ...; words of this slice per vector
  const int32_t bits = a.bits;
  const int32_t words_per_vec = (ncols / 32) * bits;

  // ---- wavefronts 0-7: the coming iteration's rows.  Called once the workgroup is past the die's barrier: nobody
  // reads row_sh / yz_sh any more in this iteration.  The wavefronts wait for their touches here, on their own:
  // wavefronts 8-15 meanwhile synchronise among themselves through an LDS counter, not the workgroup barrier.
  float warm_sink = 0.f;
  auto prepare_rows = [&](uint32_t iter) {
    StreamKey key = a.key;
    key.iter = a.key.iter + iter;
    const int32_t lines = (int32_t)((a.d + 31) / 32);
    long long row_l = 0;  // lane r: row r of this compute unit's share
    float y_l = 0.f, z_l = 0.f;
    if (lane < total) {
      int32_t slot; uint32_t tag, worker, pos;
      rl.slot_pos(rl.k0 + lane, slot, tag, worker, pos);
      row_l = sample_row(key, tag, worker, pos, a.n);
      y_l = a.y[row_l];
      z_l = a.z_snap[row_l];
    }
    float touch[kTouch];
#pragma unroll
    for (int k = 0; k < kTouch; ++k) {
      const int32_t idx = tid0 + kRowThreads * k;
      const int32_t q = idx / lines, l = idx - q * lines;
      const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)row_l, q & 63);
      const uint32_t hi = (uint32_t)__shfl((int)(uint32_t)((u64)row_l >> 32), q & 63);
      const int64_t row = (int64_t)(((u64)hi << 32) | lo);
      touch[k] = q < total ? a.X[row * a.ldx + (int64_t)l * 32] : 0.f;
    }
    if (wave == 0) {
      row_sh[lane] = row_l;
      yz_sh[lane] = make_float2(y_l, z_l);
    }
#pragma unroll
    for (int k = 0; k < kTouch; ++k) warm_sink += touch[k];
  };
  if (warm_role) prepare_rows(0u);
  uint32_t xgen = 0;
  // barrier among wavefronts 8-15 (all of their lanes call it): LDS writes before it are visible after it
  auto exchange_barrier = [&]() {
    ++xgen;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if (lane == 0) {
      __hip_atomic_fetch_add(&ctl_sh[2], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      bool ok = false;
      for (uint32_t k = 0; k < (1u << 22); ++k) {
        if ((int32_t)(__hip_atomic_load(&ctl_sh[2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) - 8u * xgen) >= 0) { ok = true; break; }
      }
      if (!ok) ctl_sh[1] = 0u;
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
  };

  const bool tracer = a.trace != nullptr && x == 0u && c == 0u && tid0 == kRowThreads;
#define RES_STAMP(k) do { if (tracer) a.trace[(int64_t)t * 16 + (k)] = wall_clock64(); } while (0)
  int buf = 0;
  for (int32_t t = 0; t < a.m; ++t) {
    const uint32_t par = (uint32_t)t & 1u;
    const uint32_t tag_t = a.tag0 + (uint32_t)t + 1u;  // what this iteration writes
    __syncthreads();  // row_sh, yz_sh of this iteration; everybody is done with the last one
    alive = __builtin_amdgcn_readfirstlane((int)ctl_sh[1]) != 0;
    if (!alive) break;
    RES_STAMP(0);
    // ================= rows: margins, slope differences, partial vectors ====================================
    float4 wreg[KR], acc[KR];
    uint32_t off1[KR];
#pragma unroll
    for (int k = 0; k < KR; ++k) off1[k] = opaque(p1_off[k]);
    if (t == 0) {
#pragma unroll
      for (int k = 0; k < KR; ++k)
        wreg[k] = off1[k] < dlen ? *reinterpret_cast<const float4 *>(a.w + off1[k]) : make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
      // the iterate the die's compute units stored at the end of the last iteration: tagged words, read until whole
      const u64 *wsrc = a.wbuf + (int64_t)x * a.d_pad;
      const uint32_t want = tag_t - 1u;
      bool whole = false;
      for (uint32_t spin = 0; spin < a.spin_limit; ++spin) {
        bool ok = true;
#pragma unroll
        for (int k = 0; k < KR; ++k) {
          // (a thread whose chunk lies past d reads the last chunk instead: every load is issued, none branches)
          const bool in = off1[k] < dlen;
          const u64 *src = wsrc + (in ? off1[k] : dlen - 4u);
          u64 q[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) q[v] = ld_agent(src + v);
#pragma unroll
          for (int v = 0; v < 4; ++v) ok = ok && tag_is(q[v], want);
          wreg[k] = in ? make_float4(value_of(q[0]), value_of(q[1]), value_of(q[2]), value_of(q[3]))
                       : make_float4(0.f, 0.f, 0.f, 0.f);
        }
        if (__ballot(!ok) == 0ull) { whole = true; break; }
        if ((spin & 63u) == 63u && ld_agent(abort_word) != 0u) break;
      }
      if (!whole && lane == 0) ctl_sh[1] = 0u;
    }
#pragma unroll
    for (int k = 0; k < KR; ++k) acc[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    int32_t cur_slot = -1;
    for (int32_t q0 = 0; q0 < total; q0 += RP) {
      float4 xr[RP][KR];
#pragma unroll
      for (int r = 0; r < RP; ++r) {
        const bool live = q0 + r < total;
        const long long rw = row_sh[live ? q0 + r : 0];
        const int64_t row = (int64_t)(((u64)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)((u64)rw >> 32)) << 32) |
                                      (u64)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(u64)rw));
        const float *src = a.X + row * a.ldx;
#pragma unroll
        for (int k = 0; k < KR; ++k)
          xr[r][k] = (live && off1[k] < dlen) ? *reinterpret_cast<const float4 *>(src + off1[k]) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int r = 0; r < RP; ++r) {
        if (q0 + r >= total) break;  // uniform
        float v = 0.f;
#pragma unroll
        for (int k = 0; k < KR; ++k) {
          v = fmaf(xr[r][k].x, wreg[k].x, v); v = fmaf(xr[r][k].y, wreg[k].y, v);
          v = fmaf(xr[r][k].z, wreg[k].z, v); v = fmaf(xr[r][k].w, wreg[k].w, v);
        }
        v = wave_sum(v);
        if (lane == 0) red[(buf * 16 + wave) * 8 + r] = v;
      }
      __syncthreads();
#pragma unroll
      for (int r = 0; r < RP; ++r) {
        if (q0 + r >= total) break;  // uniform
        // the sixteen wavefronts' shares of the margin, added in wavefront order inside a row of 16 lanes
        float z = red[(buf * 16 + (lane & 15)) * 8 + r];
        z = read_lane(row16_sum(z), 0);
        const float2 yz = yz_sh[q0 + r];
        // x_0 is the snapshot itself in Alg. 1: every difference is exactly zero there
        const float coef = (!a.alpc && t == 0) ? 0.f : loss_slope(a.loss, z, yz.x) - loss_slope(a.loss, yz.y, yz.x);
        int32_t slot; uint32_t tag, worker, pos;
        rl.slot_pos(rl.k0 + q0 + r, slot, tag, worker, pos);
        if (slot != cur_slot) {
          if (cur_slot >= 0) {
            float *dst = a.part + (((int64_t)x * a.S + cur_slot) * kCusPerXcd + c) * a.d_pad;
#pragma unroll
            for (int k = 0; k < KR; ++k)
              if (off1[k] < dlen) *reinterpret_cast<float4 *>(dst + off1[k]) = acc[k];
          }
#pragma unroll
          for (int k = 0; k < KR; ++k) acc[k] = make_float4(0.f, 0.f, 0.f, 0.f);
          cur_slot = slot;
        }
#pragma unroll
        for (int k = 0; k < KR; ++k) {
          acc[k].x = fmaf(coef, xr[r][k].x, acc[k].x); acc[k].y = fmaf(coef, xr[r][k].y, acc[k].y);
          acc[k].z = fmaf(coef, xr[r][k].z, acc[k].z); acc[k].w = fmaf(coef, xr[r][k].w, acc[k].w);
        }
      }
      buf ^= 1;
    }
    if (cur_slot >= 0) {
      float *dst = a.part + (((int64_t)x * a.S + cur_slot) * kCusPerXcd + c) * a.d_pad;
#pragma unroll
      for (int k = 0; k < KR; ++k)
        if (off1[k] < dlen) *reinterpret_cast<float4 *>(dst + off1[k]) = acc[k];
    }
    RES_STAMP(1);
    // the quantizer's random words do not depend on the data: wavefronts 8-15 draw them while the partial vectors'
    // stores are on their way
    uint32_t rnd[kResBlocks][4];
    if (!warm_role) {
      StreamKey key = a.key;
      key.iter = a.key.iter + (uint32_t)t;
#pragma unroll
      for (int q = 0; q < kResBlocks; ++q) {
        const Philox4 blk = stream_block(key, kTagQuant, opaque(qb_i[q]), opaque(qb_blk[q]));
        rnd[q][0] = blk.x; rnd[q][1] = blk.y; rnd[q][2] = blk.z; rnd[q][3] = blk.w;
      }
    }
    wait_stores();  // the partial vectors are in the die's L2
    __syncthreads();
    RES_STAMP(2);
    // ================= barrier of the die, then the fold of this compute unit's slice =======================
    if (tid0 == kRowThreads) {
      bool ok = ctl_sh[1] != 0u;
      die_add(bar, 1u);
      ++bar_count;
      ok = wait_reach(bar, (uint32_t)kCusPerXcd * bar_count, abort_word, a.spin_limit) && ok;
      ctl_sh[1] = ok ? 1u : 0u;
    }
    __syncthreads();
    RES_STAMP(3);
    alive = __builtin_amdgcn_readfirstlane((int)ctl_sh[1]) != 0;
    if (!alive) break;
    if (warm_role) {
      if (t + 1 < a.m) prepare_rows((uint32_t)(t + 1));
      weight *= (double)a.theta;
      continue;  // wavefronts 8-15 carry the iteration on; everybody meets again at the top of the next one
    }
    RES_STAMP(12);
    if (fu_on) {
      // the partial vectors of the group's compute units, all requested together (one past the range repeats the
      // last and is dropped), added in compute-unit order
      const float *src = a.part + opaque(fu_src);
      const int32_t lo = (int32_t)opaque((uint32_t)fu_lo), hi = (int32_t)opaque((uint32_t)fu_hi);
      float2 v = make_float2(0.f, 0.f);
      if (G == 8) {  // at most four compute units per group
        float2 p[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const int32_t cu = lo + k <= hi ? lo + k : (hi > 0 ? hi : 0);  // (an empty range reads compute unit 0's)
          p[k] = ld_agent2(src + (uint32_t)cu * dpad);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          bool has = lo + k <= hi;
          if (gaps) has = has && RowList::first_of(lo + k + 1, rl.R) > RowList::first_of(lo + k, rl.R);
          v.x += has ? p[k].x : 0.f;
          v.y += has ? p[k].y : 0.f;
        }
      } else {
        for (int32_t c0 = lo; c0 <= hi; c0 += 16) {
          float2 p[16];
#pragma unroll
          for (int k = 0; k < 16; ++k) {
            const int32_t cu = c0 + k <= hi ? c0 + k : hi;
            p[k] = ld_agent2(src + (uint32_t)cu * dpad);
          }
#pragma unroll
          for (int k = 0; k < 16; ++k) {
            bool has = c0 + k <= hi;
            if (gaps) has = has && RowList::first_of(c0 + k + 1, rl.R) > RowList::first_of(c0 + k, rl.R);
            v.x += has ? p[k].x : 0.f;
            v.y += has ? p[k].y : 0.f;
          }
        }
      }
      gsum[opaque(fu_slot)] = v;
    }
    RES_STAMP(15);
    exchange_barrier();  // gsum
    if (fc_on) {
      const uint32_t idx = opaque((uint32_t)e);
      float2 v = gsum[idx];
      for (int32_t g = 1; g < G; ++g) {  // the groups' sums in group order: fixed whatever the timing
        const float2 q = gsum[(uint32_t)g * (uint32_t)items + idx];
        v.x += q.x; v.y += q.y;
      }
      if (fc_zero) v = make_float2(0.f, 0.f);
      const uint32_t dsto = opaque(fc_dst);
      if (fc_shared) {
        u64 *dst = a.jbuf + (int64_t)par * kXcds * a.d_pad + dsto;
        st_agent(dst, tagged(v.x, tag_t)); st_agent(dst + 1, tagged(v.y, tag_t));
      } else {
        v.x *= a.scale; v.y *= a.scale;
        u64 *dst = a.ubuf + (int64_t)par * a.N * a.d_pad + dsto;
        st_agent(dst, tagged(v.x, tag_t)); st_agent(dst + 1, tagged(v.y, tag_t));
        *reinterpret_cast<float2 *>(u_sh + opaque(fc_ush)) = v;
      }
    }
    RES_STAMP(10);
    exchange_barrier();  // u_sh
    RES_STAMP(4);
    // statistics of the slice of every worker vector of this die: wavefront w takes vectors w, w+8, ...
    for (int32_t si = wave - 8; si < rl.nws; si += 8) {
      float fmx = 0.f;
      double sum = 0.0, sumsq = 0.0, bad = 0.0;
      for (int32_t k = lane; k < ncols; k += 64) {
        const float v = u_sh[si * a.cw + k];
        if (isfinite(v)) {
          fmx = fmaxf(fmx, fabsf(v)); sum += (double)v; sumsq += (double)v * (double)v;
        } else {
          bad += 1.0;
        }
      }
      fmx = wave_max(fmx); sum = wave_sum(sum); sumsq = wave_sum(sumsq); bad = wave_sum(bad);
      if (lane < kStatWords && ncols > 0) {
        const u64 sb = __builtin_bit_cast(u64, sum), qb = __builtin_bit_cast(u64, sumsq);
        const uint32_t word = lane == 0 ? __builtin_bit_cast(uint32_t, fmx)
                              : lane == 1 ? __builtin_bit_cast(uint32_t, (float)bad)
                              : lane == 2 ? (uint32_t)sb : lane == 3 ? (uint32_t)(sb >> 32)
                              : lane == 4 ? (uint32_t)qb : (uint32_t)(qb >> 32);
        st_agent(a.statbuf + (((int64_t)par * a.N + ((int32_t)x + 8 * si)) * kCusPerXcd + c) * 8 + lane,
                 tagged(word, tag_t));
      }
    }
    RES_STAMP(5);
    // ================= exchange: slice c of every vector, from whichever die owns it =======================
    float4 uq[kResBlocks];
    float uhat = 0.f;
    if (ncols > 0) {
      const int l32 = lane & 31;
      const bool sums = a.qs.clip_mode != LPC_CLIP_LAMBDA;  // the c*sigma rule needs the sums as well
      const u64 *ub = a.ubuf + (int64_t)par * a.N * a.d_pad;
      const u64 *jb = a.jbuf + (int64_t)par * kXcds * a.d_pad + col0 + (mine ? (uint32_t)e : 0u);
      const u64 *sb = a.statbuf + (int64_t)par * a.N * kCusPerXcd * 8;
      uint32_t src_q[kResBlocks];
#pragma unroll
      for (int q = 0; q < kResBlocks; ++q) src_q[q] = opaque(qb_src[q]);
      for (int32_t i0 = 2 * (wave - 8); i0 < a.N || i0 == 2 * (wave - 8); i0 += 16) {
        // vectors i0 (lanes 0-31) and i0+1 (lanes 32-63): slice k's statistics on lane k; in the first round also
        // this thread's blocks of the workers' vectors and its column of the shared batch's difference
        const bool first = i0 == 2 * (wave - 8);
        const int32_t i = i0 + (lane >> 5);
        const bool st_on = i < a.N && l32 < a.nslices;
        const u64 *src = sb + ((int64_t)(st_on ? i : 0) * kCusPerXcd + (st_on ? l32 : 0)) * 8;
        u64 w[kStatWords] = {0, 0, 0, 0, 0, 0};
        bool got = false;
        for (uint32_t spin = 0; spin < a.spin_limit; ++spin) {
          bool ok = true;
          if (first) {
#pragma unroll
            for (int q = 0; q < kResBlocks; ++q) {
              if (q * kRowThreads >= a.N * nquad) break;  // uniform: no thread has such a block
              u64 qv[4];
#pragma unroll
              for (int v = 0; v < 4; ++v) qv[v] = ld_agent(ub + src_q[q] + v);
#pragma unroll
              for (int v = 0; v < 4; ++v) ok = ok && (tag_is(qv[v], tag_t) || !qb_on[q]);
              uq[q] = make_float4(value_of(qv[0]), value_of(qv[1]), value_of(qv[2]), value_of(qv[3]));
            }
            if (a.alpc) {  // the shared batch's difference for this thread's column (die order, then 1/B)
              u64 pj[kXcds];
#pragma unroll
              for (int k = 0; k < kXcds; ++k) pj[k] = ld_agent(jb + (uint32_t)k * dpad);
              float sj = value_of(pj[0]);
#pragma unroll
              for (int k = 1; k < kXcds; ++k) sj += value_of(pj[k]);
#pragma unroll
              for (int k = 0; k < kXcds; ++k) ok = ok && (tag_is(pj[k], tag_t) || !mine);
              uhat = sj * a.scale;
            }
          }
          w[0] = ld_agent(src); w[1] = ld_agent(src + 1);
          ok = ok && ((tag_is(w[0], tag_t) && tag_is(w[1], tag_t)) || !st_on);
          if (sums) {
#pragma unroll
            for (int v = 2; v < kStatWords; ++v) w[v] = ld_agent(src + v);
#pragma unroll
            for (int v = 2; v < kStatWords; ++v) ok = ok && (tag_is(w[v], tag_t) || !st_on);
          }
          if (__ballot(!ok) == 0ull) { got = true; break; }
          if ((spin & 63u) == 63u && ld_agent(abort_word) != 0u) break;
        }
        if (!got && lane == 0) ctl_sh[1] = 0u;
        // eq. (3): a half wavefront folds the slice statistics of one vector
        float am = st_on ? value_of(w[0]) : 0.f;
        double bd = st_on ? (double)value_of(w[1]) : 0.0, s = 0.0, s2 = 0.0;
        am = half_max(am, lane); bd = half_sum(bd, lane);
        if (sums) {
          s = st_on ? __builtin_bit_cast(double, (u64)(uint32_t)w[2] | ((u64)(uint32_t)w[3] << 32)) : 0.0;
          s2 = st_on ? __builtin_bit_cast(double, (u64)(uint32_t)w[4] | ((u64)(uint32_t)w[5] << 32)) : 0.0;
          s = half_sum(s, lane); s2 = half_sum(s2, lane);
        }
        if (l32 == 0 && i < a.N) {
          const QParams q_i = make_qparams(a.qs, (double)am, s, s2, a.d);
          qp[i] = q_i;
          if (x == 0u && c == 0u) {
            a.delta_out[i] = q_i.delta;
            double *o = a.stats_out + (int64_t)i * 4;
            o[0] = (double)am; o[1] = s; o[2] = s2; o[3] = bd;
            if (bd > 0.0) atomicOr(a.flags, 1u);
          }
        }
      }
    }
    RES_STAMP(11);
    exchange_barrier();  // qp
    RES_STAMP(6);
    if (ncols > 0) {
      // Sec. 3.2 rules (1), (2) in fp32, one IEEE operation per step
      const float hi = (float)((1 << (a.bits - 1)) - 1);
      const float lo = -(float)(1 << (a.bits - 1));
#pragma unroll
      for (int q = 0; q < kResBlocks; ++q) {
        if (!qb_on[q]) continue;
        const QParams qi = qp[opaque(qb_i[q])];
        const float vals[4] = {uq[q].x, uq[q].y, uq[q].z, uq[q].w};
        int16_t cd[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          float s = vals[k] * qi.rdelta;
          s = fminf(fmaxf(s, lo), hi);
          const float base = floorf(s);
          const float frac = s - base;
          const float unif = (float)(rnd[q][k] >> 8) * 0x1.0p-24f;
          cd[k] = (int16_t)(qi.delta > 0.0f ? (int32_t)base + ((unif < frac) ? 1 : 0) : 0);
        }
        *reinterpret_cast<uint2 *>(codes + opaque(qb_code[q])) =
            make_uint2((uint32_t)(uint16_t)cd[0] | ((uint32_t)(uint16_t)cd[1] << 16),
                       (uint32_t)(uint16_t)cd[2] | ((uint32_t)(uint16_t)cd[3] << 16));
      }
    }
    exchange_barrier();  // codes
    RES_STAMP(7);
    if (mine) {
      float next = 0.f;
      if (own) {
        // eq. (4) in worker order
        const int16_t *cj = codes + opaque((uint32_t)e);
        float sum = 0.f;
        for (int32_t i = 0; i < a.N; ++i) sum = __builtin_fmaf(qp[i].delta, (float)cj[i * a.cw], sum);
        const float avg = sum * (1.0f / (float)a.N);
        if (!a.alpc) {
          w_j = prox_scalar(w_j, avg + mu_j, a.step, a.thr, a.shrink);  // Alg. 1 steps 9-10
          next = w_j;
        } else {
          // Alg. 2 steps 13-15 and the next step 6
          y_j = prox_scalar(w_j, avg + mu_j, a.step_y, a.thr_y, a.shrink_y);   // low-precision gradient
          z_j = prox_scalar(z_j, uhat + mu_j, a.alpha, a.thr_z, a.shrink_z);   // full precision
          const float wt = (float)weight;
          ysum_j = t == 0 ? wt * y_j : ysum_j + wt * y_j;
          w_j = (a.t1 * z_j + a.t2 * snap_j) + a.t3 * y_j;
          next = w_j;
        }
      }
      st_die(a.wbuf + (int64_t)x * a.d_pad + col0 + opaque((uint32_t)e), tagged(next, tag_t));
    }
    RES_STAMP(8);
    // the packed messages (Sec. 4.2) of the vectors this die hosts, off the path of the next margins
    for (int32_t idx = e; idx < rl.nws * words_per_vec; idx += kRowThreads) {
      const int32_t si = idx / words_per_vec, rem = idx - si * words_per_vec;
      const int32_t sgm = rem / bits, wd = rem - sgm * bits;
      const int32_t i = (int32_t)x + 8 * si;
      const uint32_t mask = (1u << bits) - 1u;
      const int32_t bit0 = 32 * wd;
      uint32_t word = 0u;
      for (int32_t k = bit0 / bits; k < 32 && k * bits < bit0 + 32; ++k) {
        const uint32_t field = (uint32_t)(int32_t)codes[i * a.cw + 32 * sgm + k] & mask;
        const int32_t sh = k * bits - bit0;
        word |= sh >= 0 ? (field << sh) : (field >> (-sh));
      }
      a.packed[(int64_t)i * a.W + ((int64_t)(col0 / 32) + sgm) * bits + wd] = word;
    }
    weight *= (double)a.theta;
    RES_STAMP(9);
  }
  if (tracer) {  // how long 4096 dependent vector instructions take at the clock the chip runs this launch at
    float v = (float)tid0;
    const unsigned long long c0 = wall_clock64();
    for (int k = 0; k < 1024; ++k) {
      asm volatile("v_fma_f32 %0, %0, %0, %0\n v_fma_f32 %0, %0, %0, %0\n v_fma_f32 %0, %0, %0, %0\n v_fma_f32 %0, %0, %0, %0" : "+v"(v));
    }
    const unsigned long long c1 = wall_clock64();
    a.trace[13] = c1 - c0;
    if (v == 1.2345f) a.trace[14] = 1;
  }
#undef RES_STAMP
  __syncthreads();
  alive = alive && __builtin_amdgcn_readfirstlane((int)ctl_sh[1]) != 0;
  if (!alive) {
    if (tid0 == 0) {
      st_agent(abort_word, 1u);
      atomicOr(a.flags, 2u);
    }
    return;
  }
  if (warm_sink == -1.2345678e-38f) a.part[0] = warm_sink;
  // die 0 stores the results
  if (x == 0u && own) {
    const int64_t j = col0 + e;
    a.w[j] = w_j;
    if (a.alpc) { a.yv[j] = y_j; a.zv[j] = z_j; a.ysum[j] = ysum_j; }
  }
}

}  // namespace

// ---- host side ----------------------------------------------------------------------------------------------

namespace {
int32_t res_cw(const lpc_ctx *c) {  // columns per slice: whole 32-coordinate segments, 32 slices at most
  const int64_t segs = c->d_pad / 32;
  return (int32_t)(32 * ((segs + kCusPerXcd - 1) / kCusPerXcd));
}
int32_t res_slots(const lpc_ctx *c) { return (c->cfg.N + kXcds - 1) / kXcds + 1; }
}  // namespace

bool resident_supported(const lpc_ctx *c) {
  if (!c->grad_ok || c->csr || c->mlp || !c->quant || c->cfg.scheme != LPC_SCHEME_A) return false;
  if (c->n_full != c->n) return false;  // the snapshot margins of every row are cached
  if (c->cfg.N > 64 || c->d_pad > 16384) return false;
  if (c->d % 4 != 0 || c->prob.ldx % 4 != 0 || (((uintptr_t)c->prob.X) & 15u) != 0) return false;
  const int32_t cw = res_cw(c);
  if ((int64_t)c->cfg.N * cw > (int64_t)kResBlocks * 4 * kRowThreads) return false;
  // rows of one iteration per die (its workers' batches and its share of a shared batch), 64 per compute unit
  const int64_t die_rows = (int64_t)((c->cfg.N + kXcds - 1) / kXcds) * c->cfg.B + (c->cfg.B + kXcds - 1) / kXcds;
  if (die_rows > (int64_t)kResRows * kCusPerXcd) return false;
  // one (vector, column pair) item of the fold per exchange thread
  if ((int64_t)((c->cfg.N + kXcds - 1) / kXcds + 1) * (cw / 2) > kRowThreads) return false;
  if (c->cus != kXcds * kCusPerXcd) return false;
  return true;
}

size_t resident_part_floats(const lpc_ctx *c) { return (size_t)kXcds * res_slots(c) * kCusPerXcd * c->d_pad; }
size_t resident_ubuf_floats(const lpc_ctx *c) { return (size_t)2 * 2 * c->cfg.N * c->d_pad; }   // tagged words
size_t resident_jbuf_floats(const lpc_ctx *c) { return (size_t)2 * 2 * kXcds * c->d_pad; }
size_t resident_stat_doubles(const lpc_ctx *c) { return (size_t)2 * c->cfg.N * kCusPerXcd * 8; }
size_t resident_wbuf_floats(const lpc_ctx *c) { return (size_t)2 * kXcds * c->d_pad; }
size_t resident_ctl_words() { return (size_t)kCtlWords; }

hipError_t launch_resident_epoch(const lpc_ctx *c, const ResidentStep &rs, hipStream_t st) {
  ResArgs a{};
  a.X = c->prob.X; a.ldx = c->prob.ldx; a.d = c->d; a.d_pad = c->d_pad; a.n = c->n; a.W = c->W;
  a.y = c->prob.y; a.z_snap = rs.z_snap; a.mu = rs.mu; a.w_snap = rs.w_snap;
  a.w = rs.w; a.yv = rs.y; a.zv = rs.z; a.ysum = rs.ysum;
  a.N = c->cfg.N; a.B = c->cfg.B; a.m = c->cfg.m; a.bits = c->cfg.bits; a.loss = c->prob.loss; a.alpc = rs.alpc ? 1 : 0;
  a.qs.bits = c->cfg.bits; a.qs.clip_mode = c->cfg.clip_mode; a.qs.clip = c->cfg.clip; a.qs.enabled = 1;
  a.key = rs.key;
  const double l1 = (double)c->prob.lambda1, l2 = (double)c->prob.lambda2;
  auto consts = [&](float step, float *thr, float *shrink) {
    *thr = (float)((double)step * l1);
    *shrink = (float)(1.0 / (1.0 + (double)step * l2));
  };
  a.step = rs.step; consts(rs.step, &a.thr, &a.shrink);
  a.step_y = rs.step_y; consts(rs.step_y, &a.thr_y, &a.shrink_y);
  a.alpha = rs.alpha; consts(rs.alpha, &a.thr_z, &a.shrink_z);
  a.t1 = rs.tau1; a.t2 = rs.tau2; a.t3 = (float)(1.0 - (double)rs.tau1 - (double)rs.tau2); a.theta = rs.theta;
  a.scale = (float)(1.0 / (double)c->cfg.B);
  a.part = c->s.res_part; a.ubuf = reinterpret_cast<u64 *>(c->s.res_ubuf); a.jbuf = reinterpret_cast<u64 *>(c->s.res_jbuf);
  a.statbuf = reinterpret_cast<u64 *>(c->s.res_stat); a.wbuf = reinterpret_cast<u64 *>(c->s.res_wbuf); a.ctl = c->s.res_ctl;
  a.tag0 = rs.tag0;
  a.packed = c->s.packed; a.delta_out = c->s.delta; a.stats_out = c->s.stats; a.flags = c->s.flags;
  a.S = res_slots(c); a.cw = res_cw(c); a.nslices = (int32_t)((c->d_pad + a.cw - 1) / a.cw);
  a.spin_limit = c->spin_limit;
  a.trace = c->res_trace_on ? c->s.res_trace : nullptr;
  // counters and flags of the launch start at zero (a fill kernel: the caller may be capturing the stream)
  hipError_t err = launch_fill_u32(c->s.res_ctl, 0u, (int64_t)kCtlWords, st);
  if (err != hipSuccess) return err;
  const int64_t chunks = (c->d + 4 * kResThreads - 1) / (4 * kResThreads);  // float4 chunks of a row per thread
  const void *fn = nullptr;
  if (chunks <= 1) fn = reinterpret_cast<const void *>(&resident_epoch_kernel<1, 4>);
  else if (chunks <= 2) fn = reinterpret_cast<const void *>(&resident_epoch_kernel<2, 5>);
  else fn = reinterpret_cast<const void *>(&resident_epoch_kernel<4, 3>);
  static thread_local const void *prepared[4] = {nullptr, nullptr, nullptr, nullptr};
  bool known = false;
  for (const void *p : prepared) known = known || p == fn;
  if (!known) {
    err = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kResLds);
    if (err != hipSuccess) return err;
    for (const void *&p : prepared)
      if (!p) { p = fn; break; }
  }
  void *args[] = {&a};
  return hipLaunchCooperativeKernel(fn, dim3(kXcds * kCusPerXcd), dim3(kResThreads), args, kResLds, st);
}

}  // namespace lpc
