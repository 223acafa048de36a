// The inner loop of an epoch (Alg. 1 steps 5-11; Alg. 2 steps 5-15) as ONE resident launch for dense data of
// moderate width (d_pad <= 16384, N <= 64): 256 workgroups of 1024 threads, one per compute unit, stay on the chip
// for all m inner iterations and hand each other what the paper's workers send over the wire.
//
// The chip is used the way the method is distributed.  An MI355X is eight dies (XCDs) of 32 compute units, each
// die with its own L2; workgroup k of a launch runs on die k mod 8, and a workgroup reads its die's number from the
// XCC_ID hardware register.  Worker i lives on die i mod 8:
//
//   rows      each compute unit of a die takes a share of the rows that the die's workers sample (Alg. 1 step 6:
//             margin, slope difference against the cached snapshot margin, slope * row) and leaves one partial
//             vector per worker in the die's L2;
//   fold      after a barrier among the die's 32 workgroups, compute unit c adds the 32 partial vectors over
//             its own slice of the coordinates (a fixed order), takes the slice's statistics, and publishes the
//             slice of u^i and the statistics for every die to read;
//   exchange  compute unit c of EVERY die waits for the eight publishers of slice c (one flag each, no chip-wide
//             barrier), folds the statistics of all slices into delta_i (eq. (3)), quantizes the slice of every
//             worker's vector (Sec. 3.2 rules (1), (2); the random stream is a function of (worker, coordinate,
//             iteration), so all dies get the same codes), averages the codes (eq. (4)) and takes the proximal step
//             (Alg. 1 steps 9-10, or Alg. 2 steps 13-15 with the next step 6) for its slice.  Die 0 also stores the
//             packed messages.  Every die thus holds the new iterate, one slice per compute unit;
//   iterate   a second barrier inside the die, after which every compute unit reads the whole iterate from its
//             die's L2 for the next margins.
//
// Two barriers among 32 workgroups and one set of eight flags per iteration replace three kernel launches.
// The shared batch J of Alg. 2 is spread over the dies (position p on die p mod 8); each die publishes its partial
// sum and the exchange step adds the eight.
//
// Memory rules.  Data that crosses workgroups INSIDE a die is written with ordinary stores (the vector L1 writes
// through to the die's L2; a wave waits for its stores to be acknowledged before its workgroup arrives at the
// barrier) and read with agent-scope atomic loads, which bypass the reader's L1.  Data that crosses dies is
// written and read with agent-scope atomic stores and loads.  Barrier counters are bumped with atomics that execute
// in the die's L2; flags are agent-scope words holding the iteration number.  Every wait is bounded: after
// spin_limit polls a workgroup raises the abort word and flag bit 1, leaves the loop, and every other workgroup
// follows at its next wait, so all waves exit whatever happens; the host then reports LPC_EDEVICE.  The launch is
// cooperative, so all 256 workgroups are resident together.
//
// Inside a workgroup the first eight wavefronts own the rows (512 threads, each a fixed set of columns) and the
// last eight do fold and exchange.  The row wavefronts request the rows of iteration t+1 as soon as iteration t's
// are consumed (which rows are sampled does not depend on the iterate), so that they travel from HBM while the
// other eight wavefronts synchronise; the split keeps those long-latency loads out of the wavefronts whose waits on
// short loads would otherwise have to wait for them too (loads return in order within a wavefront).
#include <hip/hip_runtime.h>

#include "lpc_device.h"
#include "lpc_internal.h"

namespace lpc {

namespace {

constexpr int kResThreads = 1024;
constexpr int kRowThreads = 512;
constexpr int kXcds = 8;
constexpr int kCusPerXcd = 32;
constexpr int kResBlocks = 2;
constexpr int kTouch = 6;     // words a thread of wavefronts 0-7 touches of the coming iteration's rows, at most  // Philox blocks (four coordinates each) per exchange thread, at most
// control block (32-bit words; every counter on a 128-byte line of its own)
constexpr int kCtlTicket = 0;                 // [8][32]: arrival order of the workgroups of a die
constexpr int kCtlBar = 8 * 32;               // [8][32]: barrier counter of a die
constexpr int kCtlFlag = 16 * 32;             // [32][32]: slice c: words 0..7 = iterations published by die 0..7
constexpr int kCtlAbort = 16 * 32 + 32 * 32;  // [32]
constexpr int kCtlWords = kCtlAbort + 32;
// dynamic LDS: more than half of a compute unit's, so that no two of these workgroups share one
constexpr size_t kResLds = 84 * 1024;

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
  float *ubuf;              // [2][N][d_pad] u^i as published
  float *jbuf;              // [2][8][d_pad] the dies' partial sums of the shared batch's difference
  double *statbuf;          // [2][N][32][4] slice statistics
  float *wbuf;              // [8][d_pad] the iterate, one copy per die
  uint32_t *ctl;
  uint32_t *packed;
  float *delta_out;
  double *stats_out;
  uint32_t *flags;
  int32_t S, cw, nslices;
  uint32_t spin_limit;
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
__device__ __forceinline__ float ld_agent(const float *p) {
  return __builtin_bit_cast(float, ld_agent(reinterpret_cast<const uint32_t *>(p)));
}
__device__ __forceinline__ double ld_agent(const double *p) {
  return __builtin_bit_cast(double, __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED,
                                                      __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void st_agent(double *p, double v) {
  __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), __builtin_bit_cast(unsigned long long, v),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_agent2(const float *p) {  // 8-byte aligned
  const unsigned long long v =
      __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__builtin_bit_cast(float, (uint32_t)v), __builtin_bit_cast(float, (uint32_t)(v >> 32)));
}
__device__ __forceinline__ void st_agent2(float *p, float a, float b) {
  const unsigned long long v =
      (unsigned long long)__builtin_bit_cast(uint32_t, a) | ((unsigned long long)__builtin_bit_cast(uint32_t, b) << 32);
  __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float4 ld_agent4(const float *p) {  // 16-byte aligned; two 8-byte loads
  const float2 lo = ld_agent2(p), hi = ld_agent2(p + 2);
  return make_float4(lo.x, lo.y, hi.x, hi.y);
}
// an atomic add that executes in the die's own L2 (no agent scope): counters shared by one die's workgroups only
__device__ __forceinline__ uint32_t die_add(uint32_t *p, uint32_t v) {
  return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// sums / maxima over the 32 adjacent lanes of a half wavefront (a fixed order); the whole wavefront takes part
__device__ __forceinline__ double half_sum(double v, int lane) {
  v = row16_sum(v);
  const double lo = read_lane(v, 0) + read_lane(v, 16), hi = read_lane(v, 32) + read_lane(v, 48);
  return lane < 32 ? lo : hi;
}
__device__ __forceinline__ double half_max(double v, int lane) {
  v = row16_max(v);
  const double lo = fmax(read_lane(v, 0), read_lane(v, 16)), hi = fmax(read_lane(v, 32), read_lane(v, 48));
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

// Rows of one compute unit.  Die x hosts workers x, x+8, ... (slots 0, 1, ...); compute unit c takes positions
// c, c+32, ... of each of their batches, and positions x+8c, x+8(c+32), ... of the shared batch J (slot S-1).
struct RowList {
  int32_t nws, cntW, cntJ, total;
  uint32_t x, c;
  int32_t S;
  __device__ __forceinline__ void slot_pos(int32_t q, int32_t &slot, uint32_t &tag, uint32_t &worker, uint32_t &pos) const {
    const int32_t nw = nws * cntW;
    if (q < nw) {
      const int32_t s = q / cntW, k = q - s * cntW;
      slot = s; tag = kTagBatch; worker = x + 8u * (uint32_t)s; pos = c + 32u * (uint32_t)k;
    } else {
      slot = S - 1; tag = kTagShared; worker = kSharedWorkerField; pos = x + 8u * (c + 32u * (uint32_t)(q - nw));
    }
  }
};

template <int KR, int RP>
__global__ __launch_bounds__(kResThreads) void resident_epoch_kernel(ResArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float *red = reinterpret_cast<float *>(smem);                                  // [2][16][8]
  QParams *qp = reinterpret_cast<QParams *>(smem + 1024);                        // [64]
  uint32_t *ctl_sh = reinterpret_cast<uint32_t *>(smem + 2048);                  // [4]: rank, alive
  float *u_sh = reinterpret_cast<float *>(smem + 2560);                          // [slots][cw] <= 8 * 512 floats
  int16_t *codes = reinterpret_cast<int16_t *>(smem + 2560 + 16384);             // [N][cw] <= 4096 codes

  const int tid0 = threadIdx.x;
  int tid = tid0, lane = tid0 & 63, e = tid0 - kRowThreads;  // e: index among the exchange threads (>= 0 for them)
  const int wave = tid0 >> 6;
  const bool warm_role = tid0 < kRowThreads;  // wavefronts 0-7 request the coming rows; 8-15 fold and exchange
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
    ctl_sh[0] = rank; ctl_sh[1] = ok;
  }
  __syncthreads();
  // (read back as scalars: everything derived from the rank is uniform over the workgroup)
  const uint32_t c = (uint32_t)__builtin_amdgcn_readfirstlane((int)ctl_sh[0]);
  bool alive = __builtin_amdgcn_readfirstlane((int)ctl_sh[1]) != 0;
  if (!alive) return;  // whole workgroup

  uint32_t *bar = a.ctl + kCtlBar + 32 * x;
  uint32_t bar_count = 0;  // barriers of the die this workgroup has arrived at (thread kRowThreads keeps it)

  RowList rl;
  rl.x = x; rl.c = c; rl.S = a.S;
  rl.nws = x < (uint32_t)a.N ? (a.N - (int32_t)x + 7) / 8 : 0;
  rl.cntW = c < (uint32_t)a.B ? (a.B - (int32_t)c + 31) / 32 : 0;
  const int32_t nJ = (a.alpc && x < (uint32_t)a.B) ? (a.B - (int32_t)x + 7) / 8 : 0;
  rl.cntJ = c < (uint32_t)nJ ? (nJ - (int32_t)c + 31) / 32 : 0;
  rl.total = rl.nws * rl.cntW + rl.cntJ;

  // ---- this compute unit's slice of the coordinates
  const int64_t col0 = (int64_t)c * a.cw;
  const int32_t ncols = (int32_t)c < a.nslices ? (int32_t)((a.d_pad - col0) < a.cw ? (a.d_pad - col0) : a.cw) : 0;
  // per-coordinate state of the update, held by exchange thread e for column col0 + e
  float w_j = 0.f, mu_j = 0.f, z_j = 0.f, ysum_j = 0.f, snap_j = 0.f, y_j = 0.f;
  const bool own = !warm_role && e < ncols && col0 + e < a.d;
  if (own) {
    const int64_t j = col0 + e;
    w_j = a.w[j]; mu_j = a.mu[j];
    if (a.alpc) { z_j = a.zv[j]; snap_j = a.w_snap[j]; }
  }
  double weight = 1.0;

  // Rows of the COMING iteration are touched, one word per 128-byte line, by wavefronts 0-7 as soon as this
  // iteration's rows are consumed (which rows are sampled does not depend on the iterate): they travel from HBM to
  // the die's L2 while wavefronts 8-15 fold and exchange, and the next row pass reads them from there.  The words
  // stay in registers until that pass, so no wait on them sits in the way; what they add up to is stored only if it
  // equals a value it cannot take.  (The loads of a wavefront return in order: a wavefront that synchronises on
  // short loads must not have such long ones outstanding, hence the split of the workgroup.)
  float touch[kTouch];
#pragma unroll
  for (int k = 0; k < kTouch; ++k) touch[k] = 0.f;
  float warm_sink = 0.f;
  auto touch_rows = [&](uint32_t iter) {
    StreamKey key = a.key;
    key.iter = a.key.iter + iter;
    const int32_t lines = (int32_t)((a.d + 31) / 32);
    int64_t mine = 0;  // lane r draws row r of this compute unit's list (the first 64 rows are touched)
    if (lane < rl.total) {
      int32_t slot; uint32_t tag, worker, pos;
      rl.slot_pos(lane, slot, tag, worker, pos);
      mine = sample_row(key, tag, worker, pos, a.n);
    }
    const int32_t nrows = rl.total < 64 ? rl.total : 64;
#pragma unroll
    for (int k = 0; k < kTouch; ++k) {
      const int32_t idx = tid + kRowThreads * k;
      const int32_t q = idx / lines, l = idx - q * lines;
      const uint32_t lo = (uint32_t)__shfl((int)(uint32_t)mine, q & 63), hi = (uint32_t)__shfl((int)(uint32_t)((uint64_t)mine >> 32), q & 63);
      const int64_t row = (int64_t)(((uint64_t)hi << 32) | lo);
      touch[k] = q < nrows ? a.X[row * a.ldx + (int64_t)l * 32] : 0.f;
    }
  };
  if (warm_role) touch_rows(0u);

  const bool tracer = a.trace != nullptr && x == 0u && c == 0u && tid0 == kRowThreads;
#define RES_STAMP(k) do { if (tracer) a.trace[(int64_t)t * 16 + (k)] = wall_clock64(); } while (0)
  int buf = 0;
  for (int32_t t = 0; t < a.m; ++t) {
    const int par = t & 1;
    // The thread index is made opaque once per iteration: otherwise every per-thread address of the loop body is
    // formed ahead of the loop and kept (or spilled) across all of it.
    tid = tid0;
    asm volatile("" : "+v"(tid));
    lane = tid & 63;
    e = tid - kRowThreads;
    RES_STAMP(0);
    // ================= rows: margins, slope differences, partial vectors ====================================
    float4 wreg[KR], acc[KR];
    {
      const float *wsrc = t == 0 ? a.w : a.wbuf + (int64_t)x * a.d_pad;
#pragma unroll
      for (int k = 0; k < KR; ++k) {
        const int64_t col = ((int64_t)k * kResThreads + tid) * 4;
        wreg[k] = col < a.d ? ld_agent4(wsrc + col) : make_float4(0.f, 0.f, 0.f, 0.f);
        acc[k] = make_float4(0.f, 0.f, 0.f, 0.f);
      }
    }
    int32_t cur_slot = -1;
    for (int32_t q0 = 0; q0 < rl.total; q0 += RP) {
      float4 xr[RP][KR];
      float yr[RP], zr[RP];
      {
        // lane r of a wavefront draws row q0 + r's index
        StreamKey key = a.key;
        key.iter = a.key.iter + (uint32_t)t;
        int64_t mine = 0;
        if (lane < RP && q0 + lane < rl.total) {
          int32_t slot; uint32_t tag, worker, pos;
          rl.slot_pos(q0 + lane, slot, tag, worker, pos);
          mine = sample_row(key, tag, worker, pos, a.n);
        }
#pragma unroll
        for (int r = 0; r < RP; ++r) {
          const uint32_t lo = read_lane((uint32_t)mine, r), hi = read_lane((uint32_t)((uint64_t)mine >> 32), r);
          const int64_t row = (int64_t)(((uint64_t)hi << 32) | lo);
          const bool live = q0 + r < rl.total;
          const float *src = a.X + row * a.ldx;
          yr[r] = live ? a.y[row] : 0.f;
          zr[r] = live ? a.z_snap[row] : 0.f;
#pragma unroll
          for (int k = 0; k < KR; ++k) {
            const int64_t col = ((int64_t)k * kResThreads + tid) * 4;
            xr[r][k] = (live && col < a.d) ? *reinterpret_cast<const float4 *>(src + col) : make_float4(0.f, 0.f, 0.f, 0.f);
          }
        }
      }
      if (q0 == 0 && warm_role) {  // the words that warmed these rows have arrived by now
#pragma unroll
        for (int k = 0; k < kTouch; ++k) warm_sink += touch[k];
      }
      {
        float s[RP];
#pragma unroll
        for (int r = 0; r < RP; ++r) {
          float v = 0.f;
#pragma unroll
          for (int k = 0; k < KR; ++k) {
            v = fmaf(xr[r][k].x, wreg[k].x, v); v = fmaf(xr[r][k].y, wreg[k].y, v);
            v = fmaf(xr[r][k].z, wreg[k].z, v); v = fmaf(xr[r][k].w, wreg[k].w, v);
          }
          s[r] = wave_sum(v);
        }
        if (lane == 0) {
#pragma unroll
          for (int r = 0; r < RP; ++r) red[(buf * 16 + wave) * 8 + r] = s[r];
        }
      }
      __syncthreads();
#pragma unroll
      for (int r = 0; r < RP; ++r) {
        if (q0 + r >= rl.total) break;  // uniform
        float z = red[(buf * 16 + 0) * 8 + r];
#pragma unroll
        for (int wv = 1; wv < 16; ++wv) z += red[(buf * 16 + wv) * 8 + r];
        // x_0 is the snapshot itself in Alg. 1: every difference is exactly zero there
        const float coef = (!a.alpc && t == 0) ? 0.f : loss_slope(a.loss, z, yr[r]) - loss_slope(a.loss, zr[r], yr[r]);
        int32_t slot; uint32_t tag, worker, pos;
        rl.slot_pos(q0 + r, slot, tag, worker, pos);
        if (slot != cur_slot) {
          if (cur_slot >= 0) {
            float *dst = a.part + (((int64_t)x * a.S + cur_slot) * kCusPerXcd + c) * a.d_pad;
#pragma unroll
            for (int k = 0; k < KR; ++k) {
              const int64_t col = ((int64_t)k * kResThreads + tid) * 4;
              if (col < a.d) *reinterpret_cast<float4 *>(dst + col) = acc[k];
            }
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
      for (int k = 0; k < KR; ++k) {
        const int64_t col = ((int64_t)k * kResThreads + tid) * 4;
        if (col < a.d) *reinterpret_cast<float4 *>(dst + col) = acc[k];
      }
    }
    RES_STAMP(1);
    wait_stores();  // the partial vectors are in the die's L2
    if (warm_role && t + 1 < a.m) touch_rows((uint32_t)(t + 1));
    __syncthreads();
    RES_STAMP(2);
    // ================= barrier of the die, then the fold of this compute unit's slice =======================
    if (tid == kRowThreads) {
      die_add(bar, 1u);
      ++bar_count;
      const bool ok = wait_reach(bar, (uint32_t)kCusPerXcd * bar_count, abort_word, a.spin_limit);
      ctl_sh[1] = ok ? 1u : 0u;
    }
    __syncthreads();
    RES_STAMP(3);
    alive = __builtin_amdgcn_readfirstlane((int)ctl_sh[1]) != 0;
    if (!alive) break;
    const int32_t nfold = rl.nws + (a.alpc ? 1 : 0);  // vectors this die folds
    const int32_t npair = ncols / 2;
    if (!warm_role) {
      for (int32_t idx = e; idx < nfold * npair; idx += kRowThreads) {
        const int32_t si = idx / npair, pr = idx - si * npair;
        const bool shared = si >= rl.nws;
        const int32_t slot = shared ? a.S - 1 : si;
        const int32_t ncu = shared ? (nJ < kCusPerXcd ? nJ : kCusPerXcd) : (a.B < kCusPerXcd ? a.B : kCusPerXcd);
        const float *src = a.part + ((int64_t)x * a.S + slot) * kCusPerXcd * a.d_pad + col0 + 2 * pr;
        float2 v = make_float2(0.f, 0.f);
        for (int32_t c0 = 0; c0 < ncu; c0 += 8) {  // eight partial vectors in flight
          float2 p[8];
#pragma unroll
          for (int k = 0; k < 8; ++k)
            p[k] = c0 + k < ncu ? ld_agent2(src + (int64_t)(c0 + k) * a.d_pad) : make_float2(0.f, 0.f);
#pragma unroll
          for (int k = 0; k < 8; ++k) { v.x += p[k].x; v.y += p[k].y; }
        }
        const int64_t col = col0 + 2 * pr;
        if (col >= a.d) v = make_float2(0.f, 0.f);
        if (shared) {
          st_agent2(a.jbuf + ((int64_t)par * kXcds + x) * a.d_pad + col, v.x, v.y);
        } else {
          v.x *= a.scale; v.y *= a.scale;
          const int32_t worker = (int32_t)x + 8 * si;
          st_agent2(a.ubuf + ((int64_t)par * a.N + worker) * a.d_pad + col, v.x, v.y);
          u_sh[si * a.cw + 2 * pr] = v.x;
          u_sh[si * a.cw + 2 * pr + 1] = v.y;
        }
      }
    }
    __syncthreads();
    RES_STAMP(4);
    if (!warm_role) {
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
        if (lane == 0 && ncols > 0) {
          double *dst = a.statbuf + (((int64_t)par * a.N + ((int32_t)x + 8 * si)) * kCusPerXcd + c) * 4;
          st_agent(dst, (double)fmx); st_agent(dst + 1, sum); st_agent(dst + 2, sumsq); st_agent(dst + 3, bad);
        }
      }
      wait_stores();  // everything this slice publishes has been written
    }
    __syncthreads();
    RES_STAMP(5);
    // ================= exchange: wait for the eight publishers of this slice =================================
    if (tid == kRowThreads && ncols > 0) st_agent(a.ctl + kCtlFlag + 32 * c + x, (uint32_t)(t + 1));
    if (wave == 8) {
      bool ok = true;
      if (ncols > 0) {
        ok = false;
        const uint32_t *f = a.ctl + kCtlFlag + 32 * c + (lane & 7);
        for (uint32_t k = 0; k < a.spin_limit; ++k) {
          const bool ready = lane >= 8 || (int32_t)(ld_agent(f) - (uint32_t)(t + 1)) >= 0;
          if (__ballot(!ready) == 0ull) { ok = true; break; }
          if ((k & 63u) == 63u && ld_agent(abort_word) != 0u) break;
          __builtin_amdgcn_s_sleep(1);
        }
      }
      if (lane == 0) ctl_sh[1] = ok ? 1u : 0u;
    }
    __syncthreads();
    RES_STAMP(6);
    alive = __builtin_amdgcn_readfirstlane((int)ctl_sh[1]) != 0;
    if (!alive) break;
    float4 uq[kResBlocks];
    float uhat = 0.f;
    const int32_t nquad = ncols / 4;
    if (!warm_role && ncols > 0) {
      // this thread's blocks of four coordinates of the workers' vectors ...
#pragma unroll
      for (int q = 0; q < kResBlocks; ++q) {
        const int32_t b = e + kRowThreads * q;
        uq[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (b < a.N * nquad) {
          const int32_t i = b / nquad, l = b - i * nquad;
          uq[q] = ld_agent4(a.ubuf + ((int64_t)par * a.N + i) * a.d_pad + col0 + 4 * l);
        }
      }
      // ... the shared batch's difference for this thread's column (die order, then 1/B) ...
      if (a.alpc && e < ncols) {
        float pj[kXcds];
#pragma unroll
        for (int k = 0; k < kXcds; ++k) pj[k] = ld_agent(a.jbuf + ((int64_t)par * kXcds + k) * a.d_pad + col0 + e);
        float sj = pj[0];
#pragma unroll
        for (int k = 1; k < kXcds; ++k) sj += pj[k];
        uhat = sj * a.scale;
      }
      // ... and eq. (3): a half wavefront folds the slice statistics of one vector (slice k on lane k)
      const int l32 = lane & 31;
      for (int32_t i0 = 2 * (wave - 8); i0 < a.N; i0 += 16) {
        const int32_t i = i0 + (lane >> 5);
        double am = 0.0, s = 0.0, s2 = 0.0, bd = 0.0;
        if (i < a.N && l32 < a.nslices) {
          const double *src = a.statbuf + (((int64_t)par * a.N + i) * kCusPerXcd + l32) * 4;
          am = ld_agent(src); s = ld_agent(src + 1); s2 = ld_agent(src + 2); bd = ld_agent(src + 3);
        }
        am = half_max(am, lane); s = half_sum(s, lane); s2 = half_sum(s2, lane); bd = half_sum(bd, lane);
        if (l32 == 0 && i < a.N) {
          const QParams q_i = make_qparams(a.qs, am, s, s2, a.d);
          qp[i] = q_i;
          if (x == 0u && c == 0u) {
            a.delta_out[i] = q_i.delta;
            double *o = a.stats_out + (int64_t)i * 4;
            o[0] = am; o[1] = s; o[2] = s2; o[3] = bd;
            if (bd > 0.0) atomicOr(a.flags, 1u);
          }
        }
      }
    }
    __syncthreads();
    RES_STAMP(7);
    if (!warm_role && ncols > 0) {
      // Sec. 3.2 rules (1), (2) in fp32, one IEEE operation per step
      const float hi = (float)((1 << (a.bits - 1)) - 1);
      const float lo = -(float)(1 << (a.bits - 1));
      StreamKey key = a.key;
      key.iter = a.key.iter + (uint32_t)t;
#pragma unroll
      for (int q = 0; q < kResBlocks; ++q) {
        const int32_t b = e + kRowThreads * q;
        if (b >= a.N * nquad) break;
        const int32_t i = b / nquad, l = b - i * nquad;
        const QParams qi = qp[i];
        const float vals[4] = {uq[q].x, uq[q].y, uq[q].z, uq[q].w};
        const Philox4 blk = stream_block(key, kTagQuant, (uint32_t)i, (uint32_t)((col0 + 4 * l) >> 2));
        const uint32_t rnd[4] = {blk.x, blk.y, blk.z, blk.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          float s = vals[k] * qi.rdelta;
          s = fminf(fmaxf(s, lo), hi);
          const float base = floorf(s);
          const float frac = s - base;
          const float unif = (float)(rnd[k] >> 8) * 0x1.0p-24f;
          const int32_t code = qi.delta > 0.0f ? (int32_t)base + ((unif < frac) ? 1 : 0) : 0;
          codes[i * a.cw + 4 * l + k] = (int16_t)code;
        }
      }
    }
    __syncthreads();
    RES_STAMP(8);
    if (!warm_role && ncols > 0) {
      if (x == 0u) {  // the packed messages (Sec. 4.2): die 0 stores them
        const int32_t bits = a.bits;
        const uint32_t mask = (1u << bits) - 1u;
        const int32_t words_per_vec = (ncols / 32) * bits;
        const int64_t seg0 = col0 / 32;
        for (int32_t idx = e; idx < a.N * words_per_vec; idx += kRowThreads) {
          const int32_t i = idx / words_per_vec, rem = idx - i * words_per_vec;
          const int32_t sgm = rem / bits, wd = rem - sgm * bits;
          const int32_t bit0 = 32 * wd;
          uint32_t word = 0u;
          for (int32_t k = bit0 / bits; k < 32 && k * bits < bit0 + 32; ++k) {
            const uint32_t field = (uint32_t)(int32_t)codes[i * a.cw + 32 * sgm + k] & mask;
            const int32_t sh = k * bits - bit0;
            word |= sh >= 0 ? (field << sh) : (field >> (-sh));
          }
          a.packed[(int64_t)i * a.W + (seg0 + sgm) * bits + wd] = word;
        }
      }
      if (e < ncols) {
        float next = 0.f;
        if (own) {
          // eq. (4) in worker order
          float sum = 0.f;
          for (int32_t i = 0; i < a.N; ++i) sum = __builtin_fmaf(qp[i].delta, (float)codes[i * a.cw + e], sum);
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
        a.wbuf[(int64_t)x * a.d_pad + col0 + e] = next;
      }
      wait_stores();  // this slice of the iterate is in the die's L2
    }
    weight *= (double)a.theta;
    __syncthreads();
    RES_STAMP(9);
    // ================= second barrier of the die: the whole iterate is there ================================
    if (tid == kRowThreads) {
      die_add(bar, 1u);
      ++bar_count;
      const bool ok = wait_reach(bar, (uint32_t)kCusPerXcd * bar_count, abort_word, a.spin_limit);
      ctl_sh[1] = ok ? 1u : 0u;
    }
    __syncthreads();
    RES_STAMP(10);
    alive = __builtin_amdgcn_readfirstlane((int)ctl_sh[1]) != 0;
    if (!alive) break;
  }
#undef RES_STAMP
  if (!alive) {
    if (tid == 0) {
      st_agent(abort_word, 1u);
      atomicOr(a.flags, 2u);
    }
    return;
  }
  if (warm_sink == -1.2345678e-38f) a.wbuf[0] = warm_sink;
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
  if (c->cus != kXcds * kCusPerXcd) return false;
  return true;
}

size_t resident_part_floats(const lpc_ctx *c) { return (size_t)kXcds * res_slots(c) * kCusPerXcd * c->d_pad; }
size_t resident_ubuf_floats(const lpc_ctx *c) { return (size_t)2 * c->cfg.N * c->d_pad; }
size_t resident_jbuf_floats(const lpc_ctx *c) { return (size_t)2 * kXcds * c->d_pad; }
size_t resident_stat_doubles(const lpc_ctx *c) { return (size_t)2 * c->cfg.N * kCusPerXcd * 4; }
size_t resident_wbuf_floats(const lpc_ctx *c) { return (size_t)kXcds * c->d_pad; }
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
  a.part = c->s.res_part; a.ubuf = c->s.res_ubuf; a.jbuf = c->s.res_jbuf; a.statbuf = c->s.res_stat;
  a.wbuf = c->s.res_wbuf; a.ctl = c->s.res_ctl;
  a.packed = c->s.packed; a.delta_out = c->s.delta; a.stats_out = c->s.stats; a.flags = c->s.flags;
  a.S = res_slots(c); a.cw = res_cw(c); a.nslices = (int32_t)((c->d_pad + a.cw - 1) / a.cw);
  a.spin_limit = c->spin_limit;
  a.trace = c->res_trace_on ? c->s.res_trace : nullptr;
  // counters and flags of the launch start at zero (a fill kernel: the caller may be capturing the stream)
  hipError_t err = launch_fill_u32(c->s.res_ctl, 0u, (int64_t)kCtlWords, st);
  if (err != hipSuccess) return err;
  const int64_t chunks = (c->d + 4 * kResThreads - 1) / (4 * kResThreads);  // float4 chunks of a row per thread
  const void *fn = nullptr;
  if (chunks <= 1) fn = reinterpret_cast<const void *>(&resident_epoch_kernel<1, 8>);
  else if (chunks <= 2) fn = reinterpret_cast<const void *>(&resident_epoch_kernel<2, 6>);
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
