// fp32 matrix-core GEMM for the MLP instance of eq. (1) (gfx950).
//
//   C[m][n] (+)= alpha * sum_{segments} sum_k opA(m,k) * opB(k,n)   (+ bias[n], ReLU, ReLU-mask)
//
// The only dense contractions of the hot path are the MLP's layer products, so
// this is where MFMA is used: v_mfma_f32_32x32x2_f32, fp32 in, fp32 accumulate.
// A workgroup of 4 wavefronts owns a 128x64 tile of C; each wavefront owns a
// 64x32 part = 2x1 MFMA tiles (32 accumulator registers).  (128x128 tiles, 64
// accumulator registers per lane, were measured no faster on any product here,
// 4096^3 included: their 164 registers allow three workgroups per CU, not four.)
// The K loop runs
// in slabs of 16: the next slab is fetched from global memory into registers
// while the current one is consumed from LDS (stored k-major so that the 32
// lanes of an MFMA operand read consecutive words).  Operands may be given
// transposed (weight gradients A'D and data gradients D W' need it) and the K
// range may consist of two segments with their own base pointers (the
// difference of two weight gradients is one contraction over stacked rows).
#include <hip/hip_runtime.h>

#include "lpc_device.h"
#include "lpc_internal.h"

namespace lpc {

namespace {

#ifndef LPC_GEMM_BK
#define LPC_GEMM_BK 16
#endif
constexpr int BM = 128, BN = 64, BK = LPC_GEMM_BK;
constexpr int LDT = BM + 4;  // LDS row pitch (floats)

typedef float floatx16 __attribute__((ext_vector_type(16)));

// element (r, c) of a row-major matrix with leading dimension ld, zero outside [0,R)x[0,C)
__device__ __forceinline__ float guarded(const float *p, int64_t ld, int r, int c, int R, int C) {
  return (r < R && c < C) ? p[(int64_t)r * ld + c] : 0.0f;
}

// Fetch this thread's share of a TILE x BK operand slab into registers, as TILE*BK/1024 groups of four.
//   TRANS == false: the operand is stored [mn][k] (k contiguous).  Group h of thread t: row t/(BK/4) +
//                   h*(1024/BK), columns k0 + 4*(t % (BK/4)) .. +3.
//   TRANS == true : the operand is stored [k][mn] (mn contiguous).  Group h of thread t: row k0 +
//                   t/(TILE/4) + h*(1024/TILE), columns 4*(t % (TILE/4)) .. +3.
// FULL: the whole slab lies inside the operand and is 16-byte aligned (the launcher checks): plain vector
// loads with no branches between them, so all of a slab's loads are in flight together.
template <bool TRANS, int TILE, bool FULL>
__device__ __forceinline__ void fetch_slab(const float *__restrict__ p, int64_t ld, int mn0, int k0, int MN, int K,
                                           bool vec_ok, int tid, float (&r)[TILE * BK / 256]) {
  constexpr int G = TILE * BK / 1024;
#pragma unroll
  for (int h = 0; h < G; ++h) {
    int row, col, R, C;
    if (!TRANS) { row = mn0 + tid / (BK / 4) + h * (1024 / BK); col = k0 + 4 * (tid % (BK / 4)); R = MN; C = K; }
    else { row = k0 + tid / (TILE / 4) + h * (1024 / TILE); col = mn0 + 4 * (tid % (TILE / 4)); R = K; C = MN; }
    if constexpr (FULL) {
      const float4 v = *reinterpret_cast<const float4 *>(p + (int64_t)row * ld + col);
      r[4 * h + 0] = v.x; r[4 * h + 1] = v.y; r[4 * h + 2] = v.z; r[4 * h + 3] = v.w;
    } else if (vec_ok && row < R && col + 3 < C) {
      const float4 v = *reinterpret_cast<const float4 *>(p + (int64_t)row * ld + col);
      r[4 * h + 0] = v.x; r[4 * h + 1] = v.y; r[4 * h + 2] = v.z; r[4 * h + 3] = v.w;
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) r[4 * h + i] = guarded(p, ld, row, col + i, R, C);
    }
  }
}

// The same shares for whole tiles (FULL), slab after slab: the thread's address is set up once per segment and
// then moved by pointer steps, so no product is formed per load.  fetch() reads the next slab, in order.
template <bool TRANS, int TILE>
struct SlabWalker {
  const float *p;
  int64_t hstep, kstep;
  __device__ __forceinline__ void init(const float *base, int64_t ld, int mn0, int tid) {
    if (!TRANS) {
      p = base + (int64_t)(mn0 + tid / (BK / 4)) * ld + 4 * (tid % (BK / 4));
      hstep = (int64_t)(1024 / BK) * ld;
      kstep = BK;
    } else {
      p = base + (int64_t)(tid / (TILE / 4)) * ld + mn0 + 4 * (tid % (TILE / 4));
      hstep = (int64_t)(1024 / TILE) * ld;
      kstep = (int64_t)BK * ld;
    }
  }
  __device__ __forceinline__ void fetch(float (&r)[TILE * BK / 256]) {
    constexpr int G = TILE * BK / 1024;
#pragma unroll
    for (int h = 0; h < G; ++h) {
      const float4 v = *reinterpret_cast<const float4 *>(p + h * hstep);
      r[4 * h + 0] = v.x; r[4 * h + 1] = v.y; r[4 * h + 2] = v.z; r[4 * h + 3] = v.w;
    }
    p += kstep;
  }
};

// Store the registers k-major into an LDS slab T[k][mn].
template <bool TRANS, int TILE>
__device__ __forceinline__ void stash_slab(float (*T)[LDT], int tid, const float (&r)[TILE * BK / 256]) {
  constexpr int G = TILE * BK / 1024;
#pragma unroll
  for (int h = 0; h < G; ++h) {
    if (!TRANS) {
      const int mn = tid / (BK / 4) + h * (1024 / BK), k = 4 * (tid % (BK / 4));
#pragma unroll
      for (int i = 0; i < 4; ++i) T[k + i][mn] = r[4 * h + i];
    } else {
      const int k = tid / (TILE / 4) + h * (1024 / TILE), mn = 4 * (tid % (TILE / 4));
      *reinterpret_cast<float4 *>(&T[k][mn]) = make_float4(r[4 * h], r[4 * h + 1], r[4 * h + 2], r[4 * h + 3]);
    }
  }
}

// Epilogue of one output tile: C (+)= alpha*acc (+ bias, ReLU, ReLU mask), and the statistics of the stored
// values (per thread in fp32 -- at most 64 terms --, in fp64 across threads).
// Accumulator layout of the 32x32 MFMA: lane l holds column (l % 32); register v holds row
// 8*(v/4) + 4*(l/32) + (v%4).
// The options are compile-time so that the 32 stores of a thread are straight-line code: FULL = the tile lies
// inside C (no row / column checks).  Rows are reached by pointer steps of ldc, not by a product per element.
template <int TN, bool FULL, bool BIAS, bool RELU, bool MASK, bool ACC, bool STAT>
__device__ __forceinline__ void store_tile_as(const GemmArgs &g, const floatx16 (&acc)[2][TN / 64], int m0, int n0,
                                              int64_t bz, int lane, int wm, int wn, float &fmx, float &ssum,
                                              float &ssq, float &sbad) {
  constexpr int NJ = TN / 64;
  const int64_t ldc = g.ldc;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      const int col = n0 + wn + 32 * j + (lane & 31);
      if (!FULL && col >= g.N) continue;
      const float bias = BIAS ? g.bias[bz * g.strideBias + col] : 0.0f;
      const int row0 = m0 + wm + 32 * i + 4 * (lane >> 5);
      const int64_t off0 = bz * g.strideC + (int64_t)row0 * ldc + col;
      float *crow = g.C + off0;
      const float *mrow = MASK ? g.relu_mask + off0 : nullptr;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int dr = 8 * (v >> 2) + (v & 3);
        if (!FULL && row0 + dr >= g.M) continue;
        float *cp = crow + dr * ldc;
        float val = g.alpha * acc[i][j][v] + bias;
        if (RELU) val = val > 0.0f ? val : 0.0f;
        if (MASK) val = mrow[dr * ldc] > 0.0f ? val : 0.0f;
        if (ACC) val += *cp;
        *cp = val;
        if (STAT) {
          if (isfinite(val)) {
            fmx = fmaxf(fmx, fabsf(val)); ssum += val; ssq = fmaf(val, val, ssq);
          } else {
            sbad += 1.0f;
          }
        }
      }
    }
  }
}

// Picks the instantiation for the (uniform) options of this launch: the MLP's products use four combinations;
// anything else takes the general one.
template <int TN, bool FULL>
__device__ __forceinline__ void store_tile(const GemmArgs &g, const floatx16 (&acc)[2][TN / 64], int m0, int n0,
                                           int64_t bz, int lane, int wm, int wn, float &fmx, float &ssum, float &ssq,
                                           float &sbad) {
  const bool bias = g.bias != nullptr, relu = g.relu != 0, mask = g.relu_mask != nullptr, accu = g.accumulate != 0,
             stat = g.stat_part != nullptr;
  if (bias && relu && !mask && !accu && !stat)          // forward layer
    store_tile_as<TN, FULL, true, true, false, false, false>(g, acc, m0, n0, bz, lane, wm, wn, fmx, ssum, ssq, sbad);
  else if (!bias && !relu && mask && !accu && !stat)    // data gradient
    store_tile_as<TN, FULL, false, false, true, false, false>(g, acc, m0, n0, bz, lane, wm, wn, fmx, ssum, ssq, sbad);
  else if (!bias && !relu && !mask && !accu && stat)    // a worker's weight gradient, with its statistics
    store_tile_as<TN, FULL, false, false, false, false, true>(g, acc, m0, n0, bz, lane, wm, wn, fmx, ssum, ssq, sbad);
  else if (!bias && !relu && !mask && !stat && accu)    // snapshot weight gradient, accumulating
    store_tile_as<TN, FULL, false, false, false, true, false>(g, acc, m0, n0, bz, lane, wm, wn, fmx, ssum, ssq, sbad);
  else if (!bias && !relu && !mask && !stat)            // snapshot weight gradient, first chunk or block
    store_tile_as<TN, FULL, false, false, false, false, false>(g, acc, m0, n0, bz, lane, wm, wn, fmx, ssum, ssq, sbad);
  else {
    // general: every option decided per element
    constexpr int NJ = TN / 64;
    float *C = g.C + bz * g.strideC;
    const float *mk = mask ? g.relu_mask + bz * g.strideC : nullptr;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        const int col = n0 + wn + 32 * j + (lane & 31);
        if (col >= g.N) continue;
        const float bv = bias ? g.bias[bz * g.strideBias + col] : 0.0f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          if (row >= g.M) continue;
          const int64_t off = (int64_t)row * g.ldc + col;
          float val = g.alpha * acc[i][j][v] + bv;
          if (relu) val = val > 0.0f ? val : 0.0f;
          if (mk) val = mk[off] > 0.0f ? val : 0.0f;
          if (accu) val += C[off];
          C[off] = val;
          if (stat) {
            if (isfinite(val)) {
              fmx = fmaxf(fmx, fabsf(val)); ssum += val; ssq = fmaf(val, val, ssq);
            } else {
              sbad += 1.0f;
            }
          }
        }
      }
    }
  }
}

// The tile's statistics: wavefront reductions, then the wavefronts in order through `red` (LDS, 4 doubles per
// wavefront, not in use by anyone else); slot `tile` of batch item bz receives them.  Contains a barrier.
__device__ __forceinline__ void tile_statistics(const GemmArgs &g, double *red, int tid, int64_t bz, int64_t tile,
                                                float fmx, double ssum, double ssq, double sbad) {
  const int lane = tid & 63, wave = tid >> 6;
  const double a_w = (double)wave_max(fmx), s_w = wave_sum(ssum), q_w = wave_sum(ssq), b_w = wave_sum(sbad);
  if (lane == 0) { red[wave * 4 + 0] = a_w; red[wave * 4 + 1] = s_w; red[wave * 4 + 2] = q_w; red[wave * 4 + 3] = b_w; }
  __syncthreads();
  if (tid == 0) {
    double a_t = 0.0, s_t = 0.0, q_t = 0.0, b_t = 0.0;
    for (int k = 0; k < 4; ++k) { a_t = fmax(a_t, red[k * 4]); s_t += red[k * 4 + 1]; q_t += red[k * 4 + 2]; b_t += red[k * 4 + 3]; }
    double *p = g.stat_part + bz * g.stat_batch_stride + ((int64_t)g.stat_slot0 + tile) * 4;
    p[0] = a_t; p[1] = s_t; p[2] = q_t; p[3] = b_t;
  }
}

// TN = 64: 128x64 tile, each wavefront 64x32 (2x1 MFMA tiles); the code is also valid for TN = 128 (2x2).
template <bool TA, bool TB, int TN, bool FULL>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs g) {
  touch_kernel_arguments<(int)(sizeof(GemmArgs))>();
  constexpr int NJ = TN / 64;
  __shared__ __attribute__((aligned(16))) float As[2][BK][LDT];
  __shared__ __attribute__((aligned(16))) float Bs[2][BK][LDT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * 64, wn = (wave & 1) * (TN / 2);
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * TN;
  const int64_t bz = blockIdx.z;

  floatx16 acc[2][NJ];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  // Two register sets per operand: while slab t is consumed from LDS, slab t+1 waits in registers and slab t+2
  // is in flight, so a slab's loads have two slabs' worth of matrix-unit time to arrive.
  float ra[2][BM * BK / 256], rb[2][TN * BK / 256];
  auto consume = [&](int cur) {
    // the wavefront that has its operands in LDS goes first: +0.5 % on the MLP workload, back to back
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      const int kr = kk + (lane >> 5), c = lane & 31;
      const float a0 = As[cur][kr][wm + c], a1 = As[cur][kr][wm + 32 + c];
      const float b0 = Bs[cur][kr][wn + c];
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      if constexpr (NJ == 2) {
        const float b1 = Bs[cur][kr][wn + 32 + c];
        acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
        acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
      }
    }
    __builtin_amdgcn_s_setprio(0);
  };
  for (int s = 0; s < g.nseg; ++s) {
    const float *A = g.A[s] + bz * g.strideA[s];
    const float *B = g.B[s] + bz * g.strideB[s];
    const int64_t lda = g.lda[s], ldb = g.ldb[s];
    const bool va = (lda % 4 == 0) && (((uintptr_t)A & 15u) == 0);
    const bool vb = (ldb % 4 == 0) && (((uintptr_t)B & 15u) == 0);
    const int K = g.K;
    const int nslab = (K + BK - 1) / BK;
    SlabWalker<TA, BM> wa;
    SlabWalker<!TB, TN> wb;
    if constexpr (FULL) {
      wa.init(A, lda, m0, tid);
      wb.init(B, ldb, n0, tid);
    }
    // slab `at` into register set P (whole tiles: the walkers deliver the slabs in order, `at` is implied)
#define LPC_GEMM_FETCH(P, at)                                                          \
    if constexpr (FULL) {                                                              \
      wa.fetch(ra[(P)]);                                                               \
      wb.fetch(rb[(P)]);                                                               \
    } else {                                                                           \
      fetch_slab<TA, BM, false>(A, lda, m0, (at)*BK, g.M, K, va, tid, ra[(P)]);        \
      fetch_slab<!TB, TN, false>(B, ldb, n0, (at)*BK, g.N, K, vb, tid, rb[(P)]);       \
    }
    LPC_GEMM_FETCH(0, 0)
    if (nslab > 1) { LPC_GEMM_FETCH(1, 1) }
    __syncthreads();  // the previous segment's last slab has been consumed
    stash_slab<TA, BM>(As[0], tid, ra[0]);
    stash_slab<!TB, TN>(Bs[0], tid, rb[0]);
    __syncthreads();
    // step p of a pair handles slab t+p, which sits in LDS buffer p; registers [1-p] hold slab t+p+1 and
    // registers [p] are free for slab t+p+2
#define LPC_GEMM_STEP(P)                                                                        \
    {                                                                                           \
      const int slab = t + (P);                                                                 \
      if (slab + 2 < nslab) { LPC_GEMM_FETCH((P), slab + 2) }                                   \
      consume((P));                                                                             \
      if (slab + 1 < nslab) {                                                                   \
        stash_slab<TA, BM>(As[1 - (P)], tid, ra[1 - (P)]);                                      \
        stash_slab<!TB, TN>(Bs[1 - (P)], tid, rb[1 - (P)]);                                     \
      }                                                                                         \
      __syncthreads();                                                                          \
    }
    for (int t = 0; t < nslab; t += 2) {
      LPC_GEMM_STEP(0)
      if (t + 1 < nslab) LPC_GEMM_STEP(1)
    }
#undef LPC_GEMM_STEP
#undef LPC_GEMM_FETCH
  }

  float fmx = 0.0f, ssum = 0.0f, ssq = 0.0f, sbad = 0.0f;
  store_tile<TN, FULL>(g, acc, m0, n0, bz, lane, wm, wn, fmx, ssum, ssq, sbad);
  // LDS is free for the statistics: the K loop ended with a barrier
  if (g.stat_part)
    tile_statistics(g, reinterpret_cast<double *>(&As[0][0][0]), tid, bz,
                    (int64_t)blockIdx.y * gridDim.x + blockIdx.x, fmx, ssum, ssq, sbad);
}

// Whole 128x64 tiles with EIGHT wavefronts (one 32x32 matrix-core tile each) instead of four: for products
// with only one or two tiles per CU this doubles the wavefronts per SIMD, so that one wavefront's operand
// staging and barrier waits are covered by another's matrix instructions.  Whole tiles only (the launcher
// checks); 512 threads fetch a slab with one 16-byte load each for A and (the first 256) for B.
template <bool TA, bool TB>
__global__ __launch_bounds__(512) void gemm_mfma8_kernel(GemmArgs g) {
  touch_kernel_arguments<(int)(sizeof(GemmArgs))>();
  static_assert(BK == 16, "thread-to-slab mapping below is for 16-deep slabs");
  __shared__ __attribute__((aligned(16))) float As[2][BK][LDT];
  __shared__ __attribute__((aligned(16))) float Bs[2][BK][LDT];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = (wave >> 1) * 32, wn = (wave & 1) * 32;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * 64;
  const int64_t bz = blockIdx.z;
  floatx16 acc;
#pragma unroll
  for (int v = 0; v < 16; ++v) acc[v] = 0.0f;
  // slab element owned by this thread: A stored [m][k] -> row tid/4, k 4*(tid%4); stored [k][m] -> k tid/32,
  // m 4*(tid%32).  B (threads 0..255) stored [n][k] -> row tid/4, k 4*(tid%4); stored [k][n] -> k tid/16, n 4*(tid%16).
  const int a_r = TA ? (tid >> 5) : (tid >> 2), a_c = TA ? 4 * (tid & 31) : 4 * (tid & 3);
  const int b_r = TB ? (tid >> 2) : (tid >> 4), b_c = TB ? 4 * (tid & 3) : 4 * (tid & 15);
  const bool b_thread = tid < 256;
  float4 ra0, ra1, rb0, rb1;  // two register sets (named, so that they stay in registers)
  ra0 = ra1 = rb0 = rb1 = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < g.nseg; ++s) {
    const float *A = g.A[s] + bz * g.strideA[s];
    const float *B = g.B[s] + bz * g.strideB[s];
    const int64_t lda = g.lda[s], ldb = g.ldb[s];
    const int nslab = g.K / BK;
    // address of this thread's element of slab 0; consecutive slabs are 16 k apart
    const float *pa = TA ? A + (int64_t)a_r * lda + m0 + a_c : A + (int64_t)(m0 + a_r) * lda + a_c;
    const float *pb = TB ? B + (int64_t)(n0 + b_r) * ldb + b_c : B + (int64_t)b_r * ldb + n0 + b_c;
    const int64_t sa = TA ? (int64_t)BK * lda : BK, sb = TB ? BK : (int64_t)BK * ldb;
#define LPC_GEMM8_FETCH(SLAB, RA, RB)                                              \
    {                                                                              \
      RA = *reinterpret_cast<const float4 *>(pa + (SLAB) * sa);                    \
      if (b_thread) RB = *reinterpret_cast<const float4 *>(pb + (SLAB) * sb);      \
    }
#define LPC_GEMM8_STASH(BUF, RA, RB)                                               \
    {                                                                              \
      if (TA) {                                                                    \
        *reinterpret_cast<float4 *>(&As[BUF][a_r][a_c]) = RA;                      \
      } else {                                                                     \
        As[BUF][a_c + 0][a_r] = RA.x; As[BUF][a_c + 1][a_r] = RA.y;                \
        As[BUF][a_c + 2][a_r] = RA.z; As[BUF][a_c + 3][a_r] = RA.w;                \
      }                                                                            \
      if (b_thread) {                                                              \
        if (!TB) {                                                                 \
          *reinterpret_cast<float4 *>(&Bs[BUF][b_r][b_c]) = RB;                    \
        } else {                                                                   \
          Bs[BUF][b_c + 0][b_r] = RB.x; Bs[BUF][b_c + 1][b_r] = RB.y;              \
          Bs[BUF][b_c + 2][b_r] = RB.z; Bs[BUF][b_c + 3][b_r] = RB.w;              \
        }                                                                          \
      }                                                                            \
    }
#define LPC_GEMM8_CONSUME(BUF)                                                                               \
    _Pragma("unroll") for (int kk = 0; kk < BK; kk += 2) {                                                   \
      const int kr = kk + (lane >> 5), c = lane & 31;                                                        \
      acc = __builtin_amdgcn_mfma_f32_32x32x2f32(As[BUF][kr][wm + c], Bs[BUF][kr][wn + c], acc, 0, 0, 0);    \
    }
    LPC_GEMM8_FETCH(0, ra0, rb0)
    if (nslab > 1) LPC_GEMM8_FETCH(1, ra1, rb1)
    __syncthreads();  // the previous segment's last slab has been consumed
    LPC_GEMM8_STASH(0, ra0, rb0)
    __syncthreads();
    // as in the four-wavefront kernel: an even slab t sits in LDS buffer 0 while slab t+1 waits in register
    // set 1 and slab t+2 is requested into set 0; for the odd slab the roles are swapped
    for (int t = 0; t < nslab; t += 2) {
      if (t + 2 < nslab) LPC_GEMM8_FETCH(t + 2, ra0, rb0)
      LPC_GEMM8_CONSUME(0)
      if (t + 1 < nslab) LPC_GEMM8_STASH(1, ra1, rb1)
      __syncthreads();
      if (t + 1 < nslab) {
        if (t + 3 < nslab) LPC_GEMM8_FETCH(t + 3, ra1, rb1)
        LPC_GEMM8_CONSUME(1)
        if (t + 2 < nslab) LPC_GEMM8_STASH(0, ra0, rb0)
        __syncthreads();
      }
    }
#undef LPC_GEMM8_FETCH
#undef LPC_GEMM8_STASH
#undef LPC_GEMM8_CONSUME
  }
  float *C = g.C + bz * g.strideC;
  const float *mask = g.relu_mask ? g.relu_mask + bz * g.strideC : nullptr;
  const int col = n0 + wn + (lane & 31);
  const float bias = g.bias ? g.bias[bz * g.strideBias + col] : 0.0f;
#pragma unroll
  for (int v = 0; v < 16; ++v) {
    const int row = m0 + wm + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
    const int64_t off = (int64_t)row * g.ldc + col;
    float val = g.alpha * acc[v] + bias;
    if (g.relu) val = val > 0.0f ? val : 0.0f;
    if (mask) val = mask[off] > 0.0f ? val : 0.0f;
    if (g.accumulate) val += C[off];
    C[off] = val;
  }
}

// ---- outputs with at most 16 columns (the last layer of the MLP) -------------------------------------
// A 128-wide matrix-core tile would be 90 % padding and the long K loop of the few tiles is pure latency,
// so these products run on the vector units with B (at most K x 16) staged in LDS.
constexpr int kSkinnyN = 16;
constexpr int kSkinnyLdsFloats = 16384;  // 64 KB

__device__ __forceinline__ float skinny_store(const GemmArgs &g, float *C, int64_t bz, int row, int col, float acc) {
  const int64_t off = (int64_t)row * g.ldc + col;
  float val = g.alpha * acc + (g.bias ? g.bias[bz * g.strideBias + col] : 0.0f);
  if (g.relu) val = val > 0.0f ? val : 0.0f;
  if (g.relu_mask) val = g.relu_mask[off + (C - g.C)] > 0.0f ? val : 0.0f;
  if (g.accumulate) val += C[off];
  C[off] = val;
  return val;
}

// C = A*B, A [M][K] row-major.  A wavefront takes one row of A at a time (16 rows per workgroup): its lanes
// split K in groups of four, read B transposed from LDS (Bt[c][k], k contiguous) and close each of the N dot
// products with a wavefront reduction.  K is walked in chunks of kc <= kSkinnyLdsFloats / N rows of B.
__global__ __launch_bounds__(256) void gemm_skinny_nn_kernel(GemmArgs g, int kc) {
  touch_kernel_arguments<(int)(sizeof(GemmArgs))>();
  extern __shared__ float Bt[];  // [N][kc + 4]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t bz = blockIdx.y;
  const int pitch = kc + 4;
  const int row0 = blockIdx.x * 16;
  float acc[4][kSkinnyN];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < kSkinnyN; ++c) acc[r][c] = 0.0f;
  for (int s = 0; s < g.nseg; ++s) {
    const float *A = g.A[s] + bz * g.strideA[s];
    const float *B = g.B[s] + bz * g.strideB[s];
    for (int k0 = 0; k0 < g.K; k0 += kc) {
      const int kn = g.K - k0 < kc ? g.K - k0 : kc;
      __syncthreads();  // the previous chunk has been consumed
      for (int i0 = tid; i0 < kn * g.N; i0 += 8 * 256) {  // eight elements in flight per thread
        float t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int i = i0 + j * 256, k = i / g.N, c = i - k * g.N;
          t[j] = i < kn * g.N ? B[(int64_t)(k0 + k) * g.ldb[s] + c] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int i = i0 + j * 256, k = i / g.N, c = i - k * g.N;
          if (i < kn * g.N) Bt[c * pitch + k] = t[j];
        }
      }
      for (int i = tid; i < 4 * g.N; i += 256) Bt[(i >> 2) * pitch + kn + (i & 3)] = 0.0f;  // pad of the last group
      __syncthreads();
      for (int k = 4 * lane; k < kn; k += 256) {
        // the wavefront's four rows are requested together, then consumed
        float av[4][4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = row0 + wave * 4 + r;
          const float *a = A + (int64_t)(row < g.M ? row : g.M - 1) * g.lda[s] + k0;
#pragma unroll
          for (int j = 0; j < 4; ++j) av[r][j] = (row < g.M && k + j < kn) ? a[k + j] : 0.0f;
        }
#pragma unroll
        for (int c = 0; c < kSkinnyN; ++c) {
          if (c < g.N) {
            const float4 b = *reinterpret_cast<const float4 *>(&Bt[c * pitch + k]);
#pragma unroll
            for (int r = 0; r < 4; ++r)
              acc[r][c] = fmaf(av[r][0], b.x, fmaf(av[r][1], b.y, fmaf(av[r][2], b.z, fmaf(av[r][3], b.w, acc[r][c]))));
          }
        }
      }
    }
  }
  float *C = g.C + bz * g.strideC;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int row = row0 + wave * 4 + r;
#pragma unroll
    for (int c = 0; c < kSkinnyN; ++c) {
      if (c < g.N) {  // uniform
        const float t = wave_sum(acc[r][c]);
        if (lane == 0 && row < g.M) skinny_store(g, C, bz, row, c, t);
      }
    }
  }
}

// C = A'*B, A stored [K][M].  A wavefront owns 64 consecutive rows m of C (one per lane: the loads of A are
// coalesced along m); the four wavefronts of a workgroup split K and are combined through LDS in wavefront
// order.  B rows (N values, the same for every lane) come from LDS in chunks of kc rows.
__global__ __launch_bounds__(256) void gemm_skinny_tn_kernel(GemmArgs g, int kc) {
  touch_kernel_arguments<(int)(sizeof(GemmArgs))>();
  extern __shared__ float Bs[];  // [kc][16], then the reduction buffer [4][64][16]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t bz = blockIdx.y;
  const int m = blockIdx.x * 64 + lane;
  float acc[kSkinnyN];
#pragma unroll
  for (int c = 0; c < kSkinnyN; ++c) acc[c] = 0.0f;
  for (int s = 0; s < g.nseg; ++s) {
    const float *A = g.A[s] + bz * g.strideA[s];
    const float *B = g.B[s] + bz * g.strideB[s];
    for (int k0 = 0; k0 < g.K; k0 += kc) {
      const int kn = g.K - k0 < kc ? g.K - k0 : kc;
      __syncthreads();
      for (int i0 = tid; i0 < kn * kSkinnyN; i0 += 8 * 256) {  // eight elements in flight per thread
        float t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int i = i0 + j * 256, k = i >> 4, c = i & 15;
          t[j] = (i < kn * kSkinnyN && c < g.N) ? B[(int64_t)(k0 + k) * g.ldb[s] + c] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j)
          if (i0 + j * 256 < kn * kSkinnyN) Bs[i0 + j * 256] = t[j];
      }
      __syncthreads();
      if (m < g.M) {
        for (int k = wave; k < kn; k += 128) {
          // 32 rows of A in flight per step
          float a[32];
#pragma unroll
          for (int j = 0; j < 32; ++j) a[j] = k + 4 * j < kn ? A[(int64_t)(k0 + k + 4 * j) * g.lda[s] + m] : 0.0f;
#pragma unroll
          for (int j = 0; j < 32; ++j) {
            const int kk = k + 4 * j < kn ? k + 4 * j : 0;  // a[j] is zero past the end
            const float4 *b = reinterpret_cast<const float4 *>(&Bs[kk * kSkinnyN]);
            const float4 b0 = b[0], b1 = b[1], b2 = b[2], b3 = b[3];
            acc[0] = fmaf(a[j], b0.x, acc[0]); acc[1] = fmaf(a[j], b0.y, acc[1]);
            acc[2] = fmaf(a[j], b0.z, acc[2]); acc[3] = fmaf(a[j], b0.w, acc[3]);
            acc[4] = fmaf(a[j], b1.x, acc[4]); acc[5] = fmaf(a[j], b1.y, acc[5]);
            acc[6] = fmaf(a[j], b1.z, acc[6]); acc[7] = fmaf(a[j], b1.w, acc[7]);
            acc[8] = fmaf(a[j], b2.x, acc[8]); acc[9] = fmaf(a[j], b2.y, acc[9]);
            acc[10] = fmaf(a[j], b2.z, acc[10]); acc[11] = fmaf(a[j], b2.w, acc[11]);
            acc[12] = fmaf(a[j], b3.x, acc[12]); acc[13] = fmaf(a[j], b3.y, acc[13]);
            acc[14] = fmaf(a[j], b3.z, acc[14]); acc[15] = fmaf(a[j], b3.w, acc[15]);
          }
        }
      }
    }
  }
  __syncthreads();
  float *red = Bs;  // [4][64][16]
#pragma unroll
  for (int c = 0; c < kSkinnyN; ++c) red[(wave * 64 + lane) * kSkinnyN + c] = acc[c];
  __syncthreads();
  float *C = g.C + bz * g.strideC;
  for (int i = tid; i < 64 * kSkinnyN; i += 256) {
    const int l = i >> 4, c = i & 15, row = blockIdx.x * 64 + l;
    if (row < g.M && c < g.N) {
      const float t = ((red[(0 * 64 + l) * kSkinnyN + c] + red[(1 * 64 + l) * kSkinnyN + c]) +
                       red[(2 * 64 + l) * kSkinnyN + c]) + red[(3 * 64 + l) * kSkinnyN + c];
      skinny_store(g, C, bz, row, c, t);
    }
  }
}

}  // namespace

bool gemm_takes_matrix_cores(const GemmArgs &g) { return !(g.N <= kSkinnyN && !g.transB && g.M >= 64); }

int gemm_tiles(const GemmArgs &g) {
  return ((g.N + BN - 1) / BN) * ((g.M + BM - 1) / BM);
}

// whether launch_gemm takes gemm_skinny_tn_short_kernel, which can leave statistic partials like the matrix-core
// kernels (g.stat_part), and how many: one per workgroup of a batch item
bool gemm_takes_skinny_short(const GemmArgs &g) {
  return !gemm_takes_matrix_cores(g) && g.transA && g.K <= 128;
}
int gemm_skinny_short_slots(const GemmArgs &g) { return (g.M + 63) / 64; }

// The same product when K <= 128 (a worker's rows of one batch): every row of A and B that the workgroup needs
// is requested before anything is consumed, one round trip instead of one per operand and parameter set.
// Rows are taken in the order of gemm_skinny_tn_kernel, so the sums are the same to the bit.
__global__ __launch_bounds__(256) void gemm_skinny_tn_short_kernel(GemmArgs g) {
  touch_kernel_arguments<(int)(sizeof(GemmArgs))>();
  __shared__ __attribute__((aligned(16))) float Bs[2 * 128 * kSkinnyN];  // [segment][k][16], then [4][64][16]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t bz = blockIdx.y;
  const int m = blockIdx.x * 64 + lane;
  const int kn = g.K;
  float a[2][32];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const float *A = g.A[s < g.nseg ? s : 0] + bz * g.strideA[s < g.nseg ? s : 0];
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      const int k = wave + 4 * j;
      a[s][j] = (s < g.nseg && k < kn && m < g.M) ? A[(int64_t)k * g.lda[s < g.nseg ? s : 0] + m] : 0.0f;
    }
  }
  float t[2][8];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const float *B = g.B[s < g.nseg ? s : 0] + bz * g.strideB[s < g.nseg ? s : 0];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int i = tid + j * 256, k = i >> 4, c = i & 15;
      t[s][j] = (s < g.nseg && k < kn && c < g.N) ? B[(int64_t)k * g.ldb[s < g.nseg ? s : 0] + c] : 0.0f;
    }
  }
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int j = 0; j < 8; ++j) Bs[s * 128 * kSkinnyN + tid + j * 256] = t[s][j];
  __syncthreads();
  float acc[kSkinnyN];
#pragma unroll
  for (int c = 0; c < kSkinnyN; ++c) acc[c] = 0.0f;
#pragma unroll
  for (int s = 0; s < 2; ++s) {
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      // rows past K and the absent second segment hold zeros in a[][] and in Bs
      const float4 *b = reinterpret_cast<const float4 *>(&Bs[(s * 128 + wave + 4 * j) * kSkinnyN]);
      const float4 b0 = b[0], b1 = b[1], b2 = b[2], b3 = b[3];
      const float av = a[s][j];
      acc[0] = fmaf(av, b0.x, acc[0]); acc[1] = fmaf(av, b0.y, acc[1]);
      acc[2] = fmaf(av, b0.z, acc[2]); acc[3] = fmaf(av, b0.w, acc[3]);
      acc[4] = fmaf(av, b1.x, acc[4]); acc[5] = fmaf(av, b1.y, acc[5]);
      acc[6] = fmaf(av, b1.z, acc[6]); acc[7] = fmaf(av, b1.w, acc[7]);
      acc[8] = fmaf(av, b2.x, acc[8]); acc[9] = fmaf(av, b2.y, acc[9]);
      acc[10] = fmaf(av, b2.z, acc[10]); acc[11] = fmaf(av, b2.w, acc[11]);
      acc[12] = fmaf(av, b3.x, acc[12]); acc[13] = fmaf(av, b3.y, acc[13]);
      acc[14] = fmaf(av, b3.z, acc[14]); acc[15] = fmaf(av, b3.w, acc[15]);
    }
  }
  __syncthreads();
  float *red = Bs;  // [4][64][16]
#pragma unroll
  for (int c = 0; c < kSkinnyN; ++c) red[(wave * 64 + lane) * kSkinnyN + c] = acc[c];
  __syncthreads();
  float *C = g.C + bz * g.strideC;
  // g.stat_part: the workgroup also leaves the statistics of what it stores, as slot stat_slot0 + blockIdx.x
  float fmx = 0.0f;
  double ssum = 0.0, ssq = 0.0, sbad = 0.0;
  for (int i = tid; i < 64 * kSkinnyN; i += 256) {
    const int l = i >> 4, c = i & 15, row = blockIdx.x * 64 + l;
    if (row < g.M && c < g.N) {
      const float r = ((red[(0 * 64 + l) * kSkinnyN + c] + red[(1 * 64 + l) * kSkinnyN + c]) +
                       red[(2 * 64 + l) * kSkinnyN + c]) + red[(3 * 64 + l) * kSkinnyN + c];
      const float val = skinny_store(g, C, bz, row, c, r);
      if (isfinite(val)) {
        fmx = fmaxf(fmx, fabsf(val)); ssum += (double)val; ssq += (double)val * (double)val;
      } else {
        sbad += 1.0;
      }
    }
  }
  if (g.stat_part) {  // uniform
    __shared__ double stat_red[16];
    tile_statistics(g, stat_red, tid, bz, blockIdx.x, fmx, ssum, ssq, sbad);
  }
}

// Validates shapes on the host (every access in the kernel is guarded by M, N, K).
hipError_t launch_gemm(const GemmArgs &g, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0 || g.nseg < 1 || g.nseg > 2 || g.batch < 1) return hipErrorInvalidValue;
  if (!gemm_takes_matrix_cores(g)) {
    if (!g.transA) {
      int kc = kSkinnyLdsFloats / g.N - 4;
      kc = kc / 4 * 4;
      if (kc > g.K) kc = (g.K + 3) / 4 * 4;
      const size_t lds = (size_t)g.N * (kc + 4) * sizeof(float);
      hipLaunchKernelGGL(gemm_skinny_nn_kernel, dim3((unsigned)((g.M + 15) / 16), (unsigned)g.batch), dim3(256), lds, st,
                         g, kc);
    } else if (g.K <= 128) {
      hipLaunchKernelGGL(gemm_skinny_tn_short_kernel, dim3((unsigned)((g.M + 63) / 64), (unsigned)g.batch), dim3(256), 0,
                         st, g);
    } else {
      int kc = 768;  // 48 KB of B rows; the reduction buffer needs 16 KB
      if (kc > g.K) kc = g.K;
      const size_t floats = (size_t)kc * kSkinnyN > 4u * 64 * kSkinnyN ? (size_t)kc * kSkinnyN : 4u * 64 * kSkinnyN;
      hipLaunchKernelGGL(gemm_skinny_tn_kernel, dim3((unsigned)((g.M + 63) / 64), (unsigned)g.batch), dim3(256),
                         floats * sizeof(float), st, g, kc);
    }
    return hipGetLastError();
  }
  constexpr int tn = BN;
  const dim3 grid((unsigned)((g.N + tn - 1) / tn), (unsigned)((g.M + BM - 1) / BM), (unsigned)g.batch);
  // whole tiles and slabs, 16-byte aligned rows: the branch-free fetch
  bool full = g.M % BM == 0 && g.N % tn == 0 && g.K % BK == 0;
  for (int s = 0; s < g.nseg; ++s)
    full = full && g.lda[s] % 4 == 0 && g.ldb[s] % 4 == 0 && ((uintptr_t)g.A[s] & 15u) == 0 &&
           ((uintptr_t)g.B[s] & 15u) == 0 && g.strideA[s] % 4 == 0 && g.strideB[s] % 4 == 0;
#define LPC_GEMM_LAUNCH2(TA_, TB_, FULL_) \
  hipLaunchKernelGGL((gemm_mfma_kernel<TA_, TB_, BN, FULL_>), grid, dim3(256), 0, st, g)
  // at most one whole tile per CU: eight wavefronts per tile (measured: 6-30 % faster there, no gain
  // once two four-wavefront workgroups share a CU)
  const bool eight = full && (int64_t)grid.x * grid.y * grid.z <= 256 && !g.stat_part;
#define LPC_GEMM_LAUNCH(TA_, TB_)                                                                   \
  do {                                                                                              \
    if (eight) hipLaunchKernelGGL((gemm_mfma8_kernel<TA_, TB_>), grid, dim3(512), 0, st, g);        \
    else if (full) LPC_GEMM_LAUNCH2(TA_, TB_, true);                                                \
    else LPC_GEMM_LAUNCH2(TA_, TB_, false);                                                         \
  } while (0)
  if (!g.transA && !g.transB) LPC_GEMM_LAUNCH(false, false);
  else if (!g.transA && g.transB) LPC_GEMM_LAUNCH(false, true);
  else if (g.transA && !g.transB) LPC_GEMM_LAUNCH(true, false);
  else LPC_GEMM_LAUNCH(true, true);
#undef LPC_GEMM_LAUNCH
#undef LPC_GEMM_LAUNCH2
  return hipGetLastError();
}

}  // namespace lpc

// Declared in include/lpc.h among the measurement and test aids.
extern "C" lpc_status lpc_debug_gemm(const float *A, const float *B, float *C, int32_t M, int32_t N, int32_t K,
                                     int64_t lda, int64_t ldb, int64_t ldc, int32_t transA, int32_t transB,
                                     float alpha, const float *bias, int32_t relu, int32_t accumulate, void *stream) {
  if (!A || !B || !C) return LPC_ENULL;
  if (M <= 0 || N <= 0 || K <= 0) return LPC_ESHAPE;
  if (lda < (transA ? M : K) || ldb < (transB ? K : N) || ldc < N) return LPC_ESHAPE;
  lpc::GemmArgs g{};
  g.A[0] = A; g.B[0] = B; g.C = C; g.M = M; g.N = N; g.K = K; g.lda[0] = lda; g.ldb[0] = ldb; g.ldc = ldc;
  g.transA = transA; g.transB = transB; g.alpha = alpha; g.bias = bias; g.relu = relu; g.accumulate = accumulate;
  g.nseg = 1; g.batch = 1;
  return lpc::launch_gemm(g, (hipStream_t)stream) == hipSuccess ? LPC_OK : LPC_EDEVICE;
}
