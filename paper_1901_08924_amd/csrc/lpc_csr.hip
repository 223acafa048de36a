// CSR generalised-linear-model passes (gfx950): the snapshot gradient of
// Alg. 1 step 4 and the workers' variance-reduced differences of Alg. 1 step 6
// for sparse rows.
//
// Sixteen lanes own one row at a time (a wavefront works on four rows at once):
// the row's (column, value) pairs are read as contiguous spans, w is gathered
// (it stays cache resident), the dot product is closed with a 16-lane
// butterfly, and the row is scattered back as coef * value into the gradient.
// A row costs three dependent memory round trips (row_ptr -> pairs -> w), so
// small groups keep many rows in flight per CU.
// Text-like data has Zipf-distributed column ids, so a handful of "head"
// columns receive most of the scatter: each workgroup accumulates the first
// kHead columns privately in LDS and writes them once as a partial row that is
// folded in a fixed order; only the rare tail columns use global float atomics.
#include <hip/hip_runtime.h>

#include "lpc_device.h"
#include "lpc_internal.h"

namespace lpc {

namespace {

constexpr int kThreads = 256;
constexpr int kGroup = 16;                     // lanes per row
constexpr int kGroups = kThreads / kGroup;     // rows in flight per workgroup

__device__ __forceinline__ float loss_slope(int32_t loss, float z, float y) {
  if (loss == LPC_LOSS_LOGISTIC) return -y / (1.0f + expf(y * z));
  return z - y;
}

__device__ __forceinline__ float loss_value(int32_t loss, float z, float y) {
  if (loss == LPC_LOSS_LOGISTIC) {
    const float t = -y * z;
    return t > 0.0f ? t + log1pf(expf(-t)) : log1pf(expf(t));
  }
  return 0.5f * (z - y) * (z - y);
}

struct CsrArgs {
  const int32_t *row_ptr;
  const int32_t *col_idx;
  const float *vals;
  const float *y;
  const float *w;
  const float *w_snap;
  const float *z_snap;
  float *z_out;
  float *tail;        // snapshot pass: d floats, zeroed; tail columns accumulate here
  float *part;        // snapshot pass: [workgroup][head] partial rows
  double *part_loss;  // snapshot pass
  float *U;           // worker pass: [N][d_pad], zeroed
  uint32_t *touched;  // sparse worker pass: [N][bitmap_words], one bit per 32-coordinate segment
  int64_t bitmap_words;
  int32_t parts, rows_per_part;  // sparse worker pass: workgroups per worker, sampled rows per workgroup
  int64_t n, d, d_pad, n_rows;
  int32_t head;       // columns [0, head) are privatised in LDS (snapshot pass)
  int32_t loss, want_loss;
  StreamKey key;
  uint32_t tag;
  int32_t worker_begin, B;
  float scale;
};

// sum over the 16 lanes of a group; every lane of the group returns it
__device__ __forceinline__ float group_sum(float v) {
  static_assert(kGroup == 16, "a group is one row of 16 lanes");
  return row16_sum(v);
}

// Snapshot pass.  Workgroup b takes rows [b*rows_per_wg, ...); group g of it every kGroups-th row.
__global__ __launch_bounds__(kThreads) void csr_full_kernel(CsrArgs a, int64_t rows_per_wg) {
  extern __shared__ float head_acc[];
  __shared__ double loss_red[kGroups];
  const int tid = threadIdx.x, gl = tid & (kGroup - 1), grp = tid / kGroup;
  for (int32_t j = tid; j < a.head; j += kThreads) head_acc[j] = 0.0f;
  __syncthreads();
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_wg;
  int64_t r1 = r0 + rows_per_wg;
  if (r1 > a.n_rows) r1 = a.n_rows;
  double loss_acc = 0.0;
  for (int64_t r = r0 + grp; r < r1; r += kGroups) {
    const int32_t lo = a.row_ptr[r], hi = a.row_ptr[r + 1];
    const float yr = a.y[r];
    float s = 0.0f;
    for (int32_t e = lo + gl; e < hi; e += kGroup) s = fmaf(a.vals[e], a.w[a.col_idx[e]], s);
    const float z = group_sum(s);
    const float coef = loss_slope(a.loss, z, yr);
    if (gl == 0) {
      if (a.z_out) a.z_out[r] = z;
      if (a.want_loss) loss_acc += (double)loss_value(a.loss, z, yr);
    }
    for (int32_t e = lo + gl; e < hi; e += kGroup) {
      const int32_t c = a.col_idx[e];
      const float g = coef * a.vals[e];
      if (c < a.head) atomicAdd(&head_acc[c], g);   // LDS
      else atomicAdd(&a.tail[c], g);                // rare columns
    }
  }
  __syncthreads();
  float *dst = a.part + (int64_t)blockIdx.x * a.head;
  for (int32_t j = tid; j < a.head; j += kThreads) dst[j] = head_acc[j];
  if (a.want_loss) {
    if (gl == 0) loss_red[grp] = loss_acc;
    __syncthreads();
    if (tid == 0) {
      double t = 0.0;
      for (int k = 0; k < kGroups; ++k) t += loss_red[k];
      a.part_loss[blockIdx.x] = t;
    }
  }
}

// mu[j] = scale * tail[j] for the tail columns (the head comes from the fold of the partial rows)
__global__ void csr_tail_kernel(const float *__restrict__ tail, float scale, int64_t head, int64_t d,
                                float *__restrict__ mu) {
  const int64_t j = head + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j < d) mu[j] = tail[j] * scale;
}

// Worker pass: sixteen lanes per sampled row, scatter into the worker's zeroed row of U.
template <bool CACHED>
__global__ __launch_bounds__(kThreads) void csr_vr_kernel(CsrArgs a, int32_t nworkers) {
  const int tid = threadIdx.x, gl = tid & (kGroup - 1), grp = tid / kGroup;
  const int64_t slot = (int64_t)blockIdx.x * kGroups + grp;   // (worker, position) pair
  if (slot >= (int64_t)nworkers * a.B) return;                // whole groups leave together
  const int32_t wrel = (int32_t)(slot / a.B), pos = (int32_t)(slot % a.B);
  const uint32_t worker = (a.tag == kTagShared) ? kSharedWorkerField : (uint32_t)(a.worker_begin + wrel);
  const int64_t r = sample_row(a.key, a.tag, worker, (uint32_t)pos, a.n);
  const int32_t lo = a.row_ptr[r], hi = a.row_ptr[r + 1];
  const float yr = a.y[r];
  float s = 0.0f, s2 = 0.0f;
  for (int32_t e = lo + gl; e < hi; e += kGroup) {
    const int32_t c = a.col_idx[e];
    const float v = a.vals[e];
    s = fmaf(v, a.w[c], s);
    if (!CACHED) s2 = fmaf(v, a.w_snap[c], s2);
  }
  const float z = group_sum(s);
  const float zs = CACHED ? a.z_snap[r] : group_sum(s2);
  const float coef = (loss_slope(a.loss, z, yr) - loss_slope(a.loss, zs, yr)) * a.scale;
  float *u = a.U + (int64_t)wrel * a.d_pad;
  for (int32_t e = lo + gl; e < hi; e += kGroup) atomicAdd(&u[a.col_idx[e]], coef * a.vals[e]);
}

// Worker pass that keeps u^i sparse.  A workgroup takes rows_per_part sampled rows of one worker, sixteen
// lanes per row.  Head columns accumulate in LDS and leave as one partial row per workgroup (a.part, folded by
// the statistics pass); a tail column is added to the worker's row of U, which is all zero outside the
// segments touched in this iteration, and its 32-coordinate segment is marked in the bitmap so that the
// statistics, quantizer and receiver passes visit only marked segments (an unmarked segment codes to zero).
constexpr int kSparseThreads = 1024;
constexpr int kSparseGroups = kSparseThreads / kGroup;

template <bool CACHED>
__global__ __launch_bounds__(kSparseThreads) void csr_vr_sparse_kernel(CsrArgs a) {
  extern __shared__ float head_acc[];
  const int tid = threadIdx.x, gl = tid & (kGroup - 1), grp = tid / kGroup;
  for (int32_t j = tid; j < a.head; j += kSparseThreads) head_acc[j] = 0.0f;
  __syncthreads();
  const int32_t wrel = blockIdx.x / a.parts, part = blockIdx.x % a.parts;
  const uint32_t worker = (uint32_t)(a.worker_begin + wrel);
  const int32_t pos0 = part * a.rows_per_part;
  const int32_t pos1 = pos0 + a.rows_per_part < a.B ? pos0 + a.rows_per_part : a.B;
  float *u = a.U + (int64_t)wrel * a.d_pad;
  uint32_t *bm = a.touched + (int64_t)wrel * a.bitmap_words;
  for (int32_t pos = pos0 + grp; pos < pos1; pos += kSparseGroups) {
    const int64_t r = sample_row(a.key, a.tag, worker, (uint32_t)pos, a.n);
    const int32_t lo = a.row_ptr[r], hi = a.row_ptr[r + 1];
    const float yr = a.y[r];
    const float zc = CACHED ? a.z_snap[r] : 0.0f;
    // 64 entries of the row per step, all loads of a step in flight together (most rows need one step)
    float s = 0.0f, s2 = 0.0f;
    int32_t c[4];
    float v[4];
    for (int32_t base = lo; base < hi; base += 4 * kGroup) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int32_t e = base + q * kGroup + gl;
        const bool ok = e < hi;
        c[q] = ok ? a.col_idx[e] : 0;
        v[q] = ok ? a.vals[e] : 0.0f;
      }
      float wv[4], wsv[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        wv[q] = a.w[c[q]];
        wsv[q] = CACHED ? 0.0f : a.w_snap[c[q]];
      }
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        s = fmaf(v[q], wv[q], s);
        if (!CACHED) s2 = fmaf(v[q], wsv[q], s2);
      }
    }
    const float z = group_sum(s);
    const float zs = CACHED ? zc : group_sum(s2);
    const float coef = (loss_slope(a.loss, z, yr) - loss_slope(a.loss, zs, yr)) * a.scale;
    const bool one_step = hi - lo <= 4 * kGroup;  // then c[], v[] still hold the whole row
    for (int32_t base = lo; base < hi; base += 4 * kGroup) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int32_t e = base + q * kGroup + gl;
        if (e >= hi) continue;
        const int32_t col = one_step ? c[q] : a.col_idx[e];
        const float g = coef * (one_step ? v[q] : a.vals[e]);
        if (col < a.head) {
          atomicAdd(&head_acc[col], g);
        } else {
          atomicAdd(&u[col], g);
          atomicOr(&bm[col >> 10], 1u << ((col >> 5) & 31));
        }
      }
    }
  }
  __syncthreads();
  float *dst = a.part + (int64_t)blockIdx.x * a.head;
  for (int32_t j = tid; j < a.head; j += kSparseThreads) dst[j] = head_acc[j];
}

__global__ void zero_kernel(float4 *__restrict__ dst, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n4) dst[i] = make_float4(0.f, 0.f, 0.f, 0.f);
}

}  // namespace

// 32 KB of LDS per workgroup.  Measured on the Zipf(1.1) design with d = 2^20: the global float atomics of
// the remaining tail columns (19 % of the entries) take about 70 % of the snapshot pass; the gathers of w and
// the LDS atomics are not the limit.
int csr_head_columns(int64_t d) { return (int)(d < 8192 ? d : 8192); }

int csr_full_grad_wgs(int64_t n) {
  int64_t wgs = 1024;  // 4 resident workgroups per CU (LDS)
  const int64_t by_rows = (n + 63) / 64;
  if (wgs > by_rows) wgs = by_rows;
  if (wgs >= 32) wgs = wgs / 16 * 16;
  return (int)(wgs < 1 ? 1 : wgs);
}

hipError_t launch_zero(float *dst, int64_t n, hipStream_t st) {
  // n is a multiple of 4 and dst is 16-byte aligned at every call site
  const int64_t n4 = n / 4;
  hipLaunchKernelGGL(zero_kernel, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0, st,
                     reinterpret_cast<float4 *>(dst), n4);
  return hipGetLastError();
}

hipError_t launch_csr_full_grad(const lpc_ctx *c, const float *w, float *mu, float *z, bool want_loss, int64_t n_rows,
                                hipStream_t st) {
  CsrArgs a{};
  a.row_ptr = c->prob.row_ptr; a.col_idx = c->prob.col_idx; a.vals = c->prob.vals; a.y = c->prob.y;
  a.w = w; a.z_out = z; a.tail = c->s.csr_tail; a.part = c->s.part; a.part_loss = c->s.part_loss;
  a.n = c->n; a.d = c->d; a.d_pad = c->d_pad; a.n_rows = n_rows;
  a.head = csr_head_columns(c->d); a.loss = c->prob.loss; a.want_loss = want_loss ? 1 : 0;
  const int wgs = c->full_grad_wgs;
  const int64_t rpw = (n_rows + wgs - 1) / wgs;
  hipError_t e = launch_zero(c->s.csr_tail, c->d_pad, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(csr_full_kernel, dim3((unsigned)wgs), dim3(kThreads), (size_t)a.head * sizeof(float), st, a,
                     rpw);
  e = hipGetLastError();
  if (e != hipSuccess || !mu) return e;
  if (c->d > a.head) {
    const int64_t tail_n = c->d - a.head;
    hipLaunchKernelGGL(csr_tail_kernel, dim3((unsigned)((tail_n + 255) / 256)), dim3(256), 0, st,
                       (const float *)c->s.csr_tail, (float)(1.0 / (double)n_rows), (int64_t)a.head, c->d, mu);
  }
  return hipGetLastError();
}

hipError_t launch_csr_vr_grad(const lpc_ctx *c, const float *w, const float *w_snap, const float *z_snap,
                              StreamKey key, uint32_t tag, int32_t worker_begin, int32_t worker_end, float *U,
                              hipStream_t st) {
  CsrArgs a{};
  a.row_ptr = c->prob.row_ptr; a.col_idx = c->prob.col_idx; a.vals = c->prob.vals; a.y = c->prob.y;
  a.w = w; a.w_snap = w_snap; a.z_snap = z_snap; a.U = U;
  a.n = c->n; a.d = c->d; a.d_pad = c->d_pad; a.loss = c->prob.loss;
  a.key = key; a.tag = tag; a.worker_begin = worker_begin; a.B = c->cfg.B;
  a.scale = (float)(1.0 / (double)c->cfg.B);
  const int32_t nworkers = worker_end - worker_begin;
  hipError_t e = launch_zero(U, (int64_t)nworkers * c->d_pad, st);
  if (e != hipSuccess) return e;
  const int64_t slots = (int64_t)nworkers * c->cfg.B;
  const dim3 grid((unsigned)((slots + kGroups - 1) / kGroups));
  if (z_snap) hipLaunchKernelGGL(csr_vr_kernel<true>, grid, dim3(kThreads), 0, st, a, nworkers);
  else hipLaunchKernelGGL(csr_vr_kernel<false>, grid, dim3(kThreads), 0, st, a, nworkers);
  return hipGetLastError();
}

// Sparse worker pass (all N workers).  s.U rows and the bitmap must be zero outside what this call adds.
int csr_sparse_parts(int32_t B) { return (B + kSparseGroups - 1) / kSparseGroups; }

hipError_t launch_csr_vr_sparse(const lpc_ctx *c, const float *w, const float *w_snap, const float *z_snap,
                                StreamKey key, hipStream_t st) {
  CsrArgs a{};
  a.row_ptr = c->prob.row_ptr; a.col_idx = c->prob.col_idx; a.vals = c->prob.vals; a.y = c->prob.y;
  a.w = w; a.w_snap = w_snap; a.z_snap = z_snap; a.U = c->s.U; a.part = c->s.part;
  a.touched = c->s.touched; a.bitmap_words = c->bitmap_words;
  a.n = c->n; a.d = c->d; a.d_pad = c->d_pad; a.loss = c->prob.loss;
  a.head = c->sparse_head;
  a.key = key; a.tag = kTagBatch; a.worker_begin = 0; a.B = c->cfg.B;
  a.scale = (float)(1.0 / (double)c->cfg.B);
  a.parts = csr_sparse_parts(c->cfg.B);
  a.rows_per_part = (c->cfg.B + a.parts - 1) / a.parts;
  const dim3 grid((unsigned)(c->cfg.N * a.parts));
  const size_t lds = (size_t)a.head * sizeof(float);
  if (z_snap) hipLaunchKernelGGL(csr_vr_sparse_kernel<true>, grid, dim3(kSparseThreads), lds, st, a);
  else hipLaunchKernelGGL(csr_vr_sparse_kernel<false>, grid, dim3(kSparseThreads), lds, st, a);
  return hipGetLastError();
}

}  // namespace lpc
