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
#pragma unroll
  for (int off = kGroup / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kGroup);
  return v;
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

}  // namespace lpc
