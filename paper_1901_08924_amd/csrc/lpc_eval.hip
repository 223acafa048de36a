// Evaluators beside the hot path (gfx950): the gradient-mapping metric of
// Sec. 3.3, the histogram of a packed message's codes and the optimal
// prefix-code size it implies (entropy coding of the messages, Sec. 6.1), and
// the left-hand side of Theorem 2's step-size conditions (eq. (6), (7)), and the emission of the entropy-coded
// bit stream (canonical prefix code, codewords most significant bit first).
// None of these runs inside an epoch; they are written for clarity, with fp64
// accumulation in a fixed order.
#include <hip/hip_runtime.h>

#include <functional>
#include <queue>
#include <vector>

#include "lpc_device.h"
#include "lpc_internal.h"

namespace lpc {

namespace {

// |G_eta(w)|^2 with G_eta(w) = (w - prox_{eta h}(w - eta*grad))/eta, one workgroup, fixed summation order.
__global__ __launch_bounds__(1024) void gradient_mapping_kernel(const float *__restrict__ w,
                                                                const float *__restrict__ grad, int64_t d, double eta,
                                                                double l1, double l2, double *__restrict__ out) {
  __shared__ double red[16];
  const int tid = threadIdx.x;
  const double thr = eta * l1, shrink = 1.0 / (1.0 + eta * l2);
  double a = 0.0;
  for (int64_t j = tid; j < d; j += 1024) {
    const double x = (double)w[j];
    const double p = x - eta * (double)grad[j];
    const double mag = fabs(p) - thr;
    const double px = mag > 0.0 ? copysign(mag, p) * shrink : 0.0;
    const double g = (x - px) / eta;
    a += g * g;
  }
  a = wave_sum(a);
  if ((tid & 63) == 0) red[tid >> 6] = a;
  __syncthreads();
  if (tid == 0) {
    double t = 0.0;
    for (int k = 0; k < 16; ++k) t += red[k];
    *out = t;
  }
}

// total += sum_i n_clipped[i] (one thread; N is the number of workers)
__global__ void accumulate_clipped_kernel(const uint32_t *__restrict__ n_clipped, int32_t N,
                                          unsigned long long *__restrict__ total) {
  unsigned long long t = *total;
  for (int32_t i = 0; i < N; ++i) t += n_clipped[i];
  *total = t;
}

__global__ void zero_u64_kernel(unsigned long long *__restrict__ dst, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = 0ull;
}

// counts[code + 2^(b-1)] += 1 for the first d coordinates of one packed message.  A thread takes one
// 32-coordinate segment (b words).  Up to kLdsBins bins are privatised per workgroup.
constexpr int kLdsBins = 8192;

__global__ __launch_bounds__(256) void code_histogram_kernel(const uint32_t *__restrict__ words, int64_t d, int32_t b,
                                                             unsigned long long *__restrict__ counts) {
  __shared__ uint32_t bins[kLdsBins];
  const int nbins = 1 << b;
  const bool priv = nbins <= kLdsBins;
  if (priv) {
    for (int k = threadIdx.x; k < nbins; k += 256) bins[k] = 0u;
    __syncthreads();
  }
  const int64_t segs = (d + 31) / 32;
  const uint32_t mask = (1u << b) - 1u, bias = 1u << (b - 1);
  for (int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x; s < segs; s += (int64_t)gridDim.x * 256) {
    const uint32_t *seg = words + s * b;
    const int64_t left = d - s * 32;
    const int cnt = left < 32 ? (int)left : 32;
    for (int j = 0; j < cnt; ++j) {
      const int off = j * b, wi = off >> 5, sh = off & 31;
      uint32_t f = seg[wi] >> sh;
      if (sh + b > 32) f |= seg[wi + 1] << (32 - sh);   // wi+1 < b here: the last field ends at bit 32*b
      // two's complement field -> bin index: adding 2^(b-1) modulo 2^b maps -2^(b-1).. to 0..
      const uint32_t bin = ((f & mask) + bias) & mask;
      if (priv) atomicAdd(&bins[bin], 1u);
      else atomicAdd(&counts[bin], 1ull);
    }
  }
  if (priv) {
    __syncthreads();
    for (int k = threadIdx.x; k < nbins; k += 256)
      if (bins[k]) atomicAdd(&counts[k], (unsigned long long)bins[k]);
  }
}

}  // namespace

hipError_t launch_gradient_mapping(const lpc_ctx *c, const float *w, const float *grad, double eta, double *out,
                                   hipStream_t st) {
  hipLaunchKernelGGL(gradient_mapping_kernel, dim3(1), dim3(1024), 0, st, w, grad, c->d, eta,
                     (double)c->prob.lambda1, (double)c->prob.lambda2, out);
  return hipGetLastError();
}

namespace {

// symbol (bin index) of coordinate j of a 32-coordinate segment
__device__ __forceinline__ uint32_t segment_symbol(const uint32_t *seg, int j, int b, uint32_t mask, uint32_t bias) {
  const int off = j * b, wi = off >> 5, sh = off & 31;
  uint32_t f = seg[wi] >> sh;
  if (sh + b > 32) f |= seg[wi + 1] << (32 - sh);
  return ((f & mask) + bias) & mask;
}

// seg_bits[s] = encoded size of segment s; meta[1] != 0 if some coordinate's symbol has no codeword
__global__ __launch_bounds__(256) void huffman_measure_kernel(const uint32_t *__restrict__ words, int64_t d, int32_t b,
                                                              const HuffEntry *__restrict__ table,
                                                              uint32_t *__restrict__ seg_bits,
                                                              unsigned long long *__restrict__ meta) {
  const int64_t segs = (d + 31) / 32;
  const int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (s >= segs) return;
  const uint32_t mask = (1u << b) - 1u, bias = 1u << (b - 1);
  const int64_t left = d - s * 32;
  const int cnt = left < 32 ? (int)left : 32;
  uint32_t total = 0;
  bool bad = false;
  for (int j = 0; j < cnt; ++j) {
    const uint32_t len = table[segment_symbol(words + s * b, j, b, mask, bias)].len;
    bad = bad || len == 0;
    total += len;
  }
  seg_bits[s] = total;
  if (bad) atomicOr(&meta[1], 1ull);
}

// off[s] = sum of seg_bits[0..s), meta[0] = the total; one workgroup, each thread a contiguous share
__global__ __launch_bounds__(1024) void huffman_scan_kernel(const uint32_t *__restrict__ seg_bits, int64_t segs,
                                                            unsigned long long *__restrict__ off,
                                                            unsigned long long *__restrict__ meta) {
  __shared__ unsigned long long share[1024];
  const int tid = threadIdx.x;
  const int64_t per = (segs + 1023) / 1024;
  const int64_t lo = tid * per, hi = lo + per < segs ? lo + per : segs;
  unsigned long long mine = 0;
  for (int64_t s = lo; s < hi; ++s) mine += seg_bits[s];
  share[tid] = mine;
  __syncthreads();
  if (tid == 0) {
    unsigned long long run = 0;
    for (int k = 0; k < 1024; ++k) {
      const unsigned long long t = share[k];
      share[k] = run;
      run += t;
    }
    meta[0] = run;
  }
  __syncthreads();
  unsigned long long pos = share[tid];
  for (int64_t s = lo; s < hi; ++s) {
    off[s] = pos;
    pos += seg_bits[s];
  }
}

// A thread appends the codewords of its segment from stream position off[s] on.  Words shared with the
// neighbouring segments are merged with atomic ORs (the stream was zero-filled).
__global__ __launch_bounds__(256) void huffman_emit_kernel(const uint32_t *__restrict__ words, int64_t d, int32_t b,
                                                           const HuffEntry *__restrict__ table,
                                                           const unsigned long long *__restrict__ off,
                                                           uint32_t *__restrict__ out) {
  const int64_t segs = (d + 31) / 32;
  const int64_t s = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (s >= segs) return;
  const uint32_t mask = (1u << b) - 1u, bias = 1u << (b - 1);
  const int64_t left = d - s * 32;
  const int cnt = left < 32 ? (int)left : 32;
  const unsigned long long pos = off[s];
  int64_t wi = (int64_t)(pos >> 5);
  uint32_t filled = (uint32_t)(pos & 31ull);   // bits of out[wi] that belong to earlier segments
  unsigned long long acc = 0;
  for (int j = 0; j < cnt; ++j) {
    const HuffEntry e = table[segment_symbol(words + s * b, j, b, mask, bias)];
    acc |= (unsigned long long)e.rev << filled;   // filled <= 31, e.len <= 32
    filled += e.len;
    if (filled >= 32) {
      if ((uint32_t)acc) atomicOr(&out[wi], (uint32_t)acc);
      acc >>= 32;
      filled -= 32;
      ++wi;
    }
  }
  if ((uint32_t)acc) atomicOr(&out[wi], (uint32_t)acc);
}

}  // namespace

hipError_t launch_huffman_measure(const lpc_ctx *c, const uint32_t *words, hipStream_t st) {
  const int64_t segs = c->d_pad / 32;
  hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(64), 0, st, c->s.huff_meta, (int64_t)2);
  hipLaunchKernelGGL(huffman_measure_kernel, dim3((unsigned)((segs + 255) / 256)), dim3(256), 0, st, words, c->d,
                     c->cfg.bits, (const HuffEntry *)c->s.huff_table, c->s.huff_seg_bits, c->s.huff_meta);
  hipLaunchKernelGGL(huffman_scan_kernel, dim3(1), dim3(1024), 0, st, (const uint32_t *)c->s.huff_seg_bits, segs,
                     c->s.huff_off, c->s.huff_meta);
  return hipGetLastError();
}

hipError_t launch_huffman_emit(const lpc_ctx *c, const uint32_t *words, uint32_t *out, int64_t out_words,
                               hipStream_t st) {
  const int64_t segs = c->d_pad / 32;
  hipError_t e = launch_fill_u32(out, 0u, out_words, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(huffman_emit_kernel, dim3((unsigned)((segs + 255) / 256)), dim3(256), 0, st, words, c->d,
                     c->cfg.bits, (const HuffEntry *)c->s.huff_table, (const unsigned long long *)c->s.huff_off, out);
  return hipGetLastError();
}

// out[0] = sum of the n clip counts, out[1] = bits of the largest of the n scale factors (one workgroup, fixed order)
__global__ __launch_bounds__(256) void epoch_report_kernel(const float *__restrict__ delta,
                                                           const uint32_t *__restrict__ nclip, int64_t n,
                                                           unsigned long long *__restrict__ out) {
  __shared__ double sum_sh[4];
  __shared__ float max_sh[4];
  const int tid = threadIdx.x;
  double sum = 0.0;
  float mx = 0.0f;
  for (int64_t k = tid; k < n; k += 256) {
    sum += (double)nclip[k];
    mx = fmaxf(mx, delta[k]);
  }
  sum = wave_sum(sum);
  mx = wave_max(mx);
  if ((tid & 63) == 0) { sum_sh[tid >> 6] = sum; max_sh[tid >> 6] = mx; }
  __syncthreads();
  if (tid == 0) {
    out[0] = (unsigned long long)(((sum_sh[0] + sum_sh[1]) + sum_sh[2]) + sum_sh[3]);
    out[1] = (unsigned long long)__float_as_uint(fmaxf(fmaxf(max_sh[0], max_sh[1]), fmaxf(max_sh[2], max_sh[3])));
  }
}

hipError_t launch_epoch_report(const float *delta, const uint32_t *nclip, int64_t n, unsigned long long *out,
                               hipStream_t st) {
  hipLaunchKernelGGL(epoch_report_kernel, dim3(1), dim3(256), 0, st, delta, nclip, n, out);
  return hipGetLastError();
}

hipError_t launch_accumulate_clipped(const uint32_t *n_clipped, int32_t N, unsigned long long *total, hipStream_t st) {
  hipLaunchKernelGGL(accumulate_clipped_kernel, dim3(1), dim3(1), 0, st, n_clipped, N, total);
  return hipGetLastError();
}

hipError_t launch_code_histogram(const uint32_t *words, int64_t d, int32_t bits, uint64_t *counts, hipStream_t st) {
  const int64_t nbins = (int64_t)1 << bits;
  auto *cnt = reinterpret_cast<unsigned long long *>(counts);
  hipLaunchKernelGGL(zero_u64_kernel, dim3((unsigned)((nbins + 255) / 256)), dim3(256), 0, st, cnt, nbins);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || d <= 0) return e;
  const int64_t segs = (d + 31) / 32;
  int64_t wgs = (segs + 255) / 256;
  if (wgs > 512) wgs = 512;
  hipLaunchKernelGGL(code_histogram_kernel, dim3((unsigned)wgs), dim3(256), 0, st, words, d, bits, cnt);
  return hipGetLastError();
}

}  // namespace lpc
