// Evaluators beside the hot path (gfx950): the gradient-mapping metric of
// Sec. 3.3, the histogram of a packed message's codes and the optimal
// prefix-code size it implies (entropy coding of the messages, Sec. 6.1), and
// the left-hand side of Theorem 2's step-size conditions (eq. (6), (7)).
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

// Optimal prefix-code lengths: repeatedly join the two lightest subtrees; each join puts every leaf below it
// one level deeper.  Subtrees are kept in a min-heap of (weight, node); parents are recorded so that a leaf's
// length is its distance to the root.  A lone used symbol still needs one bit per occurrence.
uint64_t huffman_code_lengths(const uint64_t *counts, int32_t nsym, int32_t *lens) {
  using Item = std::pair<uint64_t, int32_t>;
  std::priority_queue<Item, std::vector<Item>, std::greater<Item>> heap;
  std::vector<int32_t> parent((size_t)nsym, -1);
  for (int32_t k = 0; k < nsym; ++k) {
    if (lens) lens[k] = 0;
    if (counts[k]) heap.push({counts[k], k});
  }
  if (heap.empty()) return 0;
  if (heap.size() == 1) {
    const Item only = heap.top();
    if (lens) lens[only.second] = 1;
    return only.first;
  }
  uint64_t total = 0;
  while (heap.size() > 1) {
    const Item a = heap.top(); heap.pop();
    const Item b = heap.top(); heap.pop();
    const int32_t node = (int32_t)parent.size();
    parent.push_back(-1);
    parent[(size_t)a.second] = node;
    parent[(size_t)b.second] = node;
    total += a.first + b.first;
    heap.push({a.first + b.first, node});
  }
  if (lens) {
    for (int32_t k = 0; k < nsym; ++k) {
      if (!counts[k]) continue;
      int32_t depth = 0;
      for (int32_t v = k; parent[(size_t)v] >= 0; v = parent[(size_t)v]) ++depth;
      lens[k] = depth;
    }
  }
  return total;
}

}  // namespace lpc
