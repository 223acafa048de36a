// ReLU multi-layer perceptron with softmax cross-entropy as an instance of
// eq. (1) (gfx950): the snapshot gradient of Alg. 1 step 4 and the workers'
// variance-reduced differences of Alg. 1 step 6 over the whole flattened
// parameter vector (one scale factor per worker, Sec. 3.2 last paragraph).
//
// Parameter vector: layer by layer, weight matrix [in][out] row-major, then the
// bias [out].  The contractions run on the matrix cores (lpc_gemm.hip), except a last layer of at most 16
// classes, which is a per-row kernel on the vector units (below):
//   forward        H_l = relu(H_{l-1} W_l + b_l)                (rows x in) (in x out)
//   data gradient  D_{l-1} = (D_l W_l') masked by H_{l-1} > 0   (rows x out) (out x in)
//   weight grad    G_l = H_{l-1}' D_l                           (in x rows) (rows x out)
// For the workers' differences the two parameter sets (x and the snapshot)
// share the sampled rows: both forward/backward passes run over all N*B rows
// at once (the weights are shared by the workers), the snapshot's deltas are
// produced negated, and each worker's difference of weight gradients is ONE
// contraction over its 2B stacked rows (for the first layer, whose input is the
// same for both sets, over B rows with the two deltas added first).
#include <hip/hip_runtime.h>

#include "lpc_device.h"
#include "lpc_internal.h"

namespace lpc {

namespace {

// rows of X (and labels) for positions [0, rows): position r belongs to worker worker_begin + r/B
__global__ void gather_rows_kernel(const float *__restrict__ X, int64_t ldx, const float *__restrict__ y, int64_t n,
                                   int32_t in0, StreamKey key, uint32_t tag, int32_t worker_begin, int32_t B,
                                   float *__restrict__ xb, float *__restrict__ yb) {
  const int r = blockIdx.x;
  const uint32_t worker = (tag == kTagShared) ? kSharedWorkerField : (uint32_t)(worker_begin + r / B);
  const int64_t src = sample_row(key, tag, worker, (uint32_t)(r % B), n);
  const float *xs = X + src * ldx;
  float *xd = xb + (int64_t)r * in0;
  // four requests in flight before the first store (4-byte stores: with 16-byte ones the copy was quicker and the
  // product that reads it 15 us slower)
  const int step = (int)blockDim.x;
  for (int j = threadIdx.x; j < in0; j += 4 * step) {
    float t[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) t[q] = j + q * step < in0 ? xs[j + q * step] : 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      if (j + q * step < in0) xd[j + q * step] = t[q];
  }
  if (threadIdx.x == 0) yb[r] = y[src];
}

// delta = sign * (softmax(logits) - onehot(label)); optionally the row's loss
__global__ void softmax_delta_kernel(const float *__restrict__ logits, const float *__restrict__ labels, int rows,
                                     int classes, float sign, float *__restrict__ delta,
                                     double *__restrict__ row_loss) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows) return;
  const float *z = logits + (int64_t)r * classes;
  float mx = z[0];
  for (int c = 1; c < classes; ++c) mx = fmaxf(mx, z[c]);
  float sum = 0.0f;
  for (int c = 0; c < classes; ++c) sum += expf(z[c] - mx);
  const int label = (int)labels[r];
  const float inv = 1.0f / sum;
  for (int c = 0; c < classes; ++c)
    delta[(int64_t)r * classes + c] = sign * (expf(z[c] - mx) * inv - (c == label ? 1.0f : 0.0f));
  if (row_loss) row_loss[r] = (double)(logf(sum) + mx - z[label]);
}

// The last layer as one launch per pass: logits = a*W + b, softmax cross-entropy delta, and the delta handed
// to the layer below, delta_prev = (a > 0) .* (delta * W').  With at most 16 classes W ([K][C]) fits LDS
// (transposed, Wt[c][k]) and everything is a per-row computation: a wavefront takes four rows at a time, lane l
// owns the activations k = 256*q + 4*l .. +3, one read of a column of W serves the four rows, the C dot products
// close with wavefront reductions, the softmax runs inside a row of 16 lanes (lane c holds class c), and the
// activations are still in registers when delta_prev needs their signs.  blockIdx.y selects the parameter set
// (set 1 = snapshot parameters, negated deltas).
constexpr int kLastMaxC = 16;
constexpr int kLastMaxK = 1024;
constexpr int kLastRows = 16;  // rows per workgroup

struct LastArgs {
  const float *a;       // [set][rows][lda]
  int64_t lda, a_set_stride;
  const float *W;       // parameters of the layer, set s at W + s*w_set_stride: weights [K][C] then bias [C]
  int64_t w_set_stride, bias_off;
  const float *labels;
  int rows, K, C;
  float *delta;         // [set][rows][C]
  int64_t d_set_stride;
  float *delta_prev;    // [set][rows][K] or nullptr
  int64_t dp_set_stride;
  double *row_loss;     // set 0 only, or nullptr
};

template <int R>
__global__ __launch_bounds__(64 * kLastRows / R) void last_layer_kernel(LastArgs g) {
  touch_kernel_arguments<(int)(sizeof(LastArgs))>();
  constexpr int kThreadsLast = 64 * kLastRows / R;
  extern __shared__ float Wt[];  // [C][K + 4], then bias [C]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int set = blockIdx.y;
  const int pitch = g.K + 4;
  const float *W = g.W + (int64_t)set * g.w_set_stride;
  float *bias = Wt + g.C * pitch;
  const float sign = set == 0 ? 1.0f : -1.0f;
  const int row0 = blockIdx.x * kLastRows + wave * R;
  const int lc = lane & 15;
  const float *a = g.a + (int64_t)set * g.a_set_stride;
  // this lane's activations of the wavefront's R rows (K <= 1024: at most four groups of four per row)
  float4 av[R][4];
#pragma unroll
  for (int r = 0; r < R; ++r)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int k = 256 * q + 4 * lane;
      av[r][q] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (row0 + r < g.rows && k < g.K) av[r][q] = *reinterpret_cast<const float4 *>(a + (int64_t)(row0 + r) * g.lda + k);
    }
  // W goes to LDS while the activations are on their way
  const uint32_t inv_c = (uint32_t)((0x100000000ull + (uint32_t)g.C - 1) / (uint32_t)g.C);
  constexpr int kStage = 20;  // elements in flight per thread
  for (int i0 = tid; i0 < g.K * g.C; i0 += kStage * kThreadsLast) {
    float t[kStage];
#pragma unroll
    for (int j = 0; j < kStage; ++j) t[j] = i0 + j * kThreadsLast < g.K * g.C ? W[i0 + j * kThreadsLast] : 0.0f;
#pragma unroll
    for (int j = 0; j < kStage; ++j) {
      // i / C by a multiply: exact for i < 2^16 and C <= 16 with the rounded-up reciprocal 2^32 / C
      const int i = i0 + j * kThreadsLast, k = (int)__umulhi((uint32_t)i, inv_c), c = i - k * g.C;
      if (i < g.K * g.C) Wt[c * pitch + k] = t[j];
    }
  }
  if (tid < g.C) bias[tid] = W[g.bias_off + tid];
  __syncthreads();
  // logits: one read of a column of W serves the wavefront's rows; lane (16j + c) keeps z[c] of each row
  float z[R];
#pragma unroll
  for (int r = 0; r < R; ++r) z[r] = -INFINITY;
#pragma unroll
  for (int c = 0; c < kLastMaxC; ++c) {
    if (c < g.C) {  // uniform
      float s[R];
#pragma unroll
      for (int r = 0; r < R; ++r) s[r] = 0.0f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int k = 256 * q + 4 * lane;
        if (k < g.K) {
          const float4 w4 = *reinterpret_cast<const float4 *>(&Wt[c * pitch + k]);
#pragma unroll
          for (int r = 0; r < R; ++r)
            s[r] = fmaf(av[r][q].x, w4.x, fmaf(av[r][q].y, w4.y, fmaf(av[r][q].z, w4.z, fmaf(av[r][q].w, w4.w, s[r]))));
        }
      }
      const float bc = bias[c];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const float t = wave_sum(s[r]) + bc;
        z[r] = lc == c ? t : z[r];
      }
    }
  }
  // softmax cross-entropy inside each row of 16 lanes (lanes c >= C hold -inf and contribute exp = 0)
  float dl[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int row = row0 + r < g.rows ? row0 + r : g.rows - 1;
    const float mx = row16_max(z[r]);
    const float e = lc < g.C ? expf(z[r] - mx) : 0.0f;
    const float sum = row16_sum(e);
    const int label = (int)g.labels[row];
    dl[r] = sign * (e * (1.0f / sum) - (lc == label ? 1.0f : 0.0f));
    if (row0 + r < g.rows) {
      if (lane < g.C) g.delta[(int64_t)set * g.d_set_stride + (int64_t)row * g.C + lane] = dl[r];
      if (set == 0 && g.row_loss) {
        const float zl = row16_sum(lc == label ? z[r] : 0.0f);  // uniform branch: whole rows of lanes are active
        if (lane == 0) g.row_loss[row] = (double)(logf(sum) + mx - zl);
      }
    }
  }
  if (g.delta_prev) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int k = 256 * q + 4 * lane;
      float4 o[R];
#pragma unroll
      for (int r = 0; r < R; ++r) o[r] = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int c = 0; c < kLastMaxC; ++c) {
        if (c < g.C) {
          float4 w4 = make_float4(0.f, 0.f, 0.f, 0.f);
          if (k < g.K) w4 = *reinterpret_cast<const float4 *>(&Wt[c * pitch + k]);
#pragma unroll
          for (int r = 0; r < R; ++r) {
            const float dc = read_lane(dl[r], c);
            o[r].x = fmaf(dc, w4.x, o[r].x); o[r].y = fmaf(dc, w4.y, o[r].y);
            o[r].z = fmaf(dc, w4.z, o[r].z); o[r].w = fmaf(dc, w4.w, o[r].w);
          }
        }
      }
#pragma unroll
      for (int r = 0; r < R; ++r) {
        if (row0 + r >= g.rows || k >= g.K) continue;
        float4 t = o[r];
        t.x = av[r][q].x > 0.0f ? t.x : 0.0f; t.y = av[r][q].y > 0.0f ? t.y : 0.0f;
        t.z = av[r][q].z > 0.0f ? t.z : 0.0f; t.w = av[r][q].w > 0.0f ? t.w : 0.0f;
        float *dp = g.delta_prev + (int64_t)set * g.dp_set_stride + (int64_t)(row0 + r) * g.K;
        *reinterpret_cast<float4 *>(dp + k) = t;
      }
    }
  }
}

// whether the fused last-layer launch applies: few classes, a previous layer of ReLU activations (or the
// inputs when the net has one layer) that one wavefront can hold, 16-byte aligned rows
bool last_layer_fused(int K, int C, int64_t lda, const float *a, int64_t a_stride) {
  return C <= kLastMaxC && K <= kLastMaxK && K % 4 == 0 && lda % 4 == 0 && a_stride % 4 == 0 &&
         (((uintptr_t)a) & 15u) == 0 && (int64_t)C * (K + 4) + C <= 16384;
}

// out[b][c] (+)= alpha * sum over the K rows of batch item b of (D0[row][c] + D1[row][c]).
// 64 columns per workgroup; the 4 waves take interleaved rows and are combined in wave order.
// sum_back: D0[row][c] also receives D0[row][c] + D1[row][c] (every element is read by exactly one thread).
__global__ __launch_bounds__(256) void colsum_kernel(float *__restrict__ D0, const float *__restrict__ D1, int K,
                                                     int cols, float alpha, int accumulate, float *__restrict__ out,
                                                     int64_t out_stride, int sum_back) {
  __shared__ float red[4][64];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + lane;
  const int b = blockIdx.y;
  float s = 0.0f;
  if (c < cols) {
    float *p0 = D0 + (int64_t)b * K * cols + c;
    const float *p1 = D1 ? D1 + (int64_t)b * K * cols + c : nullptr;
    for (int k = wv; k < K; k += 32) {  // eight rows of each set in flight per step
      float v0[8], v1[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const bool ok = k + 4 * j < K;
        v0[j] = ok ? p0[(int64_t)(k + 4 * j) * cols] : 0.0f;
        v1[j] = (ok && p1) ? p1[(int64_t)(k + 4 * j) * cols] : 0.0f;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float t = v0[j] + v1[j];
        s += t;
        if (sum_back && k + 4 * j < K) p0[(int64_t)(k + 4 * j) * cols] = t;
      }
    }
  }
  red[wv][lane] = s;
  __syncthreads();
  if (wv == 0 && c < cols) {
    const float t = ((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane];
    float *o = out + (int64_t)b * out_stride + c;
    *o = accumulate ? *o + alpha * t : alpha * t;
  }
}

// colsum_kernel for every layer of the worker pass in one launch (all deltas exist once the backward pass is
// through, and each of these launches is short enough to be bound by its launch): blockIdx.x runs over the
// layers' 64-column blocks, first[l] being layer l's first.  Same arithmetic per column as colsum_kernel.
constexpr int kColsumMaxLayers = 8;
struct ColsumLayers {
  float *D0[kColsumMaxLayers];
  const float *D1[kColsumMaxLayers];
  float *out[kColsumMaxLayers];
  int cols[kColsumMaxLayers], first[kColsumMaxLayers + 1], sum_back[kColsumMaxLayers];
  int n, K;
  float alpha;
  int64_t out_stride;
  // not null: block x of batch item b also leaves the statistics of its 64 sums (Sec. 3.2 needs those of u^i) as
  // slot stat_slot0 + x of the item's partials
  double *stat_part;
  int64_t stat_batch_stride;
  int32_t stat_slot0;
};

__global__ __launch_bounds__(256) void colsum_layers_kernel(ColsumLayers g) {
  __shared__ float red[4][64];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  int l = 0;
#pragma unroll
  for (int k = 1; k < kColsumMaxLayers; ++k)
    if (k < g.n && (int)blockIdx.x >= g.first[k]) l = k;
  // the layer's fields, selected without indexing the argument arrays by a run-time value
  float *D0 = g.D0[0], *out = g.out[0];
  const float *D1 = g.D1[0];
  int cols = g.cols[0], first = g.first[0], sum_back = g.sum_back[0];
#pragma unroll
  for (int k = 1; k < kColsumMaxLayers; ++k)
    if (k == l) { D0 = g.D0[k]; D1 = g.D1[k]; out = g.out[k]; cols = g.cols[k]; first = g.first[k]; sum_back = g.sum_back[k]; }
  const int c = ((int)blockIdx.x - first) * 64 + lane;
  const int b = blockIdx.y, K = g.K;
  float s = 0.0f;
  if (c < cols) {
    float *p0 = D0 + (int64_t)b * K * cols + c;
    const float *p1 = D1 + (int64_t)b * K * cols + c;
    for (int k = wv; k < K; k += 32) {  // eight rows of each set in flight per step
      float v0[8], v1[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const bool ok = k + 4 * j < K;
        v0[j] = ok ? p0[(int64_t)(k + 4 * j) * cols] : 0.0f;
        v1[j] = ok ? p1[(int64_t)(k + 4 * j) * cols] : 0.0f;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float t = v0[j] + v1[j];
        s += t;
        if (sum_back && k + 4 * j < K) p0[(int64_t)(k + 4 * j) * cols] = t;
      }
    }
  }
  red[wv][lane] = s;
  __syncthreads();
  if (wv == 0) {  // the whole wavefront
    float val = 0.0f;
    if (c < cols) {
      val = g.alpha * (((red[0][lane] + red[1][lane]) + red[2][lane]) + red[3][lane]);
      out[(int64_t)b * g.out_stride + c] = val;
    }
    if (g.stat_part) {  // uniform; a lane past the layer's columns holds 0, which adds nothing
      const bool fin = isfinite(val);
      const double a_w = (double)wave_max(fin ? fabsf(val) : 0.0f), s_w = wave_sum(fin ? (double)val : 0.0),
                   q_w = wave_sum(fin ? (double)val * (double)val : 0.0), b_w = wave_sum(fin ? 0.0 : 1.0);
      if (lane == 0) {
        double *p = g.stat_part + (int64_t)b * g.stat_batch_stride + ((int64_t)g.stat_slot0 + blockIdx.x) * 4;
        p[0] = a_w; p[1] = s_w; p[2] = q_w; p[3] = b_w;
      }
    }
  }
}

// out[j] (+)= alpha * (P[0][j] + P[1][j] + ... + P[nb-1][j]) for j < count, the partial vectors `stride` floats
// apart; summed in block order.  count and the pointers are multiples of four floats / 16 bytes.
__global__ __launch_bounds__(256) void fold_blocks_kernel(const float *__restrict__ P, int nb, int64_t stride,
                                                          int64_t count, float alpha, int accumulate,
                                                          float *__restrict__ out) {
  const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (4 * q >= count) return;
  float4 acc = *reinterpret_cast<const float4 *>(P + 4 * q);
  for (int b0 = 1; b0 < nb; b0 += 4) {  // up to four partial vectors in flight
    float4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
      v[j] = b0 + j < nb ? *reinterpret_cast<const float4 *>(P + (int64_t)(b0 + j) * stride + 4 * q)
                         : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int j = 0; j < 4; ++j) { acc.x += v[j].x; acc.y += v[j].y; acc.z += v[j].z; acc.w += v[j].w; }
  }
  float4 *o = reinterpret_cast<float4 *>(out + 4 * q);
  float4 r = make_float4(alpha * acc.x, alpha * acc.y, alpha * acc.z, alpha * acc.w);
  if (accumulate) { const float4 t = *o; r.x += t.x; r.y += t.y; r.z += t.z; r.w += t.w; }
  *o = r;
}

__global__ void sum_rows_loss_kernel(const double *__restrict__ row_loss, int rows, double scale, int accumulate,
                                     double *__restrict__ f_out) {
  __shared__ double red[4];
  const int tid = threadIdx.x;
  double acc = 0.0;
  for (int r = tid; r < rows; r += 256) acc += row_loss[r];
  acc = wave_sum(acc);
  if ((tid & 63) == 0) red[tid >> 6] = acc;
  __syncthreads();
  if (tid == 0) {
    const double t = (((red[0] + red[1]) + red[2]) + red[3]) * scale;
    *f_out = accumulate ? *f_out + t : t;
  }
}

__global__ void zero_tail_kernel(float *__restrict__ U, int64_t d, int64_t d_pad, int nvec) {
  const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t pad = d_pad - d;
  if (k < pad * nvec) U[(k / pad) * d_pad + d + (k % pad)] = 0.0f;
}

struct Net {
  int L;
  const int32_t *dims;
  const lpc_ctx *c;
  int64_t rows_cap;  // rows the activation buffers were sized for
  float *act(int l, int set) const { return c->s.mlp_act + c->mlp_act_off[l] + (int64_t)set * rows_cap * dims[l]; }
  float *del(int l, int set) const { return c->s.mlp_del + c->mlp_act_off[l] + (int64_t)set * rows_cap * dims[l]; }
};

// Forward pass of `rows` rows whose inputs start at in0 (leading dimension ld0) into activation sets
// 0..nsets-1: set s uses the parameters at W + s*wstride (one batched product per layer).
// input rows of the last layer and whether backward_data() computes that layer itself (fused launch)
struct LastIn {
  const float *a;
  int64_t lda, set_stride;
  bool fused;
};
LastIn last_layer_input(const Net &nn, const float *in0, int64_t ld0) {
  LastIn li;
  const int l = nn.L - 1;
  li.a = l == 0 ? in0 : nn.act(l, 0);
  li.lda = l == 0 ? ld0 : nn.dims[l];
  li.set_stride = l == 0 ? 0 : nn.rows_cap * nn.dims[l];
  li.fused = last_layer_fused(nn.dims[l], nn.dims[l + 1], li.lda, li.a, li.set_stride);
  return li;
}

hipError_t forward(const Net &nn, const float *W, int64_t wstride, int nsets, const float *in0, int64_t ld0, int rows,
                   hipStream_t st) {
  const bool skip_last = last_layer_input(nn, in0, ld0).fused;
  for (int l = 0; l < nn.L; ++l) {
    if (l == nn.L - 1 && skip_last) break;  // logits are formed inside the fused last-layer launch
    GemmArgs g{};
    g.A[0] = l == 0 ? in0 : nn.act(l, 0);
    g.lda[0] = l == 0 ? ld0 : nn.dims[l];
    g.strideA[0] = l == 0 ? 0 : nn.rows_cap * nn.dims[l];
    g.B[0] = W + nn.c->mlp_woff[l];
    g.ldb[0] = nn.dims[l + 1];
    g.strideB[0] = wstride;
    g.C = nn.act(l + 1, 0);
    g.ldc = nn.dims[l + 1];
    g.strideC = nn.rows_cap * nn.dims[l + 1];
    g.M = rows; g.N = nn.dims[l + 1]; g.K = nn.dims[l];
    g.alpha = 1.0f; g.bias = W + nn.c->mlp_boff[l]; g.strideBias = wstride; g.relu = (l + 1 < nn.L) ? 1 : 0;
    g.nseg = 1; g.batch = nsets;
    hipError_t e = launch_gemm(g, st);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// Deltas of every layer from the logits down for sets 0..nsets-1; set 1 (the snapshot parameters) gets
// negated deltas, so that the weight gradients of the two sets add up to the variance-reduced difference.
hipError_t backward_data(const Net &nn, const float *W, int64_t wstride, int nsets, const float *in0, int64_t ld0,
                         const float *labels, int rows, double *row_loss, hipStream_t st) {
  const int classes = nn.dims[nn.L];
  const LastIn li = last_layer_input(nn, in0, ld0);
  int first = nn.L - 1;  // highest layer whose input delta is still to be formed by a product
  if (li.fused) {
    LastArgs g{};
    const int l = nn.L - 1;
    g.a = li.a; g.lda = li.lda; g.a_set_stride = li.set_stride;
    g.W = W + nn.c->mlp_woff[l]; g.w_set_stride = wstride; g.bias_off = nn.c->mlp_boff[l] - nn.c->mlp_woff[l];
    g.labels = labels; g.rows = rows; g.K = nn.dims[l]; g.C = classes;
    g.delta = nn.del(nn.L, 0); g.d_set_stride = nn.rows_cap * classes;
    g.delta_prev = l >= 1 ? nn.del(l, 0) : nullptr; g.dp_set_stride = nn.rows_cap * nn.dims[l];
    g.row_loss = row_loss;
    const size_t lds = ((size_t)classes * (g.K + 4) + classes) * sizeof(float);
    constexpr int kRowsPerWave = 2;  // eight wavefronts per workgroup: 21.7 us per worker pass; four rows each 24.2, one row 29.6
    hipLaunchKernelGGL(last_layer_kernel<kRowsPerWave>,
                       dim3((unsigned)((rows + kLastRows - 1) / kLastRows), (unsigned)nsets),
                       dim3(64 * kLastRows / kRowsPerWave), lds, st, g);
    first = nn.L - 2;
  } else {
    for (int set = 0; set < nsets; ++set)
      hipLaunchKernelGGL(softmax_delta_kernel, dim3((unsigned)((rows + 127) / 128)), dim3(128), 0, st,
                         (const float *)nn.act(nn.L, set), labels, rows, classes, set == 0 ? 1.0f : -1.0f,
                         nn.del(nn.L, set), set == 0 ? row_loss : nullptr);
  }
  for (int l = first; l >= 1; --l) {
    GemmArgs g{};
    g.A[0] = nn.del(l + 1, 0); g.lda[0] = nn.dims[l + 1]; g.strideA[0] = nn.rows_cap * nn.dims[l + 1];
    g.B[0] = W + nn.c->mlp_woff[l]; g.ldb[0] = nn.dims[l + 1]; g.transB = 1;  // W_l is [in][out]; we need W_l'
    g.strideB[0] = wstride;
    g.C = nn.del(l, 0); g.ldc = nn.dims[l]; g.strideC = nn.rows_cap * nn.dims[l];
    g.M = rows; g.N = nn.dims[l]; g.K = nn.dims[l + 1];
    g.alpha = 1.0f; g.relu_mask = nn.act(l, 0);
    g.nseg = 1; g.batch = nsets;
    hipError_t e = launch_gemm(g, st);
    if (e != hipSuccess) return e;
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_mlp_clear_padding(const lpc_ctx *c, hipStream_t st) {
  if (c->d_pad == c->d) return hipSuccess;
  const int nvec = c->cfg.N + 1;
  const int64_t cnt = (c->d_pad - c->d) * nvec;
  hipLaunchKernelGGL(zero_tail_kernel, dim3((unsigned)((cnt + 63) / 64)), dim3(64), 0, st, c->s.U, c->d, c->d_pad, nvec);
  return hipGetLastError();
}

void mlp_plan(lpc_ctx *c) {
  const int L = c->prob.mlp_nlayers;
  const int32_t *dims = c->mlp_dims.data();
  c->mlp_rows = (int64_t)c->cfg.N * c->cfg.B;
  // the snapshot pass works through chunks of 2*mlp_cap rows: at least 8192, so that its products are large
  // enough to fill the chip
  c->mlp_cap = c->mlp_rows > 4096 ? c->mlp_rows : 4096;
  c->mlp_woff.assign(L, 0);
  c->mlp_boff.assign(L, 0);
  c->mlp_act_off.assign(L + 1, 0);
  int64_t off = 0, aoff = 0;
  for (int l = 0; l < L; ++l) {
    c->mlp_woff[l] = off; off += (int64_t)dims[l] * dims[l + 1];
    c->mlp_boff[l] = off; off += dims[l + 1];
  }
  for (int l = 1; l <= L; ++l) {
    c->mlp_act_off[l] = aoff;
    aoff += 2 * c->mlp_cap * dims[l];
    aoff = (aoff + 63) / 64 * 64;
  }
  c->mlp_act_floats = aoff;
  // partial sums of the snapshot pass's row blocks: per block the bias column sums of the widest layer and
  // the largest weight gradient that is formed on the vector units
  int64_t widest = 0, skinny = 0;
  for (int l = 0; l < L; ++l) {
    GemmArgs g{};
    g.M = dims[l]; g.N = dims[l + 1];
    if (dims[l + 1] > widest) widest = dims[l + 1];
    if (!gemm_takes_matrix_cores(g) && (int64_t)dims[l] * dims[l + 1] > skinny) skinny = (int64_t)dims[l] * dims[l + 1];
  }
  c->mlp_part_floats = (2 * c->mlp_cap / kSnapBlock + 1) * (widest + skinny);
}

// Alg. 1 step 4 for the MLP: mean gradient (and loss) over the first n_rows samples, in chunks of N*B rows.
hipError_t launch_mlp_full_grad(const lpc_ctx *c, const float *w, float *mu, double *f_out, int64_t n_rows,
                                hipStream_t st) {
  Net nn{c->prob.mlp_nlayers, c->mlp_dims.data(), c, c->mlp_cap};
  const float alpha = (float)(1.0 / (double)n_rows);
  const int64_t chunk = 2 * c->mlp_cap;  // both activation sets, back to back, hold one chunk
  for (int64_t r0 = 0; r0 < n_rows; r0 += chunk) {
    const int rows = (int)((n_rows - r0 < chunk) ? n_rows - r0 : chunk);
    const float *in0 = c->prob.X + r0 * c->prob.ldx;
    const float *labels = c->prob.y + r0;
    hipError_t e = forward(nn, w, 0, 1, in0, c->prob.ldx, rows, st);
    if (e != hipSuccess) return e;
    e = backward_data(nn, w, 0, 1, in0, c->prob.ldx, labels, rows, f_out ? c->s.mlp_loss : nullptr, st);
    if (e != hipSuccess) return e;
    if (f_out)
      hipLaunchKernelGGL(sum_rows_loss_kernel, dim3(1), dim3(256), 0, st, (const double *)c->s.mlp_loss, rows,
                         (double)alpha, r0 > 0 ? 1 : 0, f_out);
    if (!mu) continue;
    const int nb = rows / kSnapBlock, rest = rows - nb * kSnapBlock;  // whole blocks, then a ragged remainder
    for (int l = 0; l < nn.L; ++l) {
      const int in = nn.dims[l], out = nn.dims[l + 1];
      const float *a = l == 0 ? in0 : nn.act(l, 0);
      const int64_t lda = l == 0 ? c->prob.ldx : in;
      float *dl = nn.del(l + 1, 0);
      int acc = r0 > 0 ? 1 : 0;
      GemmArgs g{};
      g.A[0] = a; g.lda[0] = lda; g.transA = 1;
      g.B[0] = dl; g.ldb[0] = out;
      g.C = mu + c->mlp_woff[l]; g.ldc = out;
      g.M = in; g.N = out; g.K = rows;
      g.alpha = alpha; g.accumulate = acc; g.nseg = 1; g.batch = 1;
      float *part_b = c->s.mlp_part, *part_w = c->s.mlp_part + (int64_t)nb * out;
      const bool blocks = nb >= 2;
      // A product on the matrix cores over thousands of rows has few output tiles (in*out/128^2): cut the rows
      // into kSnapWide-row blocks whose products run side by side into the rows of U (free during this pass)
      // and are folded afterwards, so that every CU has tiles to work on.
      const int nw = rows / kSnapWide;
      const int64_t cnt = (int64_t)in * out;
      const bool wide = gemm_takes_matrix_cores(g) && nw >= 2 && rows % kSnapWide == 0 && nw <= c->cfg.N + 1 &&
                        cnt / (128 * 128) < 2 * c->cus && cnt % 4 == 0 && c->mlp_woff[l] % 4 == 0;
      if (wide) {
        GemmArgs h = g;
        h.K = kSnapWide; h.batch = nw; h.alpha = 1.0f; h.accumulate = 0;
        h.strideA[0] = (int64_t)kSnapWide * lda; h.strideB[0] = (int64_t)kSnapWide * out;
        h.C = c->s.U + c->mlp_woff[l]; h.strideC = c->d_pad;
        e = launch_gemm(h, st);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(fold_blocks_kernel, dim3((unsigned)((cnt / 4 + 255) / 256)), dim3(256), 0, st,
                           (const float *)(c->s.U + c->mlp_woff[l]), nw, c->d_pad, cnt, alpha, acc,
                           mu + c->mlp_woff[l]);
      } else if (blocks && !gemm_takes_matrix_cores(g)) {
        GemmArgs h = g;
        h.K = kSnapBlock; h.batch = nb; h.alpha = 1.0f; h.accumulate = 0;
        h.strideA[0] = (int64_t)kSnapBlock * lda; h.strideB[0] = (int64_t)kSnapBlock * out;
        h.C = part_w; h.strideC = (int64_t)in * out;
        e = launch_gemm(h, st);
        if (e != hipSuccess) return e;
        const int cols = in * out;
        hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((cols + 63) / 64), 1u), dim3(256), 0, st,
                           part_w, (const float *)nullptr, nb, cols, alpha, acc, mu + c->mlp_woff[l], (int64_t)0, 0);
        if (rest) {
          g.A[0] = a + (int64_t)nb * kSnapBlock * lda; g.B[0] = dl + (int64_t)nb * kSnapBlock * out;
          g.K = rest; g.accumulate = 1;
          e = launch_gemm(g, st);
        }
      } else {
        e = launch_gemm(g, st);
      }
      if (e != hipSuccess) return e;
      float *db = dl;
      int brows = rows;
      if (blocks) {
        hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((out + 63) / 64), (unsigned)nb), dim3(256), 0, st, dl,
                           (const float *)nullptr, kSnapBlock, out, 1.0f, 0, part_b, (int64_t)out, 0);
        hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((out + 63) / 64), 1u), dim3(256), 0, st,
                           part_b, (const float *)nullptr, nb, out, alpha, acc, mu + c->mlp_boff[l], (int64_t)0, 0);
        db = dl + (int64_t)nb * kSnapBlock * out; brows = rest; acc = 1;
      }
      if (brows)
        hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((out + 63) / 64), 1u), dim3(256), 0, st, db,
                           (const float *)nullptr, brows, out, alpha, acc, mu + c->mlp_boff[l], (int64_t)0, 0);
    }
  }
  return hipGetLastError();
}

// Alg. 1 step 6 for the MLP: u^i = grad f_{B_i}(w) - grad f_{B_i}(w_snap) for workers [worker_begin, worker_end)
// (or the one shared batch), written to consecutive rows of U (row stride d_pad).
hipError_t launch_mlp_vr_grad(const lpc_ctx *c, const float *w, const float *w_snap, StreamKey key, uint32_t tag,
                              int32_t worker_begin, int32_t worker_end, float *U, int stats_mode, double *stats_out,
                              int32_t *stat_slots_used, hipStream_t st) {
  Net nn{c->prob.mlp_nlayers, c->mlp_dims.data(), c, c->mlp_cap};
  const int nw = worker_end - worker_begin, B = c->cfg.B, rows = nw * B;
  const int in0 = nn.dims[0];
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)rows), dim3(256), 0, st, c->prob.X, c->prob.ldx, c->prob.y,
                     c->n, in0, key, tag, worker_begin, B, c->s.mlp_xb, c->s.mlp_yb);
  // both parameter sets ride in one batched product per layer: set 1 = the snapshot, addressed as set 0's device
  // address plus a signed distance.  The two vectors are separate allocations of one flat device address space,
  // so the distance is formed from the addresses as integers (both are 16-byte aligned: the ABI layer checks).
  const intptr_t wbytes = (intptr_t)w_snap - (intptr_t)w;
  if (wbytes % 16 != 0) return hipErrorInvalidValue;
  const int64_t wstride = (int64_t)(wbytes / (intptr_t)sizeof(float));
  hipError_t e = forward(nn, w, wstride, 2, c->s.mlp_xb, in0, rows, st);
  if (e != hipSuccess) return e;
  e = backward_data(nn, w, wstride, 2, c->s.mlp_xb, in0, c->s.mlp_yb, rows, nullptr, st);
  if (e != hipSuccess) return e;
  const float alpha = (float)(1.0 / (double)B);
  // Statistics of u^i (Sec. 3.2 needs |u|_inf before anything can be quantized): the kernels that write u^i leave
  // them as partials -- the matrix-core products one per output tile from their epilogues, the bias sums and the
  // short products on the vector units one per workgroup; only what other kernels write (deep nets' biases, long
  // products on the vector units) gets a small reduction of its own.  No extra pass over U.
  // bias: column sums of the two delta sets over the worker's rows; for the first layer, whose input rows are
  // the same for both sets, the pass also leaves the sum of the two deltas in set 0 (one contraction below).
  // One launch for all layers when the net has at most kColsumMaxLayers.
  const bool biases_at_once = nn.L <= kColsumMaxLayers;
  const bool want_stats = stats_mode != kStatsNone;
  const int32_t vec0 = (tag == kTagShared) ? c->cfg.N : worker_begin;
  int32_t slot = 0;
  StatRange ranges{};
  if (biases_at_once) {
    ColsumLayers cl{};
    cl.n = nn.L; cl.K = B; cl.alpha = alpha; cl.out_stride = c->d_pad;
    int blocks = 0;
    for (int l = 0; l < nn.L; ++l) {
      cl.D0[l] = nn.del(l + 1, 0); cl.D1[l] = nn.del(l + 1, 1); cl.out[l] = U + c->mlp_boff[l];
      cl.cols[l] = nn.dims[l + 1]; cl.sum_back[l] = l == 0 ? 1 : 0; cl.first[l] = blocks;
      blocks += (nn.dims[l + 1] + 63) / 64;
    }
    cl.first[nn.L] = blocks;
    if (want_stats) {  // the launch leaves the statistics of the bias entries it writes
      cl.stat_part = c->s.stat_part + (int64_t)vec0 * c->stat_slots * 4;
      cl.stat_batch_stride = (int64_t)c->stat_slots * 4;
      cl.stat_slot0 = slot;
      slot += blocks;
    }
    hipLaunchKernelGGL(colsum_layers_kernel, dim3((unsigned)blocks, (unsigned)nw), dim3(256), 0, st, cl);
  }
  for (int l = nn.L - 1; l >= 0; --l) {
    const int out = nn.dims[l + 1], in = nn.dims[l];
    if (!biases_at_once)
      hipLaunchKernelGGL(colsum_kernel, dim3((unsigned)((out + 63) / 64), (unsigned)nw), dim3(256), 0, st,
                         nn.del(l + 1, 0), (const float *)nn.del(l + 1, 1), B, out, alpha, 0, U + c->mlp_boff[l],
                         c->d_pad, l == 0 ? 1 : 0);
    GemmArgs g{};
    g.transA = 1;
    g.C = U + c->mlp_woff[l]; g.ldc = out; g.strideC = c->d_pad;
    g.M = in; g.N = out; g.K = B; g.alpha = alpha; g.batch = nw;
    if (l == 0) {
      // same input rows for both sets: the deltas were added by the bias pass above, contract once
      g.nseg = 1;
      g.A[0] = c->s.mlp_xb; g.lda[0] = in; g.strideA[0] = (int64_t)B * in;
      g.B[0] = nn.del(1, 0); g.ldb[0] = out; g.strideB[0] = (int64_t)B * out;
    } else {
      g.nseg = 2;
      for (int set = 0; set < 2; ++set) {
        g.A[set] = nn.act(l, set); g.lda[set] = in; g.strideA[set] = (int64_t)B * in;
        g.B[set] = nn.del(l + 1, set); g.ldb[set] = out; g.strideB[set] = (int64_t)B * out;
      }
    }
    if (want_stats) {
      if (!biases_at_once) { ranges.begin[ranges.n] = c->mlp_boff[l]; ranges.len[ranges.n] = out; ++ranges.n; }
      if (gemm_takes_matrix_cores(g) || gemm_takes_skinny_short(g)) {
        g.stat_part = c->s.stat_part + (int64_t)vec0 * c->stat_slots * 4;
        g.stat_batch_stride = (int64_t)c->stat_slots * 4;
        g.stat_slot0 = slot;
        slot += gemm_takes_matrix_cores(g) ? gemm_tiles(g) : gemm_skinny_short_slots(g);
      } else {
        ranges.begin[ranges.n] = c->mlp_woff[l]; ranges.len[ranges.n] = (int64_t)in * out; ++ranges.n;
      }
    }
    e = launch_gemm(g, st);
    if (e != hipSuccess) return e;
    if (want_stats && ranges.n >= 6) {  // deep nets: reduce the ranges collected so far (all written by now)
      e = launch_range_stats(c, U, c->d_pad, vec0, nw, ranges, slot, st);
      if (e != hipSuccess) return e;
      slot += ranges.n;
      ranges.n = 0;
    }
  }
  // the padding of the context's own U was cleared when the context was made and nothing writes it
  const bool own_u = U >= c->s.U && U < c->s.U + (int64_t)(c->cfg.N + 1) * c->d_pad;
  if (c->d_pad > c->d && !own_u) {
    const int64_t cnt = (c->d_pad - c->d) * nw;
    hipLaunchKernelGGL(zero_tail_kernel, dim3((unsigned)((cnt + 63) / 64)), dim3(64), 0, st, U, c->d, c->d_pad, nw);
  }
  if (want_stats) {
    e = launch_range_stats(c, U, c->d_pad, vec0, nw, ranges, slot, st);
    if (e != hipSuccess) return e;
    slot += ranges.n;
    if (slot > c->stat_slots) return hipErrorInvalidValue;  // cannot happen: a tile covers at least 64 coordinates
    if (stats_mode == kStatsFinal) {
      e = launch_finalize_stats(c, vec0, nw, slot, stats_out, st);
      if (e != hipSuccess) return e;
    }
    if (stat_slots_used) *stat_slots_used = slot;
  }
  return hipGetLastError();
}

}  // namespace lpc
