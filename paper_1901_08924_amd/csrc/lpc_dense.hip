// Dense generalised-linear-model passes (gfx950): the snapshot gradient of
// Alg. 1 step 4 and the workers' variance-reduced differences of Alg. 1 step 6.
//
// Both are "GEMV pairs": z = x_r'w per row, then g += c_r * x_r.  They are
// HBM-bound (about one flop per byte), so the kernels are built around reading
// every row of X exactly once: a workgroup keeps R rows in registers between
// the dot product and the scaled accumulation.  Thread t of a workgroup of T
// threads owns the columns {(k*T + t)*VEC + v}, so every global load
// instruction of the workgroup covers one contiguous T*VEC*4-byte span of a
// row.  The per-row dot products are reduced with wavefront butterflies and one
// LDS exchange per R rows (double-buffered, one barrier per group).  Each
// workgroup writes its d-long partial gradient once; a second small kernel adds
// the partials in a fixed order, which keeps results independent of scheduling.
#include <hip/hip_runtime.h>

#include "lpc_device.h"
#include "lpc_internal.h"

namespace lpc {

namespace {

struct DenseArgs {
  const float *X;
  int64_t ldx, d, n;
  const float *y;
  const float *w;
  const float *w_snap;  // worker pass without cached margins
  const float *z_snap;  // cached margins X*w_snap or nullptr
  float *z_out;         // snapshot pass: margins (may be nullptr)
  float *part;          // [workgroup][d]
  double *part_loss;    // snapshot pass: per-workgroup loss
  int64_t rows_per_wg;  // snapshot pass
  int64_t n_rows;       // snapshot pass
  int32_t loss;
  int32_t want_loss;
  int32_t stream_loads;
  // worker pass
  StreamKey key;
  uint32_t tag;
  int32_t worker_begin;
  int32_t B, parts, rows_per_part;
  int32_t shared_rel;  // relative worker index that draws the shared batch J instead (-1: none)
};

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

template <int VEC>
struct Chunk {
  float v[VEC];
};

template <int VEC>
__device__ __forceinline__ Chunk<VEC> load_chunk(const float *p) {
  Chunk<VEC> c;
  if constexpr (VEC == 4) {
    const float4 t = *reinterpret_cast<const float4 *>(p);
    c.v[0] = t.x; c.v[1] = t.y; c.v[2] = t.z; c.v[3] = t.w;
  } else {
    c.v[0] = *p;
  }
  return c;
}

// streamed-once data: non-temporal loads keep it from displacing what the caches should hold
typedef float floatx4 __attribute__((ext_vector_type(4)));
template <int VEC>
__device__ __forceinline__ Chunk<VEC> load_chunk_stream(const float *p) {
  Chunk<VEC> c;
  if constexpr (VEC == 4) {
    const floatx4 t = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(p));
    c.v[0] = t.x; c.v[1] = t.y; c.v[2] = t.z; c.v[3] = t.w;
  } else {
    c.v[0] = __builtin_nontemporal_load(p);
  }
  return c;
}

template <int VEC>
__device__ __forceinline__ void store_chunk(float *p, const Chunk<VEC> &c) {
  if constexpr (VEC == 4) {
    *reinterpret_cast<float4 *>(p) = make_float4(c.v[0], c.v[1], c.v[2], c.v[3]);
  } else {
    *p = c.v[0];
  }
}

// MODE 0: snapshot pass over contiguous rows.  MODE 1: worker pass over sampled rows with cached
// snapshot margins.  MODE 2: worker pass that recomputes the snapshot margins (two dot products).
template <int VEC, int K, int T, int R, int MODE>
__global__ __launch_bounds__(T) void dense_rows_kernel(DenseArgs a) {
  constexpr int NW = T / 64;
  constexpr int NDOT = (MODE == 2) ? 2 : 1;
  __shared__ float red[2][NW][R * NDOT];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;

  // columns owned by this thread and the matching slices of w (and w_snap)
  bool live[K];
  Chunk<VEC> wreg[K], wsreg[(MODE == 2) ? K : 1], acc[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int64_t col = ((int64_t)k * T + tid) * VEC;
    live[k] = col < a.d;
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[k].v[v] = 0.0f;
    if (live[k]) {
      wreg[k] = load_chunk<VEC>(a.w + col);
      if constexpr (MODE == 2) wsreg[k] = load_chunk<VEC>(a.w_snap + col);
    } else {
#pragma unroll
      for (int v = 0; v < VEC; ++v) wreg[k].v[v] = 0.0f;
      if constexpr (MODE == 2) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) wsreg[k].v[v] = 0.0f;
      }
    }
  }

  int64_t pos_begin, pos_end;
  uint32_t worker = 0, tag = a.tag;
  if constexpr (MODE == 0) {
    pos_begin = (int64_t)blockIdx.x * a.rows_per_wg;
    pos_end = pos_begin + a.rows_per_wg;
    if (pos_end > a.n_rows) pos_end = a.n_rows;
  } else {
    const int32_t wrel = blockIdx.x / a.parts, part = blockIdx.x % a.parts;
    if (wrel == a.shared_rel) tag = kTagShared;
    worker = (tag == kTagShared) ? kSharedWorkerField : (uint32_t)(a.worker_begin + wrel);
    pos_begin = (int64_t)part * a.rows_per_part;
    pos_end = pos_begin + a.rows_per_part;
    if (pos_end > a.B) pos_end = a.B;
  }

  double loss_acc = 0.0;
  int buf = 0;
  for (int64_t g0 = pos_begin; g0 < pos_end; g0 += R) {
    int64_t row[R];
    bool rowlive[R];
    Chunk<VEC> x[R][K];
    float dot[R * NDOT];
    float yv[R], zsv[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
      rowlive[r] = g0 + r < pos_end;
      if constexpr (MODE == 0) {
        row[r] = g0 + r;
      } else {
        row[r] = rowlive[r] ? sample_row(a.key, tag, worker, (uint32_t)(g0 + r), a.n) : 0;
      }
      // labels and cached margins are requested together with the rows, not after the reduction
      yv[r] = rowlive[r] ? a.y[row[r]] : 0.0f;
      zsv[r] = (MODE == 1 && rowlive[r]) ? a.z_snap[row[r]] : 0.0f;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const float *xr = a.X + row[r] * a.ldx;
#pragma unroll
      for (int k = 0; k < K; ++k) {
        if (rowlive[r] && live[k]) {
          if (MODE == 0 && a.stream_loads)
            x[r][k] = load_chunk_stream<VEC>(xr + ((int64_t)k * T + tid) * VEC);
          else
            x[r][k] = load_chunk<VEC>(xr + ((int64_t)k * T + tid) * VEC);
        } else {
#pragma unroll
          for (int v = 0; v < VEC; ++v) x[r][k].v[v] = 0.0f;
        }
      }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float s = 0.0f, s2 = 0.0f;
#pragma unroll
      for (int k = 0; k < K; ++k) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
          s = fmaf(x[r][k].v[v], wreg[k].v[v], s);
          if constexpr (MODE == 2) s2 = fmaf(x[r][k].v[v], wsreg[k].v[v], s2);
        }
      }
      dot[r * NDOT] = wave_sum(s);
      if constexpr (MODE == 2) dot[r * NDOT + 1] = wave_sum(s2);
    }
    if constexpr (NW > 1) {
      if (lane == 0) {
#pragma unroll
        for (int i = 0; i < R * NDOT; ++i) red[buf][wv][i] = dot[i];
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < R * NDOT; ++i) {
        float t = red[buf][0][i];
#pragma unroll
        for (int q = 1; q < NW; ++q) t += red[buf][q][i];
        dot[i] = t;
      }
      buf ^= 1;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
      float coef = 0.0f;
      if (rowlive[r]) {
        const float yr = yv[r];
        const float z = dot[r * NDOT];
        if constexpr (MODE == 0) {
          coef = loss_slope(a.loss, z, yr);
          if (tid == 0) {
            if (a.z_out) a.z_out[row[r]] = z;
            if (a.want_loss) loss_acc += (double)loss_value(a.loss, z, yr);
          }
        } else {
          const float zs = (MODE == 2) ? dot[r * NDOT + (NDOT - 1)] : zsv[r];
          coef = loss_slope(a.loss, z, yr) - loss_slope(a.loss, zs, yr);
        }
      }
#pragma unroll
      for (int k = 0; k < K; ++k) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[k].v[v] = fmaf(coef, x[r][k].v[v], acc[k].v[v]);
      }
    }
  }

  float *dst = a.part + (int64_t)blockIdx.x * a.d;
#pragma unroll
  for (int k = 0; k < K; ++k) {
    if (live[k]) store_chunk<VEC>(dst + ((int64_t)k * T + tid) * VEC, acc[k]);
  }
  if constexpr (MODE == 0) {
    if (tid == 0 && a.want_loss) a.part_loss[blockIdx.x] = loss_acc;
  }
}

struct Shape {
  int vec, k, t;
};

// choose the thread/column tiling: T threads, K chunks of VEC floats per thread, T*K*VEC >= d
bool pick_shape(int64_t d, int64_t ldx, const void *X, Shape *s) {
  const bool vec4 = (d % 4 == 0) && (ldx % 4 == 0) && (((uintptr_t)X & 15u) == 0);
  const int vec = vec4 ? 4 : 1;
  const int64_t chunks = (d + vec - 1) / vec;
  static const int table[][2] = {{64, 1}, {64, 4}, {256, 2}, {256, 4}, {512, 4}, {1024, 4}, {1024, 8}};
  for (const auto &e : table) {
    if ((int64_t)e[0] * e[1] >= chunks) {
      s->vec = vec; s->t = e[0]; s->k = e[1];
      return true;
    }
  }
  return false;
}

// R rows are held in registers at once; the caller asks for rows_hint rows per group and gets the
// largest instantiated R that does not exceed it (and fits the register budget of the tiling).
template <int VEC, int K, int T, int MODE>
void launch_shape(const DenseArgs &a, int grid, int rows_hint, hipStream_t st) {
  constexpr int RMAX = (K >= 8) ? 1 : ((K * VEC >= 16 && MODE == 2) ? 2 : 4);
  if (RMAX >= 4 && rows_hint >= 4) {
    LPC_LAUNCH_TIMED((dense_rows_kernel<VEC, K, T, (RMAX >= 4 ? 4 : RMAX), MODE>), dim3((unsigned)grid), dim3(T), st, a);
  } else if (RMAX >= 2 && rows_hint >= 2) {
    LPC_LAUNCH_TIMED((dense_rows_kernel<VEC, K, T, (RMAX >= 2 ? 2 : RMAX), MODE>), dim3((unsigned)grid), dim3(T), st, a);
  } else {
    LPC_LAUNCH_TIMED((dense_rows_kernel<VEC, K, T, 1, MODE>), dim3((unsigned)grid), dim3(T), st, a);
  }
}

template <int VEC, int MODE>
hipError_t dispatch_tk(const Shape &s, const DenseArgs &a, int grid, int rows_hint, hipStream_t st) {
  if (s.t == 64 && s.k == 1) launch_shape<VEC, 1, 64, MODE>(a, grid, rows_hint, st);
  else if (s.t == 64 && s.k == 4) launch_shape<VEC, 4, 64, MODE>(a, grid, rows_hint, st);
  else if (s.t == 256 && s.k == 2) launch_shape<VEC, 2, 256, MODE>(a, grid, rows_hint, st);
  else if (s.t == 256 && s.k == 4) launch_shape<VEC, 4, 256, MODE>(a, grid, rows_hint, st);
  else if (s.t == 512 && s.k == 2 && MODE != 0) launch_shape<VEC, 2, 512, (MODE != 0 ? MODE : 1)>(a, grid, rows_hint, st);
  else if (s.t == 512 && s.k == 4) launch_shape<VEC, 4, 512, MODE>(a, grid, rows_hint, st);
  else if (s.t == 1024 && s.k == 4) launch_shape<VEC, 4, 1024, MODE>(a, grid, rows_hint, st);
  else if (s.t == 1024 && s.k == 8) launch_shape<VEC, 8, 1024, MODE>(a, grid, rows_hint, st);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

template <int MODE>
hipError_t dispatch(const Shape &s, const DenseArgs &a, int grid, int rows_hint, hipStream_t st) {
  return s.vec == 4 ? dispatch_tk<4, MODE>(s, a, grid, rows_hint, st) : dispatch_tk<1, MODE>(s, a, grid, rows_hint, st);
}

int rows_per_group(const Shape &s) { return s.k >= 8 ? 1 : 4; }

}  // namespace

bool dense_supported(int64_t d, int64_t ldx, const void *X) {
  Shape s;
  return pick_shape(d, ldx, X, &s);
}

// Workgroups of the snapshot pass: enough to keep every CU busy with several
// resident groups, few enough that the partial-gradient rows stay a small
// fraction of the traffic of X.
// Measured on MI355X: the pass streams fastest with about 64 KB of rows in flight per workgroup and
// about 128 KB per CU (two such workgroups); more resident workgroups lower the achieved bandwidth.
int snapshot_rows_in_flight(int64_t d) {
  const int64_t r = 65536 / (4 * d);
  return r >= 4 ? 4 : (r >= 2 ? 2 : 1);
}

int dense_full_grad_wgs(int64_t n, int64_t d, int cus) {
  const int64_t group_bytes = (int64_t)snapshot_rows_in_flight(d) * 4 * d;
  int64_t per_cu = 131072 / group_bytes;
  per_cu = per_cu < 1 ? 1 : (per_cu > 8 ? 8 : per_cu);
  int64_t wgs = (int64_t)cus * per_cu;
  const int64_t by_rows = (n + 15) / 16;  // at least 16 rows per workgroup
  if (wgs > by_rows) wgs = by_rows;
  if (wgs < 1) wgs = 1;
  if (wgs > 16) wgs = wgs / 16 * 16;      // the partial rows are folded in 16 equal slices
  return (int)wgs;
}

// Partial rows per worker in the worker pass.  The pass is latency-bound (a few MB per launch), so
// the sampled rows are spread over about one workgroup per CU: 1, 2 or 4 rows per workgroup.
int dense_vr_parts(int64_t d, int32_t N, int32_t B, int cus) {
  (void)d;
  int64_t rows = (int64_t)N * B / cus;
  // measured: below four sampled rows per CU two rows per workgroup beat four (more workgroups pulling rows
  // outweigh the extra partial rows the fold has to read); at four rows per CU four per workgroup win (worker
  // pass +0.8 us, fold -1.3 us)
  int rpw = rows >= 4 ? 4 : (rows >= 2 ? 2 : 1);
  return (B + rpw - 1) / rpw;
}

hipError_t launch_dense_full_grad(const lpc_ctx *c, const float *w, float *z, bool want_loss, int64_t n_rows,
                                  hipStream_t st) {
  Shape s;
  if (!pick_shape(c->d, c->prob.ldx, c->prob.X, &s)) return hipErrorInvalidValue;
  DenseArgs a{};
  a.X = c->prob.X; a.ldx = c->prob.ldx; a.d = c->d; a.n = c->n; a.y = c->prob.y;
  a.w = w; a.z_out = z; a.part = c->s.part; a.part_loss = c->s.part_loss;
  a.n_rows = n_rows; a.loss = c->prob.loss; a.want_loss = want_loss ? 1 : 0;
  const int wgs = c->full_grad_wgs;
  const int rows_hint = snapshot_rows_in_flight(c->d);
  a.stream_loads = 1;  // X is read once per pass
  const int rg = rows_per_group(s);
  int64_t rpw = (n_rows + wgs - 1) / wgs;
  rpw = ((rpw + rg - 1) / rg) * rg;
  a.rows_per_wg = rpw;
  return dispatch<0>(s, a, wgs, rows_hint, st);
}

hipError_t launch_dense_vr_grad(const lpc_ctx *c, const float *w, const float *w_snap, const float *z_snap,
                                StreamKey key, uint32_t tag, int32_t worker_begin, int32_t worker_end,
                                bool plus_shared, hipStream_t st) {
  Shape s;
  if (!pick_shape(c->d, c->prob.ldx, c->prob.X, &s)) return hipErrorInvalidValue;
  // thinner threads for the latency-bound worker pass: 512 threads with eight columns each instead of 256 with
  // sixteen (C2: +0.7 % inner iterations/s, measured back to back on one machine); 1024 threads with eight columns for d = 8192 measured slower (13.1 -> 15.0 us)
  if (s.k == 4 && s.t == 256) { s.t = 512; s.k = 2; }
  DenseArgs a{};
  a.X = c->prob.X; a.ldx = c->prob.ldx; a.d = c->d; a.n = c->n; a.y = c->prob.y;
  a.w = w; a.w_snap = w_snap; a.z_snap = z_snap; a.part = c->s.part;
  a.loss = c->prob.loss; a.key = key; a.tag = tag; a.worker_begin = worker_begin;
  a.B = c->cfg.B; a.parts = c->vr_parts;
  a.rows_per_part = (c->cfg.B + c->vr_parts - 1) / c->vr_parts;
  a.shared_rel = plus_shared ? worker_end - worker_begin : -1;
  const int grid = (worker_end - worker_begin + (plus_shared ? 1 : 0)) * c->vr_parts;
  return z_snap ? dispatch<1>(s, a, grid, a.rows_per_part, st) : dispatch<2>(s, a, grid, a.rows_per_part, st);
}

}  // namespace lpc
