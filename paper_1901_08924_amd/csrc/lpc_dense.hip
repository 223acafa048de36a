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
  touch_kernel_arguments<(int)(sizeof(DenseArgs))>();
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

// ---------------------------------------------------------------------------------------------------------
// The worker pass in column tiles ("columns" form), for the small-d inner iteration.
//
// The rows kernel above needs all of w for a row's margin, so a workgroup owns whole rows and leaves a d-long
// partial gradient that a second launch folds.  Here the margins come from outside: the launch that produced w
// (the exchange, or dense_dots_kernel) also left, for every row the coming iteration samples, the partial dot
// products of the row with each 128-column tile of w.  A workgroup then owns ONE tile of ONE vector: it adds a
// row's partial dots (fixed order) to get the margin, forms the slope difference, and accumulates
// slope * x[tile] over the vector's B rows in a fixed order -- u^i's tile is complete inside the workgroup, with
// its statistics, and nothing is left to fold.  The rows are read twice (once for the dots, once here, the second
// time out of the cache) instead of once plus a write and a read of the partial rows.
// (kColTile = 128 columns per workgroup, kColThreads = 512: 16 groups of 32 lanes; a group takes one row at a time,
// a lane four columns; both in lpc_device.h, which the exchange kernel shares)

struct ColsArgs {
  const float *X;
  int64_t ldx, d, d_pad, n;
  const float *y, *z_snap;
  const float *pd;       // [rows][C]: partial dots of the sampled rows with w, rows = (vector, batch position)
  int32_t C;             // tiles = ceil(d_pad / 128)
  float *U;              // out: [nvec][ldu]
  int64_t ldu;
  double *stat_part;     // [vector][stat_slots][4]; slot = tile
  int32_t stat_slots, stat_vec0;
  StreamKey key;
  uint32_t tag;
  int32_t worker_begin, B, shared_rel, loss, vec4;
  int32_t at_snapshot;   // the iterate IS the snapshot (t = 0 of an epoch of Alg. 1): every difference is exactly zero
  float scale;
};

__global__ __launch_bounds__(kColThreads) void dense_cols_kernel(ColsArgs a) {
  constexpr int GROUPS = kColThreads / 32;
  __shared__ float4 part[GROUPS][kColTile / 4];
  __shared__ double red[2][4];
  const int tid = threadIdx.x, lane = tid & 63, rg = tid >> 5, l = tid & 31;
  const int32_t c = blockIdx.x, wrel = blockIdx.y;
  const uint32_t tag = wrel == a.shared_rel ? kTagShared : a.tag;
  const uint32_t worker = tag == kTagShared ? kSharedWorkerField : (uint32_t)(a.worker_begin + wrel);
  const int64_t j = (int64_t)c * kColTile + 4 * l;
  const int64_t room = a.d - j;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int32_t pos0 = 0; pos0 < a.B; pos0 += 4 * GROUPS) {  // four rows per group in flight
    int64_t row[4];
    float4 x[4];
    float yv[4], zsv[4], zp[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int32_t pos = pos0 + k * GROUPS + rg;
      const bool live = pos < a.B;
      row[k] = live ? sample_row(a.key, tag, worker, (uint32_t)pos, a.n) : 0;
      x[k] = live ? load_slice(a.X + row[k] * a.ldx + j, room, a.vec4 != 0) : make_float4(0.f, 0.f, 0.f, 0.f);
      yv[k] = live ? a.y[row[k]] : 0.0f;
      zsv[k] = live ? a.z_snap[row[k]] : 0.0f;
      // this lane's share of the row's partial dots: tiles l, l+32, ...
      float s = 0.0f;
      if (live) {
        const float *pd = a.pd + ((int64_t)wrel * a.B + pos) * a.C;
        for (int32_t t = l; t < a.C; t += 32) s += pd[t];
      }
      zp[k] = s;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float z = group32_sum(zp[k], lane);
      const bool live = pos0 + k * GROUPS + rg < a.B;
      // (at the snapshot the margin summed tile by tile equals the cached one only to rounding)
      const float coef =
          live && !a.at_snapshot ? loss_slope(a.loss, z, yv[k]) - loss_slope(a.loss, zsv[k], yv[k]) : 0.0f;
      acc.x = fmaf(coef, x[k].x, acc.x); acc.y = fmaf(coef, x[k].y, acc.y);
      acc.z = fmaf(coef, x[k].z, acc.z); acc.w = fmaf(coef, x[k].w, acc.w);
    }
  }
  part[rg][l] = acc;
  __syncthreads();
  double amax = 0.0, sum = 0.0, sumsq = 0.0, bad = 0.0;
  if (tid < kColTile) {
    const float *col = reinterpret_cast<const float *>(&part[0][0]) + tid;
    float v = col[0];
#pragma unroll
    for (int g = 1; g < GROUPS; ++g) v += col[g * kColTile];
    v *= a.scale;
    const int64_t jj = (int64_t)c * kColTile + tid;
    if (jj >= a.d) v = 0.0f;
    if (jj < a.d_pad) a.U[(int64_t)wrel * a.ldu + jj] = v;
    if (isfinite(v)) {
      amax = fabs((double)v); sum = (double)v; sumsq = (double)v * (double)v;
    } else {
      bad = 1.0;
    }
  }
  if (a.stat_part && tid < kColTile) {  // two whole wavefronts
    amax = wave_max(amax); sum = wave_sum(sum); sumsq = wave_sum(sumsq); bad = wave_sum(bad);
    if (lane == 0) { red[tid >> 6][0] = amax; red[tid >> 6][1] = sum; red[tid >> 6][2] = sumsq; red[tid >> 6][3] = bad; }
  }
  __syncthreads();
  if (a.stat_part && tid == 0) {
    double *p = a.stat_part + ((int64_t)(a.stat_vec0 + wrel) * a.stat_slots + c) * 4;
    p[0] = fmax(red[0][0], red[1][0]); p[1] = red[0][1] + red[1][1]; p[2] = red[0][2] + red[1][2];
    p[3] = red[0][3] + red[1][3];
  }
}

__global__ __launch_bounds__(kColThreads) void dense_dots_kernel(DotsArgs a) {
  __shared__ __attribute__((aligned(16))) float wsh[kColTile];
  const int tid = threadIdx.x;
  const int32_t c = blockIdx.x;
  if (tid < kColTile) {
    const int64_t jj = (int64_t)c * kColTile + tid;
    wsh[tid] = jj < a.d ? a.w[jj] : 0.0f;
  }
  __syncthreads();
  const int32_t first = (int32_t)blockIdx.y * a.rows_per_wg;
  for (int32_t i0 = 0; i0 < a.rows_per_wg; i0 += kDotRows) {
    float4 x[8];
    const int32_t count = a.rows_per_wg - i0 < kDotRows ? a.rows_per_wg - i0 : kDotRows;
    tile_dots_load(a, c, first + i0, count, tid, x);
    tile_dots_finish(a, wsh, c, first + i0, count, tid, x);
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
  if constexpr (MODE == 1 && K * VEC <= 16 && T >= 256) {  // the worker pass with cached margins: up to eight rows at once
    if (rows_hint >= 8) {
      LPC_LAUNCH_TIMED((dense_rows_kernel<VEC, K, T, 8, MODE>), dim3((unsigned)grid), dim3(T), st, a);
      return;
    }
    if (rows_hint >= 6) {
      LPC_LAUNCH_TIMED((dense_rows_kernel<VEC, K, T, 6, MODE>), dim3((unsigned)grid), dim3(T), st, a);
      return;
    }
    if (rows_hint == 5) {
      LPC_LAUNCH_TIMED((dense_rows_kernel<VEC, K, T, 5, MODE>), dim3((unsigned)grid), dim3(T), st, a);
      return;
    }
    if (rows_hint == 3) {
      LPC_LAUNCH_TIMED((dense_rows_kernel<VEC, K, T, 3, MODE>), dim3((unsigned)grid), dim3(T), st, a);
      return;
    }
  }
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

// Partial rows per vector in the worker pass (nvec vectors: the N workers and, for Alg. 2 / 3, the shared batch).
// The pass is latency-bound (a few MB per launch): what counts is the largest number of rows any one CU has to
// pull, then how few workgroups and partial rows there are.  A workgroup's rows belong to one
// vector, so with r rows per workgroup there are nvec * ceil(B / r) workgroups and the busiest CU holds
// ceil(workgroups / cus) * r rows.  Measured on d = 8192, N = 16 + the shared batch, B = 64 (1088 rows on 256 CUs):
// four rows per workgroup are 272 workgroups, sixteen CUs get two of them and the pass takes 13.2 us; five rows are
// 221 workgroups, one per CU, 10.9 us; six 11.5 us; eight 16.3 us; one row per workgroup (1088 workgroups, the
// same five rows on the busiest CU, 64 partial rows per vector) is slower than all of them.  With two sampled rows
// per CU two rows per workgroup beat four, which the same ordering reproduces.  `many`: the kernel can hold 3, 5, 6 or 8 rows in registers at once
// (cached margins, 16-byte loads, at most 16 floats per thread and row).
int dense_vr_parts(int64_t d, int64_t ldx, const void *X, int32_t nvec, int32_t B, int cus, bool cached) {
  Shape s;
  bool many = cached && pick_shape(d, ldx, X, &s);
  if (many) {
    if (s.k == 4 && s.t == 256) { s.t = 512; s.k = 2; }  // as launch_dense_vr_grad reshapes it
    many = s.vec == 4 && s.k * s.vec <= 16 && s.t >= 256;
  }
  const int64_t rows = (int64_t)nvec * B;
  if (!many || rows > (int64_t)8 * cus) {
    const int64_t per_cu = rows / cus;
    const int rpw = per_cu >= 4 ? 4 : (per_cu >= 2 ? 2 : 1);
    return (B + rpw - 1) / rpw;
  }
  static const int cand[] = {1, 2, 3, 4, 5, 6, 8};
  int best = 1;
  int64_t best_load = INT64_MAX;
  for (int r : cand) {
    const int64_t wgs = (int64_t)nvec * ((B + r - 1) / r);
    const int64_t load = ((wgs + cus - 1) / cus) * r;
    if (load <= best_load) {  // ties: more rows per workgroup (fewer workgroups and partial rows)
      best = r; best_load = load;
    }
  }
  return (B + best - 1) / best;
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

bool dense_cols_supported(const lpc_ctx *c) {
  return c->grad_ok && !c->csr && !c->mlp && c->d_pad <= 16384;
}

int dense_cols_tiles(const lpc_ctx *c) { return (int)((c->d_pad + kColTile - 1) / kColTile); }

namespace {
bool rows_vec4(const lpc_ctx *c) {
  return c->d % 4 == 0 && c->prob.ldx % 4 == 0 && (((uintptr_t)c->prob.X) & 15u) == 0;
}
}  // namespace

// row groups of a dots launch over `rows` rows: enough workgroups to fill the chip, at least 16 rows each
int dense_dots_groups(const lpc_ctx *c, int32_t rows) {
  const int tiles = dense_cols_tiles(c);
  int groups = (2 * c->cus + tiles - 1) / tiles;
  const int by_rows = (rows + 15) / 16;
  if (groups > by_rows) groups = by_rows;
  return groups < 1 ? 1 : groups;
}

hipError_t launch_dense_dots(const lpc_ctx *c, const float *w, StreamKey key, int32_t worker_begin, int32_t nvec,
                             bool last_is_shared, uint32_t tag, float *pd, hipStream_t st) {
  DotsArgs a{};
  a.X = c->prob.X; a.ldx = c->prob.ldx; a.d = c->d; a.n = c->n; a.w = w; a.pd = pd;
  a.C = dense_cols_tiles(c); a.B = c->cfg.B; a.nvec = nvec; a.worker_begin = worker_begin;
  a.shared_rel = last_is_shared ? nvec - 1 : -1; a.vec4 = rows_vec4(c) ? 1 : 0; a.key = key; a.tag = tag;
  const int32_t rows = nvec * c->cfg.B;
  const int groups = dense_dots_groups(c, rows);
  a.rows_per_wg = (rows + groups - 1) / groups;
  hipLaunchKernelGGL(dense_dots_kernel, dim3((unsigned)a.C, (unsigned)groups), dim3(kColThreads), 0, st, a);
  return hipGetLastError();
}

hipError_t launch_dense_cols(const lpc_ctx *c, const float *z_snap, const float *pd, StreamKey key, uint32_t tag,
                             int32_t worker_begin, int32_t nvec, bool last_is_shared, float *U, int64_t ldu,
                             bool want_stats, int32_t stat_vec0, hipStream_t st) {
  ColsArgs a{};
  a.at_snapshot = c->at_snapshot ? 1 : 0;
  a.X = c->prob.X; a.ldx = c->prob.ldx; a.d = c->d; a.d_pad = c->d_pad; a.n = c->n;
  a.y = c->prob.y; a.z_snap = z_snap; a.pd = pd; a.C = dense_cols_tiles(c);
  a.U = U; a.ldu = ldu;
  a.stat_part = want_stats ? c->s.stat_part : nullptr; a.stat_slots = c->stat_slots; a.stat_vec0 = stat_vec0;
  a.key = key; a.tag = tag; a.worker_begin = worker_begin; a.B = c->cfg.B;
  a.shared_rel = last_is_shared ? nvec - 1 : -1; a.loss = c->prob.loss; a.vec4 = rows_vec4(c) ? 1 : 0;
  a.scale = (float)(1.0 / (double)c->cfg.B);
  LPC_LAUNCH_TIMED(dense_cols_kernel, dim3((unsigned)a.C, (unsigned)nvec), dim3(kColThreads), st, a);
  return hipGetLastError();
}

}  // namespace lpc
