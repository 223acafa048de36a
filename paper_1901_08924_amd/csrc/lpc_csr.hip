// CSR generalised-linear-model passes (gfx950): the snapshot gradient of
// Alg. 1 step 4 and the workers' variance-reduced differences of Alg. 1 step 6
// for sparse rows.
//
// Sixteen lanes own one row at a time (a wavefront works on four rows at once):
// the row's (column, value) pairs are read as contiguous spans, w is gathered
// (it stays cache resident), the dot product is closed inside the row of 16
// lanes, and the row is scattered back as coef * value into the gradient.
// A row costs three dependent memory round trips (row_ptr -> pairs -> w), so
// small groups keep many rows in flight per CU and the next row's data is
// requested while the current row is worked on.
// Text-like data has Zipf-distributed column ids, so a handful of "head"
// columns receive most of the scatter: each workgroup accumulates the first
// kHead columns privately in LDS and writes them once as a partial row that is
// folded in a fixed order.  The rare tail columns are summed column by column
// from a column-major copy of the tail entries built when the context is
// created (a gather of the per-row slopes, no atomics, fixed order); when that
// copy is not available they fall back to global float atomics.
#include <hip/hip_runtime.h>

#include "lpc_device.h"
#include "lpc_internal.h"

namespace lpc {

namespace {

constexpr int kThreads = 256;
constexpr int kGroup = 16;                     // lanes per row

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
  float *coef;        // snapshot pass with the column-major tail: per-row loss slopes
  float *tail;        // snapshot pass: d floats, zeroed; tail columns accumulate here
  float *part;        // snapshot pass: [workgroup][head] partial rows
  double *part_loss;  // snapshot pass
  float *U;           // worker pass: [N][d_pad], zeroed
  float *planes;      // sparse worker pass: [N][parts-1][d_pad] tail planes of a worker's workgroups 1..parts-1
  uint32_t *touched;  // sparse worker pass: [N][bitmap_words], one bit per 32-coordinate segment
  uint32_t *touched_parts;  // ... and [N][parts-1][bitmap_words] for the workgroups 1..parts-1 of a worker
  int64_t bitmap_words;
  int32_t parts, rows_per_part;  // sparse worker pass: workgroups per worker, sampled rows per workgroup
  const RowPlan *plan;           // sparse worker pass: [N][B] rows of this iteration, looked up ahead
  int64_t n, d, d_pad, n_rows, nnz;
  int32_t head;       // columns [0, head) are privatised in LDS (snapshot pass)
  int32_t loss, want_loss, want_grad;
  StreamKey key;
  uint32_t tag;
  int32_t worker_begin, B;
  int32_t shared_rel;   // plan of an epoch: the vector that draws the shared batch J (-1: none)
  float scale;
};

// sum over the 16 lanes of a group; every lane of the group returns it
__device__ __forceinline__ float group_sum(float v) {
  static_assert(kGroup == 16, "a group is one row of 16 lanes");
  return row16_sum(v);
}

constexpr int kFullThreads = 512;  // snapshot pass: threads per workgroup

struct RowExtent {
  int32_t lo, hi;
  float y;
};

__device__ __forceinline__ RowExtent load_extent(const CsrArgs &a, int64_t r, int64_t r1) {
  const int64_t rc = r < r1 ? r : r1 - 1;
  RowExtent x;
  x.lo = a.row_ptr[rc];
  x.hi = a.row_ptr[rc + 1];
  x.y = a.y[rc];
  if (r >= r1) x.hi = x.lo;  // past the end: an empty row
  return x;
}

// the first 64 pairs of a row, four per lane; entries past the row come back as (column 0, value 0)
__device__ __forceinline__ void load_pairs(const CsrArgs &a, const RowExtent &x, int gl, int32_t (&c)[4],
                                           float (&v)[4]) {
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int32_t e = x.lo + q * kGroup + gl;
    const bool ok = e < x.hi;
    // streamed once: non-temporal, so that the pairs do not displace w in the caches
    c[q] = ok ? __builtin_nontemporal_load(a.col_idx + e) : 0;
    v[q] = ok ? __builtin_nontemporal_load(a.vals + e) : 0.0f;
  }
}

// Ordered scatter.  Float additions into one accumulator must happen in a fixed order for the result not to
// depend on scheduling; both passes below arrange that without giving up the atomics' convenience: one
// wavefront's atomic additions to one address execute in issue order, in LDS and in memory, so it is enough that
// every accumulator receives its contributions from wavefronts that take turns in a fixed order.
struct RowRecord {
  int32_t lo, len;
  float coef;
};

// Snapshot pass.  Workgroup b takes rows [b*rows_per_wg, ...); group g of it every kFullGroups-th row.
// Built to keep many rows in flight: 512 threads (32 row groups) share one LDS head, two such workgroups
// fit a CU, the first 64 pairs of a row (most rows have no more) are requested one row ahead and the extent
// of a row two rows ahead.  (1024 threads per workgroup: with the registers the rotation below needs a CU held one
// such workgroup at a time, and sixteen wavefronts per rotation instead of eight: 297 against 280 us for the pass
// on n = d = 2^20.)
// The head columns' LDS accumulation is made independent of scheduling by a fixed rotation: a wavefront keeps
// the pairs and slopes of kTurnRounds rounds of its rows in registers and adds them into the LDS accumulator only
// when the counter `turn` reads block*NW + w (block = round / kTurnRounds, w = its index), then advances the
// counter.  One wavefront's LDS instructions execute in issue order and the counter lives in LDS too, so one
// turn's additions are complete before the next turn's begin: every accumulator receives its contributions in one
// fixed order.  Every wavefront goes through the same number of blocks (rows past the end are empty rows) and
// there is no barrier inside the loop, so the wavefront whose turn it is can always proceed.
constexpr int kFullGroups = kFullThreads / kGroup;
constexpr int kTurnRounds = 4;

template <bool CSC>
__global__ __launch_bounds__(kFullThreads) void csr_full_kernel(CsrArgs a, int64_t rows_per_wg) {
  // LDS: the head of the gradient accumulator, then a copy of the head of w.  Most entries fall into the
  // head columns; a 4-byte gather from memory costs a cache-line lookup per lane, and that lookup rate, not
  // HBM, is what bounds this pass.
  extern __shared__ float head_acc[];
  float *w_head = head_acc + a.head;
  __shared__ double loss_red[kFullGroups];
  __shared__ uint32_t turn;
  constexpr int NW = kFullThreads / 64;
  const int tid = threadIdx.x, gl = tid & (kGroup - 1), grp = tid / kGroup, wv = tid >> 6;
  for (int32_t j = tid; j < a.head; j += kFullThreads) {
    head_acc[j] = 0.0f;
    w_head[j] = a.w[j];
  }
  if (tid == 0) turn = 0u;
  __syncthreads();
  const int64_t r0 = (int64_t)blockIdx.x * rows_per_wg;
  int64_t r1 = r0 + rows_per_wg;
  if (r1 > a.n_rows) r1 = a.n_rows;
  double loss_acc = 0.0;
  if (r0 < r1) {  // uniform over the workgroup
    const int64_t rounds = (r1 - r0 + kFullGroups - 1) / kFullGroups;
    const int64_t blocks = (rounds + kTurnRounds - 1) / kTurnRounds;  // the same for every wavefront
    int64_t r = r0 + grp;
    RowExtent cur = load_extent(a, r, r1);
    RowExtent nxt = load_extent(a, r + kFullGroups, r1);
    int32_t c[4];
    float v[4];
    load_pairs(a, cur, gl, c, v);
    for (int64_t block = 0; block < blocks; ++block) {
      int32_t kc[kTurnRounds][4], klo[kTurnRounds], khi[kTurnRounds];
      float kg[kTurnRounds][4], kcoef[kTurnRounds];
#pragma unroll
      for (int t = 0; t < kTurnRounds; ++t) {
        // the gathers of this row go out first: the wait for them then leaves the prefetches below in
        // flight (memory operations complete in issue order as far as the wait counter is concerned)
        float wv4[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          wv4[q] = w_head[c[q] < a.head ? c[q] : 0];
          if (c[q] >= a.head && v[q] != 0.0f) wv4[q] = a.w[c[q]];  // only the lanes that need memory ask for it
        }
        const RowExtent nxt2 = load_extent(a, r + 2 * kFullGroups, r1);
        int32_t cn[4];
        float vn[4];
        load_pairs(a, nxt, gl, cn, vn);
        float s = 0.0f;
#pragma unroll
        for (int q = 0; q < 4; ++q) s = fmaf(v[q], wv4[q], s);
        for (int32_t e = cur.lo + 4 * kGroup + gl; e < cur.hi; e += kGroup) {  // rows longer than 64 entries
          const int32_t col = a.col_idx[e];
          // two loads and a choice between the VALUES (a choice between an LDS and a memory address would make the
          // load a generic one); rows this long are rare
          const float from_lds = w_head[col < a.head ? col : 0], from_mem = a.w[col];
          s = fmaf(a.vals[e], col < a.head ? from_lds : from_mem, s);
        }
        const float z = group_sum(s);
        const float coef = loss_slope(a.loss, z, cur.y);
        if (gl == 0 && r < r1) {
          if (a.z_out) a.z_out[r] = z;
          if (CSC) a.coef[r] = coef;
          if (a.want_loss) loss_acc += (double)loss_value(a.loss, z, cur.y);
        }
        klo[t] = cur.lo; khi[t] = cur.hi; kcoef[t] = coef;
#pragma unroll
        for (int q = 0; q < 4; ++q) { kc[t][q] = c[q]; kg[t][q] = coef * v[q]; }
        r += kFullGroups;
        cur = nxt; nxt = nxt2;
#pragma unroll
        for (int q = 0; q < 4; ++q) { c[q] = cn[q]; v[q] = vn[q]; }
      }
      if (a.want_grad) {
        const uint32_t ticket = (uint32_t)block * NW + (uint32_t)wv;
        while (__hip_atomic_load(&turn, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != ticket) {
        }
        asm volatile("" ::: "memory");  // the additions below stay behind the read of the counter
#pragma unroll
        for (int t = 0; t < kTurnRounds; ++t) {
#pragma unroll
          for (int q = 0; q < 4; ++q)  // a zero: outside the row (a stored zero adds nothing either)
            if (kg[t][q] != 0.0f && kc[t][q] < a.head) atomicAdd(&head_acc[kc[t][q]], kg[t][q]);  // LDS
          for (int32_t e = klo[t] + 4 * kGroup + gl; e < khi[t]; e += kGroup) {
            const int32_t col = a.col_idx[e];
            if (col < a.head) atomicAdd(&head_acc[col], kcoef[t] * a.vals[e]);
          }
        }
        if (!CSC) {  // without the column-major copy the tail columns take float atomics in memory
#pragma unroll
          for (int t = 0; t < kTurnRounds; ++t) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
              if (kg[t][q] != 0.0f && kc[t][q] >= a.head) atomicAdd(&a.tail[kc[t][q]], kg[t][q]);
            for (int32_t e = klo[t] + 4 * kGroup + gl; e < khi[t]; e += kGroup) {
              const int32_t col = a.col_idx[e];
              if (col >= a.head) atomicAdd(&a.tail[col], kcoef[t] * a.vals[e]);
            }
          }
        }
        // the additions above are LDS instructions issued before this store (the compiler keeps the order, the LDS
        // executes a wavefront's instructions in issue order), so whoever reads the new count finds them done
        asm volatile("" ::: "memory");
        if ((tid & 63) == 0) __hip_atomic_store(&turn, ticket + 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
      }
    }
  }
  __syncthreads();
  if (a.want_grad) {
    float *dst = a.part + (int64_t)blockIdx.x * a.head;
    for (int32_t j = tid; j < a.head; j += kFullThreads) dst[j] = head_acc[j];
  }
  if (a.want_loss) {
    if (gl == 0) loss_red[grp] = loss_acc;
    __syncthreads();
    if (tid == 0) {
      double t = 0.0;
      for (int k = 0; k < kFullGroups; ++k) t += loss_red[k];
      a.part_loss[blockIdx.x] = t;
    }
  }
}

// Tail columns from the column-major copy: mu[c] = scale * sum_k coef[row_k] * val_k over the column's
// entries, each column summed in a fixed order.  Columns are served by length so that no lane walks a long
// column alone: up to kCscShort entries one thread per column (all tail columns in index order, so that
// neighbouring lanes read neighbouring entries; longer ones are skipped here), up to kCscMedium a row of 16
// lanes per column, beyond that a wavefront per column; the two longer classes come from lists made at
// build time.  One launch: the workgroup index selects the class.
constexpr int kCscShort = 16;
constexpr int kCscMedium = 128;

struct CscArgs {
  const int32_t *ptr, *rows;
  const float *vals, *coef;
  const int32_t *medium, *longc;  // column lists
  int32_t n_medium, n_long;
  int32_t wgs_short, wgs_medium;
  int64_t head, d, n_rows;
  float scale;
  float *mu;
};

// partial sum of entries lo + lane, lo + lane + stride, ... (four entries per step, all loads in flight)
__device__ __forceinline__ float csc_column_part(const CscArgs &a, int32_t lo, int32_t hi, int lane, int stride) {
  float acc = 0.0f;
  for (int32_t k = lo + lane; k < hi; k += 4 * stride) {
    int32_t rr[4];
    float vv[4], cc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const bool ok = k + q * stride < hi;
      rr[q] = ok ? a.rows[k + q * stride] : 0;
      vv[q] = ok ? a.vals[k + q * stride] : 0.0f;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) cc[q] = (k + q * stride < hi && rr[q] < a.n_rows) ? a.coef[rr[q]] : 0.0f;
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = fmaf(cc[q], vv[q], acc);
  }
  return acc;
}

__global__ __launch_bounds__(kThreads) void csc_tail_kernel(CscArgs a) {
  const int tid = threadIdx.x;
  int32_t b = blockIdx.x;
  if (b < a.wgs_short) {
    const int64_t c = a.head + (int64_t)b * kThreads + tid;
    if (c >= a.d) return;
    const int32_t lo = a.ptr[c], hi = a.ptr[c + 1];
    if (hi - lo > kCscShort) return;
    a.mu[c] = csc_column_part(a, lo, hi, 0, 1) * a.scale;
    return;
  }
  b -= a.wgs_short;
  if (b < a.wgs_medium) {
    const int32_t i = b * (kThreads / kGroup) + tid / kGroup;
    if (i >= a.n_medium) return;  // whole rows of 16 lanes leave together
    const int32_t c = a.medium[i];
    const float t = group_sum(csc_column_part(a, a.ptr[c], a.ptr[c + 1], tid & (kGroup - 1), kGroup));
    if ((tid & (kGroup - 1)) == 0) a.mu[c] = t * a.scale;
    return;
  }
  b -= a.wgs_medium;
  const int32_t i = b * (kThreads / 64) + tid / 64;
  if (i >= a.n_long) return;  // whole wavefronts leave together
  const int32_t c = a.longc[i];
  const float t = wave_sum(csc_column_part(a, a.ptr[c], a.ptr[c + 1], tid & 63, 64));
  if ((tid & 63) == 0) a.mu[c] = t * a.scale;
}

// build: number of medium / long tail columns (cls[0], cls[1]), then their lists
__global__ void csc_classify_kernel(const int32_t *__restrict__ ptr, int64_t head, int64_t d, int32_t *cls,
                                    int32_t *__restrict__ medium, int32_t *__restrict__ longc) {
  const int64_t c = head + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= d) return;
  const int32_t len = ptr[c + 1] - ptr[c];
  if (len <= kCscShort) return;
  if (len <= kCscMedium) {
    const int32_t k = atomicAdd(&cls[0], 1);
    if (medium) medium[k] = (int32_t)c;
  } else {
    const int32_t k = atomicAdd(&cls[1], 1);
    if (longc) longc[k] = (int32_t)c;
  }
}

// ---- column-major copy of the tail entries, built once per context --------------------------------
__global__ void csc_count_kernel(const int32_t *__restrict__ col_idx, int64_t nnz, int32_t head,
                                 int32_t *__restrict__ count) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < nnz && col_idx[e] >= head) atomicAdd(&count[col_idx[e]], 1);
}

// exclusive prefix sum of count[0..d) into ptr[0..d], one workgroup walking 1024-element blocks; also the
// largest count (max_out)
__global__ __launch_bounds__(1024) void csc_scan_kernel(const int32_t *__restrict__ count, int64_t d,
                                                        int32_t *__restrict__ ptr, int32_t *__restrict__ max_out) {
  __shared__ int32_t buf[1024];
  __shared__ int32_t carry_sh;
  const int tid = threadIdx.x;
  if (tid == 0) carry_sh = 0;
  int32_t mx = 0;
  __syncthreads();
  for (int64_t base = 0; base < d; base += 1024) {
    const int64_t j = base + tid;
    const int32_t x = j < d ? count[j] : 0;
    mx = x > mx ? x : mx;
    buf[tid] = x;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {  // Hillis-Steele inclusive scan
      const int32_t t = tid >= off ? buf[tid - off] : 0;
      __syncthreads();
      buf[tid] += t;
      __syncthreads();
    }
    const int32_t carry = carry_sh;
    if (j < d) ptr[j] = carry + buf[tid] - x;
    __syncthreads();
    if (tid == 1023) carry_sh = carry + buf[1023];
    __syncthreads();
  }
  if (tid == 0) ptr[d] = carry_sh;
  buf[tid] = mx;
  __syncthreads();
  for (int off = 512; off > 0; off >>= 1) {
    if (tid < off) buf[tid] = buf[tid] > buf[tid + off] ? buf[tid] : buf[tid + off];
    __syncthreads();
  }
  if (tid == 0) *max_out = buf[0];
}

// thread per row: append the row's tail entries to their columns (any order inside a column)
__global__ void csc_fill_kernel(const int32_t *__restrict__ row_ptr, const int32_t *__restrict__ col_idx,
                                const float *__restrict__ vals, int64_t n, int32_t head,
                                int32_t *__restrict__ cursor, int32_t *__restrict__ rows, float *__restrict__ cvals) {
  const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n) return;
  for (int32_t e = row_ptr[r]; e < row_ptr[r + 1]; ++e) {
    const int32_t c = col_idx[e];
    if (c < head) continue;
    const int32_t k = atomicAdd(&cursor[c], 1);
    rows[k] = (int32_t)r;
    cvals[k] = vals[e];
  }
}

// thread per column: order the column's entries by row (insertion sort; the build refuses long tail columns)
__global__ void csc_sort_kernel(const int32_t *__restrict__ ptr, int64_t head, int64_t d, int32_t *__restrict__ rows,
                                float *__restrict__ cvals) {
  const int64_t c = head + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= d) return;
  const int32_t lo = ptr[c], hi = ptr[c + 1];
  for (int32_t i = lo + 1; i < hi; ++i) {
    const int32_t rk = rows[i];
    const float vk = cvals[i];
    int32_t j = i - 1;
    while (j >= lo && rows[j] > rk) {
      rows[j + 1] = rows[j];
      cvals[j + 1] = cvals[j];
      --j;
    }
    rows[j + 1] = rk;
    cvals[j + 1] = vk;
  }
}

__global__ void fill_i32_kernel(int32_t *dst, int32_t v, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = v;
}

// mu[j] = scale * tail[j] for the tail columns (the head comes from the fold of the partial rows)
__global__ void csr_tail_kernel(const float *__restrict__ tail, float scale, int64_t head, int64_t d,
                                float *__restrict__ mu) {
  const int64_t j = head + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j < d) mu[j] = tail[j] * scale;
}

// Worker pass, with the ordered scatter described above.  A workgroup takes rows_per_part consecutive batch
// positions of one worker: wavefronts 0 and 1 scatter, the kRowGroups groups of the others take the rows.
//   SPARSE = false: one workgroup per worker; u^i is the worker's zeroed row of U; the two scatter wavefronts
//     split the columns by parity.
//   SPARSE = true:  u^i stays sparse, and a worker's batch is cut into `parts` workgroups of one round each.  Head
//     columns accumulate in LDS (scatter wavefront 0) and leave as the workgroup's head row (a.part); a tail column
//     (scatter wavefront 1) is added to the workgroup's own plane of the worker's tail -- plane 0 is the worker's
//     row of U, plane p > 0 lies in a.planes -- which is all zero outside the segments touched in this
//     iteration, and its 32-coordinate segment is marked in the worker's bitmap.  The statistics pass adds head
//     rows and planes in workgroup order, so the result is one fixed sum whatever the timing.
//     A scatter wavefront pays per instruction, not per active lane, and a row has only about six tail entries: the
//     row groups count their tail entries, take their offsets from the counts of the rows before them, and write
//     one dense list in batch-position order, which the tail wavefront applies 64 entries at a time.  Two entries
//     of one instruction must not meet in one accumulator (the order of the two additions would be open): every
//     lane enters its list position into a small hash table with an atomic minimum on the accumulator's slot, the
//     lanes that find their own position there add and clear the slot, the others try again -- so entries of one
//     accumulator are added in list order, one instruction apart.  (The head entries stay row by row: such a list
//     of them, with the table's LDS round trips for every 64 entries, made the launch 3 us longer.)
constexpr int kSparseThreads = 1024;
constexpr int kScatterWaves = 2;
constexpr int kRowGroups = (kSparseThreads - 64 * kScatterWaves) / kGroup;  // rows per round: 56
// SPARSE: the kHotCols leading columns take almost half of all entries, and LDS float atomics run at about three
// cycles per lane, which would set the length of the scatter.  A row group leaves its values for these columns in a
// dense row of `hot` instead (plain stores), and one wavefront sums the rows' copies in batch-position order.
constexpr int kHotCols = 64;
constexpr int kPairCap = kRowGroups * 64;  // SPARSE: room for the list of tail entries
constexpr int kHashSlots = 2048;

template <bool CACHED, bool SPARSE>
__global__ __launch_bounds__(kSparseThreads) void csr_vr_ordered_kernel(CsrArgs a) {
  touch_kernel_arguments<(int)(sizeof(CsrArgs))>();
  extern __shared__ __align__(16) float head_acc[];  // SPARSE: a.head floats
  __shared__ RowRecord rec[SPARSE ? 1 : 2][kRowGroups];
  // a row's first 64 (column, coef * value) pairs, double-buffered over the rounds unless SPARSE (one round per
  // workgroup); SPARSE: column -1 where the pair went to `hot` or to the list of tail entries
  __shared__ int2 stage[SPARSE ? 1 : 2][kRowGroups][64];
  __shared__ int2 tail_list[SPARSE ? kPairCap : 1];
  __shared__ float hot[SPARSE ? kRowGroups : 1][kHotCols];
  __shared__ int32_t cnt[SPARSE ? kRowGroups : 1];  // a row's tail entries among its first 64
  __shared__ uint32_t hsh[SPARSE ? kHashSlots : 1];
  float hot_sum = 0.0f;
  const int tid = threadIdx.x, gl = tid & (kGroup - 1), lane = tid & 63, wv = tid >> 6;
  const int32_t wrel = blockIdx.x / a.parts, part = blockIdx.x % a.parts;
  const int32_t pos0 = part * a.rows_per_part;
  const int32_t pos1 = pos0 + a.rows_per_part < a.B ? pos0 + a.rows_per_part : a.B;
  const uint32_t worker = (a.tag == kTagShared) ? kSharedWorkerField : (uint32_t)(a.worker_begin + wrel);
  const int32_t rounds = (pos1 - pos0 + kRowGroups - 1) / kRowGroups;
  // SPARSE: the head accumulator starts at zero (a.head is a multiple of 4096); the row wavefronts clear their share
  // behind their first requests
  auto clear_head = [&]() {
    if (SPARSE) {
      for (int32_t j = tid * 4; j < a.head; j += kSparseThreads * 4)
        *reinterpret_cast<float4 *>(head_acc + j) = make_float4(0.f, 0.f, 0.f, 0.f);
      for (int32_t j = tid; j < kHashSlots; j += kSparseThreads) hsh[j] = 0xffffffffu;  // free
      __syncthreads();
    }
  };
  if (wv >= kScatterWaves) {
    // ---- row wavefronts ------------------------------------------------------------------------------------
    const int grp = (tid - 64 * kScatterWaves) / kGroup;
    const RowPlan *plan = SPARSE ? a.plan + (int64_t)wrel * a.B : nullptr;
    auto fetch_row = [&](int32_t pos) {  // extent, label and snapshot margin of batch position pos
      RowPlan p{0, 0, 0.0f, 0.0f};
      if (pos >= pos1) return p;
      if (SPARSE) return plan[pos];
      const int64_t r = sample_row(a.key, a.tag, worker, (uint32_t)pos, a.n);
      p.lo = a.row_ptr[r]; p.hi = a.row_ptr[r + 1];
      p.y = a.y[r];
      p.z = CACHED ? a.z_snap[r] : 0.0f;
      return p;
    };
    auto fetch_pairs = [&](const RowPlan &p, int32_t (&c)[4], float (&v)[4]) {  // the row's first 64 pairs
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int32_t e = p.lo + q * kGroup + gl;
        const bool ok = e < p.hi;
        c[q] = ok ? a.col_idx[e] : 0;
        v[q] = ok ? a.vals[e] : 0.0f;
      }
    };
    RowPlan cur = fetch_row(pos0 + grp), nxt = fetch_row(pos0 + kRowGroups + grp);
    int32_t c[4];
    float v[4];
    fetch_pairs(cur, c, v);
    clear_head();
    for (int32_t round = 0; round < rounds; ++round) {
      // this row's gathers first, then the requests for the rounds ahead stay in flight behind them
      float wv4[4], wsv[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        wv4[q] = a.w[c[q]];
        wsv[q] = CACHED ? 0.0f : a.w_snap[c[q]];
      }
      RowPlan nxt2{0, 0, 0.0f, 0.0f};
      int32_t cn[4] = {0, 0, 0, 0};
      float vn[4] = {0.f, 0.f, 0.f, 0.f};
      if (round + 1 < rounds) {  // uniform
        nxt2 = fetch_row(pos0 + (round + 2) * kRowGroups + grp);
        fetch_pairs(nxt, cn, vn);
      }
      float s = 0.0f, s2 = 0.0f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        s = fmaf(v[q], wv4[q], s);
        if (!CACHED) s2 = fmaf(v[q], wsv[q], s2);
      }
      for (int32_t e = cur.lo + 4 * kGroup + gl; e < cur.hi; e += kGroup) {  // rows longer than 64 entries
        const int32_t col = a.col_idx[e];
        const float val = a.vals[e];
        s = fmaf(val, a.w[col], s);
        if (!CACHED) s2 = fmaf(val, a.w_snap[col], s2);
      }
      const float z = group_sum(s);
      const float zs = CACHED ? cur.z : group_sum(s2);
      const float coef = (loss_slope(a.loss, z, cur.y) - loss_slope(a.loss, zs, cur.y)) * a.scale;
      if constexpr (SPARSE) {
        // class of each of the row's first 64 entries: 3 hot, 1 other head, 2 tail, 0 past the row's end
        const int32_t len = cur.hi - cur.lo;
        *reinterpret_cast<float4 *>(&hot[grp][gl * 4]) = make_float4(0.f, 0.f, 0.f, 0.f);  // kHotCols = 4 * kGroup
        const int sh = lane & 48;  // this group's first lane in the wavefront
        int32_t cls[4], rt[4], nt = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          cls[q] = q * kGroup + gl >= len ? 0 : c[q] < kHotCols ? 3 : c[q] < a.head ? 1 : 2;
          if (cls[q] == 3) hot[grp][c[q]] = coef * v[q];
          stage[0][grp][q * kGroup + gl] = make_int2(cls[q] == 1 ? c[q] : -1, __float_as_int(coef * v[q]));
          const uint32_t gt = (uint32_t)(__ballot(cls[q] == 2) >> sh) & 0xffffu;
          rt[q] = nt + __popc(gt & ((1u << gl) - 1u)); nt += __popc(gt);
        }
        if (gl == 0) {
          cnt[grp] = nt;
          rec[0][grp] = RowRecord{cur.lo, len, coef};
        }
        __syncthreads();  // the rows' counts and staged head pairs are complete
        int32_t bt = 0;
        for (int k = gl; k < grp; k += kGroup) bt += cnt[k];
        bt = row16_sum(bt);
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (cls[q] == 2) tail_list[bt + rt[q]] = make_int2(c[q], __float_as_int(coef * v[q]));
        __syncthreads();  // the list of tail entries is complete
        if (wv == kScatterWaves) {  // first row wavefront: lane c sums hot column c over the rows, in order
          float acc = 0.0f;
#pragma unroll 8
          for (int r = 0; r < kRowGroups; ++r) acc += hot[r][lane];
          hot_sum = acc;
        }
      } else {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          stage[round & 1][grp][q * kGroup + gl] = make_int2(c[q], __float_as_int(coef * v[q]));
        if (gl == 0) rec[round & 1][grp] = RowRecord{cur.lo, cur.hi - cur.lo, coef};
        __syncthreads();  // barrier `round`: the round's records and staged pairs are complete
      }
      cur = nxt; nxt = nxt2;
#pragma unroll
      for (int q = 0; q < 4; ++q) { c[q] = cn[q]; v[q] = vn[q]; }
    }
  } else {
    // ---- scatter wavefronts --------------------------------------------------------------------------------
    float *u = a.U + (int64_t)wrel * a.d_pad;
    if (SPARSE && part > 0) u = a.planes + ((int64_t)wrel * (a.parts - 1) + (part - 1)) * a.d_pad;
    uint32_t *bm = SPARSE ? a.touched + (int64_t)wrel * a.bitmap_words : nullptr;
    if (SPARSE && part > 0) bm = a.touched_parts + ((int64_t)wrel * (a.parts - 1) + (part - 1)) * a.bitmap_words;
    clear_head();
    for (int32_t round = 0; round < rounds; ++round) {
      if constexpr (SPARSE) {
        __syncthreads();  // the rows' counts and staged head pairs are complete
        __syncthreads();  // the list of tail entries is complete
        if (wv == 0) {
          // head: rows in batch-position order, eight staged rows at a time, the next eight requested ahead
          const uint64_t long_rows = __ballot((lane < kRowGroups ? rec[0][lane].len : 0) > 64);
          static_assert(kRowGroups % 8 == 0, "the walk takes eight rows at a time");
          int2 t[8], tn[8];
#pragma unroll
          for (int q = 0; q < 8; ++q) t[q] = stage[0][q][lane];
          for (int32_t row0 = 0; row0 < kRowGroups; row0 += 8) {
            if (row0 + 8 < kRowGroups) {
#pragma unroll
              for (int q = 0; q < 8; ++q) tn[q] = stage[0][row0 + 8 + q][lane];
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) {
              if (t[q].x >= 0) atomicAdd(&head_acc[t[q].x], __int_as_float(t[q].y));
              if ((long_rows >> (row0 + q)) & 1ull) {  // uniform and rare: the rest of a long row comes from memory
                const RowRecord m = rec[0][row0 + q];
                for (int32_t k = 64 + lane; k < m.len; k += 64) {
                  const int32_t col = a.col_idx[m.lo + k];
                  if (col < a.head) atomicAdd(&head_acc[col], m.coef * a.vals[m.lo + k]);
                }
              }
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) t[q] = tn[q];
          }
        } else {
          const int32_t total = (int32_t)wave_sum((uint32_t)(lane < kRowGroups ? cnt[lane] : 0));
          uint64_t long_rows = __ballot((lane < kRowGroups ? rec[0][lane].len : 0) > 64);
          auto add = [&](int32_t col, float g) {
            atomicAdd(&u[col], g);
            atomicOr(&bm[col >> 10], 1u << ((col >> 5) & 31));
          };
          for (int32_t i0 = 0; i0 < total; i0 += 64) {
            const int32_t idx = i0 + lane;
            bool pending = idx < total;
            const int2 pr = pending ? tail_list[idx] : make_int2(0, 0);
            const uint32_t slot = ((uint32_t)pr.x ^ ((uint32_t)pr.x >> 11)) & (kHashSlots - 1);
            while (__ballot(pending) != 0ull) {  // uniform; every turn retires at least the smallest pending position
              if (pending) atomicMin(&hsh[slot], (uint32_t)idx);
              __builtin_amdgcn_wave_barrier();
              const bool won =
                  pending && __hip_atomic_load(&hsh[slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT) == (uint32_t)idx;
              __builtin_amdgcn_wave_barrier();
              if (won) {
                add(pr.x, __int_as_float(pr.y));
                __hip_atomic_store(&hsh[slot], 0xffffffffu, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
                pending = false;
              }
              __builtin_amdgcn_wave_barrier();
            }
          }
          // what rows longer than 64 entries hold past their first 64 comes from memory, after the list, row by row
          while (long_rows != 0ull) {
            const RowRecord m = rec[0][__builtin_ctzll(long_rows)];
            long_rows &= long_rows - 1ull;
            for (int32_t k = 64 + lane; k < m.len; k += 64) {
              const int32_t col = a.col_idx[m.lo + k];
              if (col >= a.head) add(col, m.coef * a.vals[m.lo + k]);
            }
          }
        }
      } else {
        __syncthreads();  // barrier `round`
        // rows in batch-position order, eight staged rows read at a time; wavefront wv takes the columns of its parity
        const int buf = round & 1;
        for (int32_t row0 = 0; row0 < kRowGroups; row0 += 8) {
          RowRecord m[8];
          int2 t[8];
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            m[q] = rec[buf][row0 + q];
            t[q] = stage[buf][row0 + q][lane];
          }
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            if (lane < m[q].len && (t[q].x & (kScatterWaves - 1)) == wv) atomicAdd(&u[t[q].x], __int_as_float(t[q].y));
            for (int32_t k = 64 + lane; k < m[q].len; k += 64) {  // the rest of a long row comes from memory
              const int32_t col = a.col_idx[m[q].lo + k];
              if ((col & (kScatterWaves - 1)) == wv) atomicAdd(&u[col], m[q].coef * a.vals[m[q].lo + k]);
            }
          }
        }
      }
    }
  }
  if (SPARSE) {
    __syncthreads();
    if (wv == kScatterWaves) head_acc[lane] += hot_sum;  // behind what a long row's further entries left there
    __syncthreads();
    float *dst = a.part + (int64_t)blockIdx.x * a.head;
    for (int32_t j = tid * 4; j < a.head; j += kSparseThreads * 4)
      *reinterpret_cast<float4 *>(dst + j) = *reinterpret_cast<const float4 *>(head_acc + j);
  }
}

// plan[(t*N + i)*B + pos] for every inner iteration t < m of an epoch: the draws do not depend on the iterates,
// so the random stream, row_ptr, y and the cached margins are read once here instead of at the head of every
// iteration's dependency chain.
__global__ void csr_plan_kernel(CsrArgs a, int32_t m, int32_t N, RowPlan *__restrict__ plan) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t per_iter = (int64_t)N * a.B;
  if (idx >= (int64_t)m * per_iter) return;
  StreamKey key = a.key;
  key.iter = (uint32_t)(idx / per_iter);
  const int64_t rem = idx % per_iter;
  const uint32_t vec = (uint32_t)(rem / a.B), pos = (uint32_t)(rem % a.B);
  // vector shared_rel, if any, draws the shared batch J of Alg. 2 (double sampling)
  const bool shared = (int32_t)vec == a.shared_rel;
  const int64_t r = sample_row(key, shared ? kTagShared : a.tag, shared ? kSharedWorkerField : vec, pos, a.n);
  RowPlan p;
  p.lo = a.row_ptr[r]; p.hi = a.row_ptr[r + 1];
  p.y = a.y[r];
  p.z = a.z_snap ? a.z_snap[r] : 0.0f;
  plan[idx] = p;
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
  int64_t wgs = 512;  // two resident 512-thread workgroups per CU (256: 305 us, 768: 345 us, 1024: 294 us against 280 us)
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

// Longest tail column the column-major copy accepts (its build sorts a column with one thread).
constexpr int32_t kCscMaxColumn = 4096;

// Builds the column-major copy of the tail entries in the context's scratch on `st` and waits for it.
// Sets c->csc_ready; leaves it false (the snapshot pass then uses atomics) when a tail column is too long.
hipError_t build_csc_tail(lpc_ctx *c, hipStream_t st) {
  c->csc_ready = false;
  const int32_t head = csr_head_columns(c->d);
  if (c->d <= head || c->prob.nnz <= 0) return hipSuccess;
  const int64_t d = c->d, nnz = c->prob.nnz;
  int32_t *count = c->s.csc_cursor;  // reused: counts, then insertion cursors
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((d + 1 + 255) / 256)), dim3(256), 0, st, count, 0, d + 1);
  hipLaunchKernelGGL(csc_count_kernel, dim3((unsigned)((nnz + 255) / 256)), dim3(256), 0, st, c->prob.col_idx, nnz, head,
                     count);
  hipLaunchKernelGGL(csc_scan_kernel, dim3(1), dim3(1024), 0, st, (const int32_t *)count, d, c->s.csc_ptr,
                     c->s.csc_ptr + d + 1);
  int32_t tail_info[1] = {0};
  hipError_t e = hipMemcpyAsync(tail_info, c->s.csc_ptr + d + 1, sizeof(int32_t), hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return e;
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return e;
  if (tail_info[0] > kCscMaxColumn) return hipSuccess;
  e = hipMemcpyAsync(count, c->s.csc_ptr, sizeof(int32_t) * (size_t)d, hipMemcpyDeviceToDevice, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(csc_fill_kernel, dim3((unsigned)((c->n + 255) / 256)), dim3(256), 0, st, c->prob.row_ptr,
                     c->prob.col_idx, c->prob.vals, c->n, head, count, c->s.csc_rows, c->s.csc_vals);
  hipLaunchKernelGGL(csc_sort_kernel, dim3((unsigned)((d - head + 255) / 256)), dim3(256), 0, st,
                     (const int32_t *)c->s.csc_ptr, (int64_t)head, d, c->s.csc_rows, c->s.csc_vals);
  // column lists by length: count, then fill (the cursor array is free again and holds both lists)
  int32_t *cls = c->s.csc_ptr + d + 2;
  int32_t counts[2] = {0, 0};
  hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, st, cls, 0, (int64_t)2);
  hipLaunchKernelGGL(csc_classify_kernel, dim3((unsigned)((d - head + 255) / 256)), dim3(256), 0, st,
                     (const int32_t *)c->s.csc_ptr, (int64_t)head, d, cls, (int32_t *)nullptr, (int32_t *)nullptr);
  e = hipMemcpyAsync(counts, cls, sizeof(counts), hipMemcpyDeviceToHost, st);
  if (e != hipSuccess) return e;
  e = hipStreamSynchronize(st);
  if (e != hipSuccess) return e;
  c->csc_medium = counts[0];
  c->csc_long = counts[1];
  hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(64), 0, st, cls, 0, (int64_t)2);
  hipLaunchKernelGGL(csc_classify_kernel, dim3((unsigned)((d - head + 255) / 256)), dim3(256), 0, st,
                     (const int32_t *)c->s.csc_ptr, (int64_t)head, d, cls, c->s.csc_cursor,
                     c->s.csc_cursor + c->csc_medium);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = hipStreamSynchronize(st);
  if (e == hipSuccess) c->csc_ready = true;
  return e;
}

hipError_t launch_csr_full_grad(const lpc_ctx *c, const float *w, float *mu, float *z, bool want_loss, int64_t n_rows,
                                hipStream_t st) {
  CsrArgs a{};
  a.row_ptr = c->prob.row_ptr; a.col_idx = c->prob.col_idx; a.vals = c->prob.vals; a.y = c->prob.y;
  a.w = w; a.z_out = z; a.tail = c->s.csr_tail; a.part = c->s.part; a.part_loss = c->s.part_loss;
  a.coef = c->s.csc_coef;
  a.n = c->n; a.d = c->d; a.d_pad = c->d_pad; a.n_rows = n_rows; a.nnz = c->prob.nnz;
  a.head = csr_head_columns(c->d); a.loss = c->prob.loss; a.want_loss = want_loss ? 1 : 0;
  a.want_grad = mu != nullptr ? 1 : 0;
  const bool csc = c->csc_ready && mu != nullptr;
  const int wgs = c->full_grad_wgs;
  const int64_t rpw = (n_rows + wgs - 1) / wgs;
  hipError_t e;
  if (!csc && mu) {
    e = launch_zero(c->s.csr_tail, c->d_pad, st);
    if (e != hipSuccess) return e;
  }
  const size_t lds = 2 * (size_t)a.head * sizeof(float);
  if (csc) hipLaunchKernelGGL(csr_full_kernel<true>, dim3((unsigned)wgs), dim3(kFullThreads), lds, st, a, rpw);
  else hipLaunchKernelGGL(csr_full_kernel<false>, dim3((unsigned)wgs), dim3(kFullThreads), lds, st, a, rpw);
  e = hipGetLastError();
  if (e != hipSuccess || !mu) return e;
  if (c->d > a.head) {
    const int64_t tail_n = c->d - a.head;
    const float scale = (float)(1.0 / (double)n_rows);
    if (csc) {
      CscArgs ca{};
      ca.ptr = c->s.csc_ptr; ca.rows = c->s.csc_rows; ca.vals = c->s.csc_vals; ca.coef = c->s.csc_coef;
      ca.medium = c->s.csc_cursor; ca.longc = c->s.csc_cursor + c->csc_medium;
      ca.n_medium = c->csc_medium; ca.n_long = c->csc_long;
      ca.wgs_short = (int32_t)((tail_n + kThreads - 1) / kThreads);
      ca.wgs_medium = (c->csc_medium + kThreads / kGroup - 1) / (kThreads / kGroup);
      const int32_t wgs_long = (c->csc_long + kThreads / 64 - 1) / (kThreads / 64);
      ca.head = a.head; ca.d = c->d; ca.n_rows = n_rows; ca.scale = scale; ca.mu = mu;
      hipLaunchKernelGGL(csc_tail_kernel, dim3((unsigned)(ca.wgs_short + ca.wgs_medium + wgs_long)), dim3(kThreads), 0,
                         st, ca);
    } else
      hipLaunchKernelGGL(csr_tail_kernel, dim3((unsigned)((tail_n + 255) / 256)), dim3(256), 0, st,
                         (const float *)c->s.csr_tail, scale, (int64_t)a.head, c->d, mu);
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
  a.parts = 1;
  a.rows_per_part = c->cfg.B;
  const dim3 grid((unsigned)nworkers);
  if (z_snap) hipLaunchKernelGGL((csr_vr_ordered_kernel<true, false>), grid, dim3(kSparseThreads), 0, st, a);
  else hipLaunchKernelGGL((csr_vr_ordered_kernel<false, false>), grid, dim3(kSparseThreads), 0, st, a);
  return hipGetLastError();
}

// Sparse worker pass (all N workers).  s.U rows and the bitmap must be zero outside what this call adds.
// workgroups per worker of the sparse worker pass: one round of rows each
// (measured on n = d = 2^20, N = 16, B = 256: two rounds per workgroup, hence three planes per worker instead of
// five, make this pass 7 us slower and the statistics pass 3.4 us faster)
int csr_sparse_parts(int32_t B) { return (B + kRowGroups - 1) / kRowGroups; }

// Leading columns the sparse inner iteration treats densely.  Twice the snapshot pass's head when d is large: the
// bitmap words right behind an 8192-column head are nearly full in every iteration, and the wavefronts of the
// statistics pass and of the quantizer that own them then need a second step of 32 segments, which sets the
// length of both launches.
int csr_sparse_head_columns(int64_t d) {
  const int h = csr_head_columns(d);
  return d >= 16 * (int64_t)h ? 2 * h : h;
}

hipError_t launch_csr_plan(const lpc_ctx *c, const float *z_snap, StreamKey key0, bool plus_shared, hipStream_t st) {
  CsrArgs a{};
  a.row_ptr = c->prob.row_ptr; a.y = c->prob.y; a.z_snap = z_snap;
  a.n = c->n; a.B = c->cfg.B; a.key = key0; a.tag = kTagBatch;
  const int32_t nvec = c->cfg.N + (plus_shared ? 1 : 0);
  a.shared_rel = plus_shared ? c->cfg.N : -1;
  const int64_t total = (int64_t)c->cfg.m * nvec * c->cfg.B;
  hipLaunchKernelGGL(csr_plan_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a, c->cfg.m, nvec,
                     c->s.csr_plan);
  return hipGetLastError();
}

hipError_t launch_csr_vr_sparse(const lpc_ctx *c, const float *w, const float *w_snap, const float *z_snap,
                                StreamKey key, const RowPlan *plan, int32_t nvec, hipStream_t st) {
  CsrArgs a{};
  a.plan = plan;
  a.row_ptr = c->prob.row_ptr; a.col_idx = c->prob.col_idx; a.vals = c->prob.vals; a.y = c->prob.y;
  a.w = w; a.w_snap = w_snap; a.z_snap = z_snap; a.U = c->s.U; a.part = c->s.part;
  a.touched = c->s.touched; a.bitmap_words = c->bitmap_words;
  a.n = c->n; a.d = c->d; a.d_pad = c->d_pad; a.loss = c->prob.loss;
  a.head = c->sparse_head;
  a.key = key; a.tag = kTagBatch; a.worker_begin = 0; a.B = c->cfg.B;
  a.scale = (float)(1.0 / (double)c->cfg.B);
  a.parts = csr_sparse_parts(c->cfg.B);
  a.rows_per_part = kRowGroups;  // one round per workgroup: the kernel's `hot` rows are single-buffered
  a.planes = c->s.sparse_planes; a.touched_parts = c->s.touched_parts;
  const dim3 grid((unsigned)(nvec * a.parts));  // the rows of vector k are plan[k*B ..]
  const size_t lds = (size_t)a.head * sizeof(float);
  if (z_snap) hipLaunchKernelGGL((csr_vr_ordered_kernel<true, true>), grid, dim3(kSparseThreads), lds, st, a);
  else hipLaunchKernelGGL((csr_vr_ordered_kernel<false, true>), grid, dim3(kSparseThreads), lds, st, a);
  return hipGetLastError();
}

}  // namespace lpc
