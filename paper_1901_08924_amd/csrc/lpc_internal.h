// Internal declarations shared by the translation units of the HIP library.
// Nothing here is part of the public ABI (include/lpc.h is).
#pragma once

#include <hip/hip_runtime.h>
#if defined(__HIPCC__)
#include <hip/hip_ext.h>   // timed launches; device translation units only
#endif
#include <stdint.h>

#include <vector>

#include "lpc.h"

namespace lpc {

constexpr uint32_t kTagQuant = 0, kTagBatch = 1, kTagShared = 2, kTagRequant = 3;
constexpr uint32_t kSharedWorkerField = 0xFFFFFFu;

// Per-vector quantizer parameters, produced on the device right after the
// statistics of the vector are known (eq. (3)).
struct QParams {
  float delta;     // scale factor; 0 for an all-zero vector
  float rdelta;    // float(1/delta); 0 when delta == 0
  float thresh;    // positive clip threshold lambda*|u|_inf
  float neg_edge;  // smallest codebook value -2^(b-1)*delta
};

struct StreamKey {
  uint32_t seed_lo, seed_hi, epoch, iter;
};

// One (possibly batched, possibly two-segment) contraction on the matrix cores, see lpc_gemm.hip:
//   C[m][n] (+)= alpha * sum_s sum_k opA_s(m,k) * opB_s(k,n)  (+ bias[n]) (ReLU) (masked by relu_mask > 0)
// transA: A is stored [k][m] instead of [m][k]; transB: B is stored [n][k] instead of [k][n].
struct GemmArgs {
  const float *A[2];
  const float *B[2];
  int64_t lda[2], ldb[2], strideA[2], strideB[2];
  float *C;
  int64_t ldc, strideC;
  int M, N, K;
  int transA, transB;
  float alpha;
  const float *bias;
  int64_t strideBias;  // per batch element
  int relu;
  const float *relu_mask;  // same layout as C
  int accumulate;
  int nseg, batch;
  // optional: every tile also leaves the statistics (|max|, sum, sum of squares, non-finite count) of the values
  // it stored as partial number stat_slot0 + tile index of its batch item (matrix-core path only)
  double *stat_part;
  int64_t stat_batch_stride;  // doubles between the partial arrays of consecutive batch items
  int32_t stat_slot0;
};

// One sampled row of a CSR epoch, looked up ahead of the inner loop: its extent in col_idx/vals, its label and
// its cached snapshot margin.
struct RowPlan {
  int32_t lo, hi;
  float y, z;
};

// One symbol of the entropy coder: the codeword with its bits reversed (the first stream bit at bit 0) and
// its length; length 0 = the symbol has no codeword.
struct HuffEntry {
  uint32_t rev, len;
};

// Kernel-class timing (lpc_profile_enable): where a class is ONE kernel launch, that launch carries the class's two
// events itself, so their interval is the dispatch's own begin and end time stamps (what a kernel trace reports)
// instead of an interval between two event records around it, which adds a few microseconds.
struct LaunchTimer {
  hipEvent_t start = nullptr, stop = nullptr;
  bool used = false;
};
extern thread_local LaunchTimer *g_launch_timer;  // set while such a class's launch is being issued, else nullptr
#define LPC_LAUNCH_TIMED(kernel, grid, block, st, ...)                                                        \
  do {                                                                                                        \
    lpc::LaunchTimer *lt_ = lpc::g_launch_timer;                                                              \
    if (lt_ && !lt_->used) {                                                                                  \
      lt_->used = true;                                                                                       \
      hipExtLaunchKernelGGL(kernel, grid, block, 0, st, lt_->start, lt_->stop, 0, __VA_ARGS__);               \
    } else {                                                                                                  \
      hipLaunchKernelGGL(kernel, grid, block, 0, st, __VA_ARGS__);                                            \
    }                                                                                                         \
  } while (0)

// ---- device scratch owned by a context (all pointers into the workspace) ----
struct Scratch {
  float *part;          // partial gradient rows
  float *part2;         // second level of the snapshot pass's fold: [fold_slices][d]
  double *part_loss;    // per-workgroup loss partials
  double *stat_part;    // [(N+1)][stat_slots][4]
  double *stats;        // [(N+1)][4]
  QParams *qparams;     // [(N+1)]
  uint32_t *flags;      // [4]: [0] = a non-finite value was seen
  uint32_t *n_clipped;  // [N]
  float *z_snap;        // [n]
  float *mu;            // [d]
  float *w;             // [d]   inner iterate x_t (Alg. 1) / x_{k+1} (Alg. 2, 3)
  float *U;             // [(N+1)][d_pad]; row N holds the shared-batch difference
  uint32_t *packed;     // [N][W]
  float *delta;         // [N]
  float *u_avg;         // [d]
  float *ysum;          // [d]   running weighted sum of y (Alg. 2 step 15 / Alg. 3 step 5)
  double *f_scalar;     // [1]
  RowPlan *csr_plan;               // sparse CSR epoch: [m][N][B] sampled rows of the epoch
  float *warm_sink;                // [1] never written in practice: keeps the cache-warming loads alive
  unsigned long long *clip_total;  // [1] clipped coordinates summed over an evaluation run
  HuffEntry *huff_table;           // [2^bits] codeword table of the entropy coder
  uint32_t *huff_seg_bits;         // [d_pad/32] encoded bits per 32-coordinate segment
  unsigned long long *huff_off;    // [d_pad/32] stream position of each segment
  unsigned long long *huff_meta;   // [2] total bits, bad-symbol flag
  float *csr_tail;      // [d_pad] CSR snapshot pass: accumulator of the non-privatised columns
  // column-major copy of the CSR entries whose column is not in the head (built by lpc_create)
  int32_t *csc_ptr;     // [d+4]: column extents (head columns are empty), the longest column, two build counters
  int32_t *csc_cursor;  // [d+1] build scratch, then the lists of medium and long tail columns
  int32_t *csc_rows;    // [nnz] row index per entry, ascending inside a column
  float *csc_vals;      // [nnz]
  float *csc_coef;      // [n] per-row loss slopes of the snapshot pass
  float *report_delta;       // [m][N] scale factors of an epoch run by lpc_epoch_report
  uint32_t *report_nclip;    // [m][N] its clip counts
  unsigned long long *report_out;  // [2] their reduction
  float *w2;            // [d] second buffer of the inner iterate (form 2 reads one and writes the other)
  float *z2;            // [d] second buffer of ALPC-SVRG's z
  float *pd;            // two sets of [(N+1)*B][tiles] partial dots of the sampled rows with the iterate
  // resident inner loop (lpc_resident.hip)
  float *res_part;      // [8][slots][32][d_pad] partial vectors per die, worker slot and compute unit
  float *res_ubuf;      // [2][N][d_pad] (value, tag) words: u^i as the dies publish them (two sets, by iteration parity)
  float *res_jbuf;      // [2][8][d_pad] words: the dies' partial sums of the shared batch's difference
  double *res_stat;     // [2][N][32][8] words: slice statistics
  float *res_wbuf;      // [8][d_pad] words: the iterate, one copy per die
  uint32_t *res_ctl;    // tickets, barrier counters, flags, abort word
  unsigned long long *res_trace;  // [m][16] time stamps of the resident loop's phases (lpc_resident_trace)
  unsigned long long *iter_slots;  // two sets of [tiles][N][4] statistics exchanged between the workgroups of the
                                   // two-launch inner iteration (all ones = empty)
  uint32_t *touched;    // [N][bitmap_words] sparse inner iteration: one bit per 32-coordinate segment of u^i
  uint32_t *touched_parts;  // [N][parts-1][bitmap_words]: the same for the worker pass's workgroups 1..parts-1
  float *sparse_planes; // [N][parts-1][d_pad] sparse inner iteration: tail contributions of a worker's workgroups
                        // 1..parts-1 (workgroup 0 adds into the worker's row of U); zero outside touched segments
  // MLP instance: gathered inputs/labels and per-layer activations / deltas for the two parameter sets
  float *mlp_xb;        // [rows][dims[0]]
  float *mlp_yb;        // [rows]
  float *mlp_act;       // layer l (1..L) at mlp_act + act_off[l]: [2][rows][dims[l]]
  float *mlp_del;       // same layout as mlp_act
  double *mlp_loss;     // [rows] per-row losses of the snapshot pass
  float *mlp_part;      // per-block partial sums of the snapshot pass (mlp_part_floats)
};

}  // namespace lpc

struct lpc_ctx {
  lpc_problem prob;
  lpc_config cfg;
  std::vector<int32_t> mlp_dims;
  int64_t n, d, d_pad, W, n_full;
  bool quant;             // bits < 32
  bool grad_ok;           // the gradient passes are built for this problem
  bool csr;               // rows are stored in CSR
  bool mlp;               // multi-layer perceptron instance
  int64_t mlp_rows;       // rows of a worker pass (N*B)
  int64_t mlp_cap;        // rows each of the two activation sets can hold (the snapshot pass uses both as one)
  std::vector<int64_t> mlp_woff, mlp_boff, mlp_act_off;  // per layer offsets
  // set only while an evaluation entry point (traced epoch, clip sweep) runs an epoch; all null otherwise
  float *trace_delta = nullptr;                // [m][N]
  uint32_t *trace_nclip = nullptr;             // [m][N]
  bool count_clipped = false;                  // add every message's clip count to s.clip_total
  uint64_t *trace_coded_host = nullptr;        // [m][N], HOST: entropy-coded size of every message
  int64_t mlp_act_floats;
  int64_t mlp_part_floats;
  int32_t full_grad_wgs;  // workgroups of the snapshot pass (= partial rows it writes)
  int32_t vr_parts;       // partial rows per worker written by the worker pass
  int32_t stat_slots;     // statistic partials per vector
  int32_t cus;            // compute units of the device (256 on MI355X)
  int32_t fold_slices;    // slices of the two-level fold of the snapshot pass's partial rows
  // form of the small-d dense inner iteration (lpc_tune): 0 = rows, fold, exchange (three launches); 1 = rows,
  // then fold + exchange in one launch whose workgroups wait for each other's statistics; 2 = column tiles fed by
  // partial dot products, then the exchange, which also leaves the next iteration's partial dots (two launches);
  // 3 = all m iterations in one resident launch (lpc_resident.hip)
  int32_t iter_form = 0;
  bool at_snapshot = false;    // set by lpc_epoch while it issues t = 0 of Alg. 1, where x_0 is the snapshot itself
  bool iter2_capable = false;  // the context's scratch holds what form 1 needs
  bool cols_capable = false;   // ... what form 2 needs
  bool res_capable = false;    // ... what form 3 (the resident inner loop) needs
  bool res_trace_on = false;   // the next resident launches leave their phase time stamps
  uint32_t res_tag = 0;        // tags handed to resident launches so far (each launch takes m + 1)
  int32_t iter_tile = 128, iter_threads = 512;  // launch shape of the second one
  uint32_t spin_limit = 1u << 15;               // polls a workgroup of it waits for the others' statistics
  bool csc_ready = false;  // the column-major tail copy exists (CSR snapshot pass without atomics)
  int32_t csc_medium = 0, csc_long = 0;  // tail columns served by 16 lanes / by a wavefront
  bool csr_sparse = false; // inner iterations of Alg. 1 keep u^i sparse (CSR rows that touch few columns)
  int32_t sparse_head = 0; // leading columns that every sparse pass visits densely
  int64_t bitmap_words = 0; // words per worker of the touched-segment bitmap
  size_t part_floats;
  void *workspace;
  size_t workspace_bytes;
  bool prof_on = false;   // kernel-class timing (lpc_profile_enable)
  std::vector<hipEvent_t> prof_start, prof_stop;
  std::vector<int> prof_cls;
  std::vector<char> prof_exact;  // the record is one kernel timed by its own dispatch
  lpc::Scratch s;
};

namespace lpc {

// ---- host-only logic (lpc_host.cpp) ----
lpc_status check_problem(const lpc_problem *p);
lpc_status check_config(const lpc_problem *p, const lpc_config *c);

// ---- launchers (each validates nothing: the ABI layer has done that) ----

// Dense GLM passes (lpc_dense.hip)
bool dense_supported(int64_t d, int64_t ldx, const void *X);
int dense_full_grad_wgs(int64_t n, int64_t d, int cus);
int dense_vr_parts(int64_t d, int64_t ldx, const void *X, int32_t nvec, int32_t B, int cus, bool cached);
hipError_t launch_dense_full_grad(const lpc_ctx *c, const float *w, float *z, bool want_loss, int64_t n_rows,
                                  hipStream_t st);
// plus_shared: one more vector after the workers', drawn from the shared batch J (double sampling)
hipError_t launch_dense_vr_grad(const lpc_ctx *c, const float *w, const float *w_snap, const float *z_snap,
                                StreamKey key, uint32_t tag, int32_t worker_begin, int32_t worker_end,
                                bool plus_shared, hipStream_t st);

// the worker pass in column tiles, fed by partial dot products (small-d inner iteration)
bool dense_cols_supported(const lpc_ctx *c);
int dense_cols_tiles(const lpc_ctx *c);
int dense_dots_groups(const lpc_ctx *c, int32_t rows);
hipError_t launch_dense_dots(const lpc_ctx *c, const float *w, StreamKey key, int32_t worker_begin, int32_t nvec,
                             bool last_is_shared, uint32_t tag, float *pd, hipStream_t st);
hipError_t launch_dense_cols(const lpc_ctx *c, const float *z_snap, const float *pd, StreamKey key, uint32_t tag,
                             int32_t worker_begin, int32_t nvec, bool last_is_shared, float *U, int64_t ldu,
                             bool want_stats, int32_t stat_vec0, hipStream_t st);

// The inner loop of an epoch as one resident launch (lpc_resident.hip)
struct ResidentStep {
  const float *z_snap, *mu, *w_snap;
  float *w;              // in: the first iterate; out: the last
  float *y, *z, *ysum;   // Alg. 2, 3 only
  bool alpc;
  StreamKey key;         // of iteration 0
  uint32_t tag0;         // tags of the launch's words start above this number (grows from launch to launch)
  float step;            // Alg. 1: eta
  float step_y, alpha, tau1, tau2, theta;
};
bool resident_supported(const lpc_ctx *c);
size_t resident_part_floats(const lpc_ctx *c);
size_t resident_ubuf_floats(const lpc_ctx *c);
size_t resident_jbuf_floats(const lpc_ctx *c);
size_t resident_stat_doubles(const lpc_ctx *c);
size_t resident_wbuf_floats(const lpc_ctx *c);
size_t resident_ctl_words();
hipError_t launch_resident_epoch(const lpc_ctx *c, const ResidentStep &rs, hipStream_t st);

// CSR GLM passes (lpc_csr.hip)
int csr_head_columns(int64_t d);
int csr_full_grad_wgs(int64_t n);
hipError_t launch_zero(float *dst, int64_t n, hipStream_t st);
hipError_t build_csc_tail(lpc_ctx *c, hipStream_t st);
hipError_t launch_csr_full_grad(const lpc_ctx *c, const float *w, float *mu, float *z, bool want_loss, int64_t n_rows,
                                hipStream_t st);
int csr_sparse_parts(int32_t B);
int csr_sparse_head_columns(int64_t d);
// plus_shared: every iteration's plan holds one more vector, the shared batch J of Alg. 2 (N+1 vectors of B rows)
hipError_t launch_csr_plan(const lpc_ctx *c, const float *z_snap, StreamKey key0, bool plus_shared, hipStream_t st);
hipError_t launch_csr_vr_sparse(const lpc_ctx *c, const float *w, const float *w_snap, const float *z_snap,
                                StreamKey key, const RowPlan *plan, int32_t nvec, hipStream_t st);
hipError_t launch_sparse_stats(const lpc_ctx *c, int32_t nvec, hipStream_t st);
// share_delta: every worker quantizes with the largest of the N scale factors (Sec. 4.2 schemes (b), (c))
hipError_t launch_sparse_quantize(const lpc_ctx *c, StreamKey key, bool share_delta, hipStream_t st);
hipError_t launch_sparse_receive_prox(const lpc_ctx *c, const float *mu, float step, float *w, hipStream_t st);
hipError_t launch_csr_vr_grad(const lpc_ctx *c, const float *w, const float *w_snap, const float *z_snap,
                              StreamKey key, uint32_t tag, int32_t worker_begin, int32_t worker_end, float *U,
                              hipStream_t st);

// MLP instance (lpc_gemm.hip, lpc_mlp.hip)
hipError_t launch_gemm(const GemmArgs &g, hipStream_t st);
bool gemm_takes_matrix_cores(const GemmArgs &g);  // false: the vector-unit path (no statistic partials)
int gemm_tiles(const GemmArgs &g);
bool gemm_takes_skinny_short(const GemmArgs &g);
int gemm_skinny_short_slots(const GemmArgs &g);                 // statistic partials a matrix-core launch writes per batch item
// Rows per block of the MLP snapshot pass's reductions over rows (bias column sums, weight gradients formed on
// the vector units): a chunk is cut into blocks that are summed side by side, one partial per block, and the
// partials are folded by a second, small column sum; a lone launch over thousands of rows would occupy 1-16 CUs.
constexpr int kSnapBlock = 256;
constexpr int kSnapWide = 2048;  // rows per block of its weight-gradient products on the matrix cores
// 0 if lens[0..nsym) (each in [0, 32]) are the lengths of a prefix code, and then table[k] holds symbol k's
// canonical codeword; -1 otherwise.
int huffman_canonical_table(const int32_t *lens, int32_t nsym, HuffEntry *table);
hipError_t launch_huffman_measure(const lpc_ctx *c, const uint32_t *words, hipStream_t st);
hipError_t launch_huffman_emit(const lpc_ctx *c, const uint32_t *words, uint32_t *out, int64_t out_words,
                               hipStream_t st);
hipError_t launch_epoch_report(const float *delta, const uint32_t *nclip, int64_t n, unsigned long long *out,
                               hipStream_t st);
hipError_t launch_accumulate_clipped(const uint32_t *n_clipped, int32_t N, unsigned long long *total, hipStream_t st);
void mlp_plan(lpc_ctx *c);
hipError_t launch_mlp_clear_padding(const lpc_ctx *c, hipStream_t st);  // padding of the context's own U rows  // fills the offsets and sizes above
hipError_t launch_mlp_full_grad(const lpc_ctx *c, const float *w, float *mu, double *f_out, int64_t n_rows,
                                hipStream_t st);
// stats_mode != kStatsNone: the statistics of the N rows of U come out of the producing kernels' epilogues
hipError_t launch_mlp_vr_grad(const lpc_ctx *c, const float *w, const float *w_snap, StreamKey key, uint32_t tag,
                              int32_t worker_begin, int32_t worker_end, float *U, int stats_mode, double *stats_out,
                              int32_t *stat_slots_used, hipStream_t st);

// Reductions, statistics, quantizer, receiver, prox (lpc_quant.hip)
// out[v][0..d_pad) = scale * sum_p part[(v*parts + p)*d + j] (zero beyond d), then statistics of each
// row and its quantizer parameters.  out / stats_out point at the first row of the launch; vec_begin
// selects the scratch slots.
hipError_t launch_reduce_parts(const lpc_ctx *c, const float *part, int32_t parts, float scale, float *out,
                               int64_t ld_out, int32_t vec_begin, int32_t nvec, int stats_mode, double *stats_out,
                               hipStream_t st);
// stats_mode values of launch_reduce_parts
constexpr int kStatsNone = 0, kStatsFinal = 1, kStatsPartial = 2;
bool fused_exchange_supported(const lpc_ctx *c);
int reduce_parts_waves(const lpc_ctx *c, int32_t parts, int32_t nvec);
struct AlpcStep;
hipError_t launch_cols_exchange(const lpc_ctx *c, const float *U, StreamKey key, uint32_t *packed, float *delta_out,
                                const float *mu, float step, const float *w_in, float *w_out, const AlpcStep *al,
                                const float *z_in, float *next_pd, hipStream_t st);
bool fused_iter_supported(const lpc_ctx *c);
int64_t fused_iter_slot_words(const lpc_ctx *c);
hipError_t launch_fused_iter_reset(const lpc_ctx *c, hipStream_t st);
hipError_t launch_fused_iter(const lpc_ctx *c, StreamKey key, uint32_t *packed, float *delta_out, const float *mu,
                             float step, float *w, const AlpcStep *al, hipStream_t st);
hipError_t launch_fused_exchange(const lpc_ctx *c, const float *U, int32_t nslots, StreamKey key, uint32_t *packed,
                                 float *delta_out, const float *mu, float step, float *w, float *u_avg_out,
                                 hipStream_t st);
// Alg. 2 steps 13-15 and the next step 6 as the epilogue of the exchange launch
struct AlpcStep {
  const float *x, *u_hat, *w_snap, *mu;
  float *y, *z, *ysum, *x_next;
  float step_y, alpha, weight, tau1, tau2;
  int first;
};
hipError_t launch_fused_exchange_alpc(const lpc_ctx *c, const float *U, int32_t nslots, StreamKey key,
                                      uint32_t *packed, float *delta_out, const AlpcStep &al, hipStream_t st);
// statistic partials of up to 8 column ranges [begin, begin+len) of nvec rows of U (one workgroup each), as slots
// slot0 .. slot0+nranges-1; then, for kStatsFinal, the fold of all nslots partials per vector
struct StatRange {
  int64_t begin[8], len[8];
  int32_t n;
};
hipError_t launch_range_stats(const lpc_ctx *c, const float *U, int64_t ld, int32_t vec_begin, int32_t nvec,
                              const StatRange &ranges, int32_t slot0, hipStream_t st);
hipError_t launch_finalize_stats(const lpc_ctx *c, int32_t vec_begin, int32_t nvec, int32_t nslots, double *stats_out,
                                 hipStream_t st);
hipError_t launch_vector_stats(const lpc_ctx *c, const float *U, int64_t ld, int32_t vec_begin, int32_t nvec,
                               double *stats_out, int stats_mode, int32_t *slots_used, hipStream_t st);
hipError_t launch_prepare_qparams(const lpc_ctx *c, const double *stats, const float *delta_in, int32_t nvec,
                                  hipStream_t st);
hipError_t launch_quantize(const lpc_ctx *c, const float *U, StreamKey key, uint32_t *packed, float *delta_out,
                           uint32_t *n_clipped, hipStream_t st);
hipError_t launch_dequantize_avg(const lpc_ctx *c, const uint32_t *packed, const float *delta, float *u_avg,
                                 hipStream_t st);
hipError_t launch_plain_avg(const lpc_ctx *c, const float *U, float *u_avg, hipStream_t st);
// schemes (b)/(c): unify the scale factors of vectors 0..nvec-1 to their maximum; integer-sum receiver
hipError_t launch_share_delta(const lpc_ctx *c, int32_t nvec, float *delta_out, hipStream_t st);
hipError_t launch_dequantize_shared(const lpc_ctx *c, const uint32_t *packed, const float *delta, bool requant,
                                    StreamKey key, float *u_avg, hipStream_t st);
hipError_t launch_prox(const lpc_ctx *c, float *w, const float *u_avg, const float *mu, float step, hipStream_t st);
// fused receiver + prox of Alg. 1: w <- prox(w - eta*(avg + mu)); optionally also stores the average
hipError_t launch_dequantize_prox(const lpc_ctx *c, const uint32_t *packed, const float *delta, const float *mu,
                                  float step, float *w, float *u_avg_out, hipStream_t st);
hipError_t launch_finish_full_grad(const lpc_ctx *c, int32_t parts, int64_t cols, float scale, float *mu,
                                   double *f_out, bool want_loss, hipStream_t st);
hipError_t launch_copy(float *dst, const float *src, int64_t n, hipStream_t st);
hipError_t launch_fill_u32(uint32_t *dst, uint32_t v, int64_t n, hipStream_t st);
// ALPC-SVRG element-wise steps (Alg. 2 steps 6, 13-15)
hipError_t launch_alpc_couple(const lpc_ctx *c, const float *z, const float *w_snap, const float *y, float tau1,
                              float tau2, float *x, hipStream_t st);
hipError_t launch_alpc_update(const lpc_ctx *c, const float *x, const float *u_avg, const float *u_hat,
                              const float *mu, float step_y, float alpha, float weight, bool first, float *y,
                              float *z, float *ysum, hipStream_t st);
// Alg. 2 steps 13-15 and the next step 6 over d coordinates, reading the average from the context's u_avg; clears u_hat
hipError_t launch_alpc_update_couple(const lpc_ctx *c, const AlpcStep &al, hipStream_t st);
hipError_t launch_scale_to(const lpc_ctx *c, const float *src, float scale, float *dst, hipStream_t st);
hipError_t launch_objective_reg(const lpc_ctx *c, const float *w, double *acc, hipStream_t st);
// evaluators (Sec. 3.3 gradient mapping; Sec. 6.1 entropy coding of the code stream)
hipError_t launch_gradient_mapping(const lpc_ctx *c, const float *w, const float *grad, double eta, double *out,
                                   hipStream_t st);
hipError_t launch_code_histogram(const uint32_t *words, int64_t d, int32_t bits, uint64_t *counts, hipStream_t st);
uint64_t huffman_code_lengths(const uint64_t *counts, int32_t nsym, int32_t *lens);

}  // namespace lpc
