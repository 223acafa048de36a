// C ABI of the library: argument checking, workspace layout, and the host-side
// sequencing of the kernels for each call of include/lpc.h.  No arithmetic of
// the method lives here except the scalar parameter rules of Alg. 2 / Alg. 3.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstring>
#include <mutex>
#include <new>

#include "lpc_internal.h"

using namespace lpc;

thread_local lpc::LaunchTimer *lpc::g_launch_timer = nullptr;

namespace {

inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline lpc_status dev(hipError_t e) { return e == hipSuccess ? LPC_OK : LPC_EDEVICE; }
inline hipStream_t as_stream(void *s) { return (hipStream_t)s; }

bool is_csr(const lpc_problem &p) { return p.X == nullptr; }

// Optional timing of kernel classes with HIP events on the launch stream (benchmarks only; the
// events cost a little pipeline time, so the hot path leaves this off).  single = the scope issues exactly ONE
// kernel, through LPC_LAUNCH_TIMED: that launch then carries the two events itself (dispatch begin / end).
struct ProfScope {
  lpc_ctx *c;
  hipStream_t st;
  hipEvent_t stop = nullptr;
  bool single;
  LaunchTimer timer;
  ProfScope(lpc_ctx *ctx, int cls, hipStream_t s, bool single_kernel = false) : c(ctx), st(s), single(single_kernel) {
    if (!c->prof_on) return;
    hipEvent_t start = nullptr;
    if (hipEventCreate(&start) != hipSuccess || hipEventCreate(&stop) != hipSuccess) { stop = nullptr; return; }
    c->prof_start.push_back(start);
    c->prof_stop.push_back(stop);
    c->prof_cls.push_back(cls);
    c->prof_exact.push_back(single ? 1 : 0);
    if (single) {
      timer.start = start; timer.stop = stop;
      g_launch_timer = &timer;
    } else {
      (void)hipEventRecord(start, st);
    }
  }
  ~ProfScope() {
    if (!stop) return;
    if (single) g_launch_timer = nullptr;
    else (void)hipEventRecord(stop, st);
  }
};

// Computes sizes; when base != nullptr also assigns the scratch pointers.
size_t layout(lpc_ctx *c, char *base) {
  size_t off = 0;
  auto take = [&](size_t bytes) -> char * {
    char *p = base ? base + off : nullptr;
    off += round_up(bytes, 256);
    return p;
  };
  const int64_t N1 = (int64_t)c->cfg.N + 1;
  Scratch &s = c->s;
  s.part = (float *)take(c->part_floats * sizeof(float));
  s.part2 = (float *)take((size_t)c->fold_slices * c->d * sizeof(float));
  s.part_loss = (double *)take((size_t)c->full_grad_wgs * sizeof(double));
  s.stat_part = (double *)take((size_t)N1 * c->stat_slots * 4 * sizeof(double));
  s.stats = (double *)take((size_t)N1 * 4 * sizeof(double));
  s.qparams = (QParams *)take((size_t)N1 * sizeof(QParams));
  s.flags = (uint32_t *)take(4 * sizeof(uint32_t));
  s.n_clipped = (uint32_t *)take((size_t)N1 * sizeof(uint32_t));
  s.z_snap = (float *)take((size_t)c->n * sizeof(float));
  s.mu = (float *)take((size_t)c->d * sizeof(float));
  s.w = (float *)take((size_t)c->d * sizeof(float));
  s.U = (float *)take((size_t)N1 * c->d_pad * sizeof(float));
  s.packed = (uint32_t *)take((size_t)c->cfg.N * (c->quant ? c->W : 1) * sizeof(uint32_t));
  s.delta = (float *)take((size_t)N1 * sizeof(float));
  s.u_avg = (float *)take((size_t)c->d * sizeof(float));
  s.ysum = (float *)take((size_t)c->d * sizeof(float));
  s.f_scalar = (double *)take(sizeof(double));
  s.clip_total = (unsigned long long *)take(sizeof(unsigned long long));
  {
    const size_t syms = c->quant ? (size_t)1 << c->cfg.bits : 1, segs = (size_t)(c->d_pad / 32);
    s.huff_table = (HuffEntry *)take(syms * sizeof(HuffEntry));
    s.huff_seg_bits = (uint32_t *)take((c->quant ? segs : 1) * sizeof(uint32_t));
    s.huff_off = (unsigned long long *)take((c->quant ? segs : 1) * sizeof(unsigned long long));
    s.huff_meta = (unsigned long long *)take(2 * sizeof(unsigned long long));
  }
  s.csr_tail = (float *)take((c->csr ? (size_t)c->d_pad : 4) * sizeof(float));
  s.csc_ptr = (int32_t *)take((c->csr ? (size_t)c->d + 4 : 4) * sizeof(int32_t));
  s.csc_cursor = (int32_t *)take((c->csr ? (size_t)c->d + 1 : 4) * sizeof(int32_t));
  s.csc_rows = (int32_t *)take((c->csr ? (size_t)c->prob.nnz : 4) * sizeof(int32_t));
  s.csc_vals = (float *)take((c->csr ? (size_t)c->prob.nnz : 4) * sizeof(float));
  s.csc_coef = (float *)take((c->csr ? (size_t)c->n : 4) * sizeof(float));
  s.csr_plan = (RowPlan *)take((c->csr_sparse ? (size_t)c->cfg.m * N1 * c->cfg.B : 1) * sizeof(RowPlan));
  s.warm_sink = (float *)take(sizeof(float));
  s.touched = (uint32_t *)take((c->csr_sparse ? (size_t)N1 * c->bitmap_words : 4) * sizeof(uint32_t));
  {
    const size_t extra = c->csr_sparse ? (size_t)(csr_sparse_parts(c->cfg.B) - 1) : 0;
    s.sparse_planes = (float *)take((extra ? (size_t)N1 * extra * c->d_pad : 4) * sizeof(float));
    s.touched_parts = (uint32_t *)take((extra ? (size_t)N1 * extra * c->bitmap_words : 4) * sizeof(uint32_t));
  }
  s.report_delta = (float *)take((size_t)c->cfg.m * c->cfg.N * sizeof(float));
  s.report_nclip = (uint32_t *)take((size_t)c->cfg.m * c->cfg.N * sizeof(uint32_t));
  s.report_out = (unsigned long long *)take(2 * sizeof(unsigned long long));
  s.w2 = (float *)take((c->cols_capable ? (size_t)c->d : 4) * sizeof(float));
  s.z2 = (float *)take((c->cols_capable ? (size_t)c->d : 4) * sizeof(float));
  s.pd = (float *)take((c->cols_capable ? 2 * (size_t)N1 * c->cfg.B * dense_cols_tiles(c) : 4) * sizeof(float));
  s.res_part = (float *)take((c->res_capable ? resident_part_floats(c) : 4) * sizeof(float));
  s.res_ubuf = (float *)take((c->res_capable ? resident_ubuf_floats(c) : 4) * sizeof(float));
  s.res_jbuf = (float *)take((c->res_capable ? resident_jbuf_floats(c) : 4) * sizeof(float));
  s.res_stat = (double *)take((c->res_capable ? resident_stat_doubles(c) : 1) * sizeof(double));
  s.res_wbuf = (float *)take((c->res_capable ? resident_wbuf_floats(c) : 4) * sizeof(float));
  s.res_ctl = (uint32_t *)take((c->res_capable ? resident_ctl_words() : 4) * sizeof(uint32_t));
  s.res_trace = (unsigned long long *)take((c->res_capable ? (size_t)c->cfg.m * 16 : 1) * sizeof(unsigned long long));
  s.iter_slots = (unsigned long long *)take((c->iter2_capable ? (size_t)fused_iter_slot_words(c) : 1) * sizeof(unsigned long long));
  if (c->mlp) {
    s.mlp_xb = (float *)take((size_t)c->mlp_rows * c->mlp_dims[0] * sizeof(float));
    s.mlp_yb = (float *)take((size_t)c->mlp_rows * sizeof(float));
    s.mlp_act = (float *)take((size_t)c->mlp_act_floats * sizeof(float));
    s.mlp_del = (float *)take((size_t)c->mlp_act_floats * sizeof(float));
    s.mlp_loss = (double *)take((size_t)2 * c->mlp_cap * sizeof(double));
    s.mlp_part = (float *)take((size_t)c->mlp_part_floats * sizeof(float));
  }
  return off;
}

lpc_status fill_ctx(lpc_ctx *c, const lpc_problem *p, const lpc_config *cfg) {
  lpc_status st = check_problem(p);
  if (st != LPC_OK) return st;
  st = check_config(p, cfg);
  if (st != LPC_OK) return st;
  c->prob = *p;
  c->cfg = *cfg;
  if (p->loss == LPC_LOSS_MLP_SOFTMAX) {
    c->mlp_dims.assign(p->mlp_dims, p->mlp_dims + p->mlp_nlayers + 1);
    c->prob.mlp_dims = c->mlp_dims.data();
  }
  c->n = p->n;
  c->d = p->d;
  c->d_pad = lpc_d_pad(p->d);
  c->quant = cfg->bits < 32;
  c->W = c->quant ? lpc_words_per_msg(p->d, cfg->bits) : 0;
  c->n_full = cfg->n_full > 0 ? cfg->n_full : p->n;
  // The gradient passes exist for dense linear models whose rows fit the register tiling; for any
  // other problem the context still serves the quantizer / receiver / prox calls and the gradient
  // calls answer LPC_EUNSUPPORTED.
  c->grad_ok = p->loss != LPC_LOSS_MLP_SOFTMAX && !is_csr(*p) && dense_supported(p->d, p->ldx, p->X);
  c->cus = 256;  // MI355X
  c->csr = is_csr(*p);
  c->mlp = p->loss == LPC_LOSS_MLP_SOFTMAX;
  if (c->mlp) {
    mlp_plan(c);
    c->grad_ok = true;
    c->full_grad_wgs = 1;
    c->vr_parts = 1;
    c->part_floats = 64;
  } else if (c->csr) {
    c->grad_ok = true;
    c->full_grad_wgs = csr_full_grad_wgs(c->n_full);
    c->vr_parts = 1;
    c->part_floats = (size_t)c->full_grad_wgs * csr_head_columns(c->d);
    // u^i (and the shared batch's difference of Alg. 2) stays sparse when a batch touches a small part of the
    // d columns (about B*nnz/n entries against d coordinates)
    c->sparse_head = csr_sparse_head_columns(c->d);
    c->bitmap_words = (c->d_pad / 32 + 31) / 32;
    const double touched = (double)cfg->B * (double)p->nnz / (double)p->n;
    c->csr_sparse = c->quant && cfg->N <= 64 &&
                    p->d >= 4 * (int64_t)c->sparse_head && touched * 8.0 <= (double)p->d &&
                    csr_sparse_parts(cfg->B) <= 8;  // tail planes per worker the statistics pass can merge
    if (c->csr_sparse) {
      const size_t head_parts = (size_t)(cfg->N + 1) * csr_sparse_parts(cfg->B) * c->sparse_head;
      if (head_parts > c->part_floats) c->part_floats = head_parts;
    }
  } else if (c->grad_ok) {
    c->full_grad_wgs = dense_full_grad_wgs(c->n_full, c->d, c->cus);
    c->vr_parts = dense_vr_parts(c->d, p->ldx, p->X, cfg->N + (cfg->algo != LPC_ALGO_LPC ? 1 : 0), cfg->B, c->cus,
                                 c->n_full == c->n);
    const size_t a1 = (size_t)c->full_grad_wgs * c->d;
    const size_t a2 = (size_t)(cfg->N + 1) * c->vr_parts * c->d;
    c->part_floats = a1 > a2 ? a1 : a2;
  } else {
    c->full_grad_wgs = 1;
    c->vr_parts = 1;
    c->part_floats = 64;
  }
  c->fold_slices = (c->full_grad_wgs >= 32 && c->full_grad_wgs % 16 == 0) ? 16 : 1;
  c->stat_slots = (int32_t)((c->d_pad + 63) / 64);
  if (c->mlp) {
    // the MLP's statistic partials come per output tile of the weight-gradient products plus one per bias
    // vector (and per layer computed on the vector units): small layers need more slots than d_pad/64
    int64_t need = 0;
    for (int l = 0; l < p->mlp_nlayers; ++l)
      need += (int64_t)(c->mlp_dims[l] / 128 + 1) * (c->mlp_dims[l + 1] / 64 + 1) + 2 +
              (c->mlp_dims[l + 1] + 63) / 64 + (c->mlp_dims[l] + 63) / 64;  // + bias blocks, + a vector-unit product's
    if (need > c->stat_slots) c->stat_slots = (int32_t)need;
  }
  c->iter2_capable = fused_iter_supported(c);
  c->cols_capable = fused_exchange_supported(c) && dense_cols_supported(c);
  c->res_capable = resident_supported(c);
  // measured on MI355X (inner iterations/s, forms 0 / 1 / 2): d = 4096, N = 8, B = 64: 59.9 k / 50.6 k / 47.6 k;
  // d = 8192, N = 16 (+ shared batch), B = 64: 32.3 k / - / 20.2 k.  Form 1 pays about 3 us per trip of the statistics
  // through device-scope atomics; form 2 pays for reading the sampled rows a second time in 512-byte slices (its
  // exchange launch takes 13.4 / 29.3 us against 6.3 / 8.7 us).  Three launches stay the default.
  c->iter_form = 0;
  return LPC_OK;
}

StreamKey key_of(const lpc_ctx *c, uint32_t epoch, uint32_t iter) {
  StreamKey k;
  k.seed_lo = (uint32_t)(c->cfg.seed & 0xFFFFFFFFu);
  k.seed_hi = (uint32_t)(c->cfg.seed >> 32);
  k.epoch = epoch;
  k.iter = iter;
  return k;
}

#define LPC_TRY(expr)                 \
  do {                                \
    lpc_status _s = (expr);           \
    if (_s != LPC_OK) return _s;      \
  } while (0)
#define LPC_TRY_HIP(expr)                       \
  do {                                          \
    if ((expr) != hipSuccess) return LPC_EDEVICE; \
  } while (0)

// Alg. 1 step 4 into (mu, z), all on `st`
lpc_status full_grad_impl(lpc_ctx *c, const float *w, float *mu, float *z, double *f_out, int64_t n_rows,
                          hipStream_t st) {
  if (!c->grad_ok) return LPC_EUNSUPPORTED;
  hipError_t e;
  {
    ProfScope ps(c, LPC_PROF_FULL_ROWS, st, !c->mlp && !c->csr);
    if (c->mlp) return dev(launch_mlp_full_grad(c, w, mu, f_out, n_rows, st));
    e = c->csr ? launch_csr_full_grad(c, w, mu, z, f_out != nullptr, n_rows, st)
               : launch_dense_full_grad(c, w, z, f_out != nullptr, n_rows, st);
  }
  if (e != hipSuccess) return LPC_EDEVICE;
  ProfScope ps(c, LPC_PROF_FULL_FOLD, st);
  // dense: every column comes from the fold; CSR: the privatised head columns do
  const int64_t cols = c->csr ? csr_head_columns(c->d) : c->d;
  e = launch_finish_full_grad(c, c->full_grad_wgs, cols, (float)(1.0 / (double)n_rows), mu, f_out,
                              f_out != nullptr, st);
  return dev(e);
}

// Alg. 1 step 6 for workers [wb, we) (or the shared batch): U rows and statistics
lpc_status vr_grad_impl(lpc_ctx *c, const float *w, const float *w_snap, const float *z_snap, StreamKey key,
                        uint32_t tag, int32_t wb, int32_t we, float *U_row0, double *stats_row0, int stats_mode,
                        hipStream_t st, int32_t *stat_slots_used = nullptr) {
  if (!c->grad_ok) return LPC_EUNSUPPORTED;
  hipError_t e;
  const int32_t slot0 = (tag == kTagShared) ? c->cfg.N : wb;
  if (c->mlp) {
    // the products' epilogues leave the statistic partials; only their fold is a launch of its own
    ProfScope ps(c, LPC_PROF_VR_ROWS, st);
    return dev(launch_mlp_vr_grad(c, w, w_snap, key, tag, wb, we, U_row0, stats_mode, stats_row0, stat_slots_used, st));
  }
  if (c->csr) {
    {
      ProfScope ps(c, LPC_PROF_VR_ROWS, st);
      e = launch_csr_vr_grad(c, w, w_snap, z_snap, key, tag, wb, we, U_row0, st);
    }
    if (e != hipSuccess) return LPC_EDEVICE;
    if (stats_mode == kStatsNone) return LPC_OK;
    ProfScope ps(c, LPC_PROF_VR_FOLD, st);
    return dev(launch_vector_stats(c, U_row0, c->d_pad, slot0, we - wb, stats_row0, stats_mode, stat_slots_used, st));
  }
  if (c->iter_form == 2 && c->cols_capable && z_snap) {
    // column tiles: the partial dots of the sampled rows with w, then u^i tile by tile with its statistic partials
    const bool shared = tag == kTagShared;
    LPC_TRY_HIP(launch_dense_dots(c, w, key, wb, we - wb, shared, tag, c->s.pd, st));
    {
      ProfScope ps(c, LPC_PROF_VR_ROWS, st, true);
      LPC_TRY_HIP(launch_dense_cols(c, z_snap, c->s.pd, key, tag, wb, we - wb, shared, U_row0, c->d_pad,
                                    stats_mode != kStatsNone, slot0, st));
    }
    if (stat_slots_used) *stat_slots_used = dense_cols_tiles(c);
    if (stats_mode == kStatsFinal)
      LPC_TRY_HIP(launch_finalize_stats(c, slot0, we - wb, dense_cols_tiles(c), stats_row0, st));
    return LPC_OK;
  }
  {
    ProfScope ps(c, LPC_PROF_VR_ROWS, st, true);
    e = launch_dense_vr_grad(c, w, w_snap, z_snap, key, tag, wb, we, false, st);
  }
  if (e != hipSuccess) return LPC_EDEVICE;
  ProfScope ps(c, LPC_PROF_VR_FOLD, st, stats_mode != kStatsFinal);
  e = launch_reduce_parts(c, c->s.part, c->vr_parts, (float)(1.0 / (double)c->cfg.B), U_row0, c->d_pad, slot0,
                          we - wb, stats_mode, stats_row0, st);
  if (stat_slots_used) *stat_slots_used = (int32_t)((c->d_pad + 63) / 64);
  return dev(e);
}

struct AlpcParams {
  float tau1, tau2, alpha, theta;
};

// Theorem 3 (Alg. 2) and Alg. 3 step 3; non-zero config fields override the rules.
lpc_status alpc_params(const lpc_ctx *c, uint32_t epoch, AlpcParams *out) {
  const lpc_config &g = c->cfg;
  const double L = (double)g.L;
  const double sigma = g.sigma > 0.0f ? (double)g.sigma : (double)c->prob.lambda2;
  double zeta = 1.0 / ((double)g.N * (double)g.B);
  if (c->quant) {
    const double lam = g.clip_mode == LPC_CLIP_LAMBDA ? (double)g.clip : 1.0;
    const double levels = (double)((1 << (g.bits - 1)) - 1);
    zeta += (double)c->d * lam * lam / (4.0 * levels * levels);
  }
  double t2 = g.tau2 > 0.0f ? (double)g.tau2 : 5.0 * zeta / 3.0 + 1.0 / (2.0 * (double)g.B);
  if (t2 > 0.5) t2 = 0.5;
  double t1, a, th;
  if (g.algo == LPC_ALGO_ALPC_SC) {
    t1 = g.tau1 > 0.0f ? (double)g.tau1 : std::sqrt((double)g.m * sigma / (6.0 * L));
    if (t1 > 0.5) t1 = 0.5;
    if (!(t1 > 0.0)) return LPC_EINVAL;
    a = g.alpha > 0.0f ? (double)g.alpha : 1.0 / (6.0 * t1 * L);
    th = 1.0 + a * sigma;
  } else {
    t1 = 2.0 / ((double)epoch + 4.0);
    a = g.alpha > 0.0f ? (double)g.alpha / t1 : 1.0 / (6.0 * L * t1);
    th = 1.0;
  }
  out->tau1 = (float)t1; out->tau2 = (float)t2; out->alpha = (float)a; out->theta = (float)th;
  return LPC_OK;
}

// Evaluation runs only: row t of the traces <- this iteration's scale factors and clip counts (zeros with
// quantization off), and the clip counts into the running total.
lpc_status record_iteration(lpc_ctx *c, int32_t t, hipStream_t st) {
  Scratch &s = c->s;
  const int32_t N = c->cfg.N;
  const size_t row = (size_t)t * (size_t)N;
  if (!c->quant) {
    if (c->trace_delta) LPC_TRY_HIP(launch_zero(c->trace_delta + row, N, st));
    if (c->trace_nclip) LPC_TRY_HIP(launch_fill_u32(c->trace_nclip + row, 0u, N, st));
    if (c->trace_coded_host)
      for (int32_t i = 0; i < N; ++i) c->trace_coded_host[row + (size_t)i] = 32ull * (uint64_t)c->d;
    return LPC_OK;
  }
  if (c->trace_coded_host) {
    // histogram of each message on the device, code lengths on the host (the table's scratch holds the counts)
    const int32_t nsym = 1 << c->cfg.bits;
    uint64_t *counts_dev = reinterpret_cast<uint64_t *>(s.huff_table);
    std::vector<uint64_t> counts((size_t)nsym);
    for (int32_t i = 0; i < N; ++i) {
      LPC_TRY_HIP(launch_code_histogram(s.packed + (int64_t)i * c->W, c->d, c->cfg.bits, counts_dev, st));
      LPC_TRY_HIP(hipMemcpyAsync(counts.data(), counts_dev, sizeof(uint64_t) * (size_t)nsym, hipMemcpyDeviceToHost,
                                 st));
      LPC_TRY_HIP(hipStreamSynchronize(st));
      c->trace_coded_host[row + (size_t)i] = huffman_code_lengths(counts.data(), nsym, nullptr);
    }
  }
  if (c->trace_delta)
    LPC_TRY_HIP(hipMemcpyAsync(c->trace_delta + row, s.delta, sizeof(float) * (size_t)N, hipMemcpyDeviceToDevice, st));
  if (c->trace_nclip)
    LPC_TRY_HIP(hipMemcpyAsync(c->trace_nclip + row, s.n_clipped, sizeof(uint32_t) * (size_t)N,
                               hipMemcpyDeviceToDevice, st));
  if (c->count_clipped) LPC_TRY_HIP(launch_accumulate_clipped(s.n_clipped, N, s.clip_total, st));
  return LPC_OK;
}

// communication step 2 of one inner iteration followed by the update of Alg. 1
// (want_clip_counts: an evaluation run records them; the quantizer is quicker without)
lpc_status exchange_and_prox(lpc_ctx *c, StreamKey key, float *w, bool want_clip_counts, hipStream_t st) {
  Scratch &s = c->s;
  ProfScope ps(c, LPC_PROF_EXCHANGE, st);
  if (c->quant && c->cfg.scheme != LPC_SCHEME_A) {
    // schemes (b), (c): delta = max_i delta_i for every worker, integer sum at the receiver
    LPC_TRY_HIP(launch_share_delta(c, c->cfg.N, nullptr, st));
    LPC_TRY_HIP(launch_quantize(c, s.U, key, s.packed, s.delta, s.n_clipped, st));
    LPC_TRY_HIP(launch_dequantize_shared(c, s.packed, s.delta, c->cfg.scheme == LPC_SCHEME_C, key, s.u_avg, st));
    LPC_TRY_HIP(launch_prox(c, w, s.u_avg, s.mu, c->cfg.eta, st));
  } else if (c->quant) {
    LPC_TRY_HIP(launch_quantize(c, s.U, key, s.packed, s.delta, want_clip_counts ? s.n_clipped : nullptr, st));
    LPC_TRY_HIP(launch_dequantize_prox(c, s.packed, s.delta, s.mu, c->cfg.eta, w, nullptr, st));
  } else {
    LPC_TRY_HIP(launch_plain_avg(c, s.U, s.u_avg, st));
    LPC_TRY_HIP(launch_prox(c, w, s.u_avg, s.mu, c->cfg.eta, st));
  }
  return LPC_OK;
}

}  // namespace

extern "C" {

size_t lpc_workspace_bytes(const lpc_problem *problem, const lpc_config *config) {
  lpc_ctx tmp{};
  if (fill_ctx(&tmp, problem, config) != LPC_OK) return 0;
  return layout(&tmp, nullptr);
}

lpc_status lpc_create(lpc_ctx **ctx_out, const lpc_problem *problem, const lpc_config *config, void *workspace,
                      size_t workspace_bytes) {
  if (!ctx_out) return LPC_ENULL;
  *ctx_out = nullptr;
  lpc_ctx *c = new (std::nothrow) lpc_ctx{};
  if (!c) return LPC_EDEVICE;
  lpc_status st = fill_ctx(c, problem, config);
  if (st != LPC_OK) { delete c; return st; }
  const size_t need = layout(c, nullptr);
  if (!workspace || !aligned(workspace, 256) || workspace_bytes < need) { delete c; return LPC_EWORKSPACE; }
  layout(c, (char *)workspace);
  c->workspace = workspace;
  c->workspace_bytes = workspace_bytes;
  // flags and clip counts start at zero (contiguous, see layout())
  const size_t words = ((char *)c->s.z_snap - (char *)c->s.flags) / sizeof(uint32_t);
  if (launch_fill_u32(c->s.flags, 0u, (int64_t)words, nullptr) != hipSuccess ||
      (c->mlp && launch_mlp_clear_padding(c, nullptr) != hipSuccess) || hipStreamSynchronize(nullptr) != hipSuccess) {
    delete c;
    return LPC_EDEVICE;
  }
  if (c->res_capable) {
    // the resident loop's tagged words: no tag of a launch is zero, so zeroed words never pass for written ones
    const size_t words = ((char *)c->s.res_ctl - (char *)c->s.res_ubuf) / sizeof(uint32_t);
    if (launch_fill_u32(reinterpret_cast<uint32_t *>(c->s.res_ubuf), 0u, (int64_t)words, nullptr) != hipSuccess ||
        hipStreamSynchronize(nullptr) != hipSuccess) {
      delete c;
      return LPC_EDEVICE;
    }
  }
  if (c->csr && build_csc_tail(c, nullptr) != hipSuccess) {
    delete c;
    return LPC_EDEVICE;
  }
  *ctx_out = c;
  return LPC_OK;
}

void lpc_destroy(lpc_ctx *ctx) {
  if (!ctx) return;
  for (hipEvent_t e : ctx->prof_start) (void)hipEventDestroy(e);
  for (hipEvent_t e : ctx->prof_stop) (void)hipEventDestroy(e);
  delete ctx;
}

lpc_status lpc_tune(lpc_ctx *ctx, int32_t key, int64_t value) {
  if (!ctx) return LPC_ENULL;
  switch (key) {
    case LPC_TUNE_ITER_FORM:
      if (value < 0 || value > 3) return LPC_EINVAL;
      if ((value == 1 && !ctx->iter2_capable) || (value == 2 && !ctx->cols_capable) || (value == 3 && !ctx->res_capable))
        return LPC_EUNSUPPORTED;
      ctx->iter_form = (int32_t)value;
      return LPC_OK;
    case LPC_TUNE_ITER_TILE:
      if (value != 64 && value != 128) return LPC_EINVAL;
      ctx->iter_tile = (int32_t)value;
      return LPC_OK;
    case LPC_TUNE_ITER_THREADS:
      if (value != 256 && value != 512) return LPC_EINVAL;
      ctx->iter_threads = (int32_t)value;
      return LPC_OK;
    case LPC_TUNE_SPIN_LIMIT:
      if (value < 0 || value > (int64_t)(1 << 24)) return LPC_EINVAL;
      ctx->spin_limit = (uint32_t)value;
      return LPC_OK;
  }
  return LPC_EINVAL;
}

lpc_status lpc_resident_trace(lpc_ctx *ctx, int32_t on, uint64_t *stamps_out_host, void *stream) {
  if (!ctx) return LPC_ENULL;
  if (!ctx->res_capable) return LPC_EUNSUPPORTED;
  if (stamps_out_host) {
    hipStream_t st = as_stream(stream);
    LPC_TRY_HIP(hipMemcpyAsync(stamps_out_host, ctx->s.res_trace, sizeof(uint64_t) * 16 * (size_t)ctx->cfg.m,
                               hipMemcpyDeviceToHost, st));
    LPC_TRY_HIP(hipStreamSynchronize(st));
  }
  ctx->res_trace_on = on != 0;
  return LPC_OK;
}

lpc_status lpc_profile_enable(lpc_ctx *ctx, int32_t on) {
  if (!ctx) return LPC_ENULL;
  ctx->prof_on = on != 0;
  return LPC_OK;
}

lpc_status lpc_profile_read(lpc_ctx *ctx, double *ms_total, int64_t *launches, int32_t *exact, void *stream) {
  if (!ctx || !ms_total || !launches) return LPC_ENULL;
  LPC_TRY_HIP(hipStreamSynchronize(as_stream(stream)));
  for (int k = 0; k < LPC_PROF_NCLASS; ++k) { ms_total[k] = 0.0; launches[k] = 0; if (exact) exact[k] = 1; }
  for (size_t i = 0; i < ctx->prof_cls.size(); ++i) {
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, ctx->prof_start[i], ctx->prof_stop[i]) == hipSuccess) {
      ms_total[ctx->prof_cls[i]] += (double)ms;
      launches[ctx->prof_cls[i]] += 1;
      if (exact && !ctx->prof_exact[i]) exact[ctx->prof_cls[i]] = 0;
    }
    (void)hipEventDestroy(ctx->prof_start[i]);
    (void)hipEventDestroy(ctx->prof_stop[i]);
  }
  ctx->prof_start.clear(); ctx->prof_stop.clear(); ctx->prof_cls.clear(); ctx->prof_exact.clear();
  return LPC_OK;
}

lpc_status lpc_full_grad(lpc_ctx *ctx, const float *w, float *mu, float *z, double *f_out, void *stream) {
  if (!ctx || !w || !mu) return LPC_ENULL;
  if (!aligned(w, 16) || !aligned(mu, 16) || (z && !aligned(z, 4)) || (f_out && !aligned(f_out, 8)))
    return LPC_ESHAPE;
  return full_grad_impl(ctx, w, mu, z, f_out, ctx->n_full, as_stream(stream));
}

lpc_status lpc_worker_vr_grad(lpc_ctx *ctx, const float *w, const float *w_snap, const float *z_snap,
                              uint32_t epoch, uint32_t iter, int32_t kind, int32_t worker_begin, int32_t worker_end,
                              float *U, double *stats, void *stream) {
  if (!ctx || !w || !w_snap || !U) return LPC_ENULL;
  if (kind != LPC_BATCH_WORKER && kind != LPC_BATCH_SHARED) return LPC_EINVAL;
  if (worker_begin < 0 || worker_end <= worker_begin || worker_end > ctx->cfg.N) return LPC_EINVAL;
  if (!aligned(w, 16) || !aligned(w_snap, 16) || !aligned(U, 16) || (stats && !aligned(stats, 8)))
    return LPC_ESHAPE;
  const uint32_t tag = kind == LPC_BATCH_SHARED ? kTagShared : kTagBatch;
  const int32_t we = kind == LPC_BATCH_SHARED ? worker_begin + 1 : worker_end;
  return vr_grad_impl(ctx, w, w_snap, z_snap, key_of(ctx, epoch, iter), tag, worker_begin, we,
                      U + (int64_t)worker_begin * ctx->d_pad, stats ? stats + 4 * (int64_t)worker_begin : nullptr,
                      kStatsFinal, as_stream(stream));
}

lpc_status lpc_vector_stats(lpc_ctx *ctx, const float *U, int32_t nvec, double *stats, void *stream) {
  if (!ctx || !U || !stats) return LPC_ENULL;
  if (nvec <= 0 || nvec > ctx->cfg.N + 1) return LPC_EINVAL;
  if (!aligned(U, 16) || !aligned(stats, 8)) return LPC_ESHAPE;
  return dev(launch_vector_stats(ctx, U, ctx->d_pad, 0, nvec, stats, kStatsFinal, nullptr, as_stream(stream)));
}

lpc_status lpc_quantize_clip(lpc_ctx *ctx, const float *U, const double *stats, const float *delta_in,
                             uint32_t epoch, uint32_t iter, uint32_t *packed, float *delta_out, uint32_t *n_clipped,
                             void *stream) {
  if (!ctx || !U || !packed || !delta_out) return LPC_ENULL;
  if (!stats && !delta_in) return LPC_ENULL;
  if (!ctx->quant) return LPC_EINVAL;
  if (!aligned(U, 16) || !aligned(packed, 16) || (stats && !aligned(stats, 8))) return LPC_ESHAPE;
  hipStream_t st = as_stream(stream);
  LPC_TRY_HIP(launch_prepare_qparams(ctx, stats, delta_in, ctx->cfg.N, st));
  // the clip counts cost the quantizer a fifth of its time: taken only where the caller wants them
  LPC_TRY_HIP(launch_quantize(ctx, U, key_of(ctx, epoch, iter), packed, delta_out, n_clipped ? ctx->s.n_clipped : nullptr, st));
  if (n_clipped)
    LPC_TRY_HIP(hipMemcpyAsync(n_clipped, ctx->s.n_clipped, sizeof(uint32_t) * (size_t)ctx->cfg.N,
                               hipMemcpyDeviceToDevice, st));
  return LPC_OK;
}

lpc_status lpc_dequantize_avg(lpc_ctx *ctx, const uint32_t *packed, const float *delta, float *u_avg, void *stream) {
  if (!ctx || !packed || !delta || !u_avg) return LPC_ENULL;
  if (!ctx->quant) return LPC_EINVAL;
  if (!aligned(packed, 16) || !aligned(u_avg, 16)) return LPC_ESHAPE;
  return dev(launch_dequantize_avg(ctx, packed, delta, u_avg, as_stream(stream)));
}

lpc_status lpc_dequantize_shared(lpc_ctx *ctx, const uint32_t *packed, const float *delta, int32_t requantize,
                                 uint32_t epoch, uint32_t iter, float *u_avg, void *stream) {
  if (!ctx || !packed || !delta || !u_avg) return LPC_ENULL;
  if (!ctx->quant) return LPC_EINVAL;
  if (!aligned(packed, 16) || !aligned(u_avg, 16)) return LPC_ESHAPE;
  return dev(launch_dequantize_shared(ctx, packed, delta, requantize != 0, key_of(ctx, epoch, iter), u_avg,
                                      as_stream(stream)));
}

lpc_status lpc_exchange(lpc_ctx *ctx, const float *U, uint32_t epoch, uint32_t iter, uint32_t *packed,
                        float *delta_out, float *u_avg, void *stream) {
  if (!ctx || !U || !packed || !delta_out || !u_avg) return LPC_ENULL;
  if (!ctx->quant) return LPC_EINVAL;
  if (!aligned(U, 16) || !aligned(packed, 16) || !aligned(u_avg, 16)) return LPC_ESHAPE;
  hipStream_t st = as_stream(stream);
  const StreamKey key = key_of(ctx, epoch, iter);
  if (fused_exchange_supported(ctx)) {
    int32_t slots = 0;
    LPC_TRY_HIP(launch_vector_stats(ctx, U, ctx->d_pad, 0, ctx->cfg.N, nullptr, kStatsPartial, &slots, st));
    LPC_TRY_HIP(launch_fused_exchange(ctx, U, slots, key, packed, delta_out, nullptr, 0.0f, nullptr, u_avg, st));
    return LPC_OK;
  }
  LPC_TRY_HIP(launch_vector_stats(ctx, U, ctx->d_pad, 0, ctx->cfg.N, nullptr, kStatsFinal, nullptr, st));
  LPC_TRY_HIP(launch_quantize(ctx, U, key, packed, delta_out, ctx->s.n_clipped, st));
  LPC_TRY_HIP(launch_dequantize_avg(ctx, packed, delta_out, u_avg, st));
  return LPC_OK;
}

// ---- lpc_exchange for callers that cannot allocate ---------------------------------------------------------
// The scratch lpc_exchange takes from a context's workspace (statistic partials, statistics, quantizer
// parameters, clip counts, the non-finite flag) lives in a file-scope device array instead.  Every GPU the
// library runs on holds its own copy of the array at its own address until the process ends; host code reaches
// it only through the address hipGetSymbolAddress returns for the current device.
namespace {
constexpr int64_t kStaticMaxD = (int64_t)1 << 23;  // coordinates per vector
constexpr int32_t kStaticMaxN = 64;                // vectors
constexpr int32_t kStaticSlots = 256;              // statistic partials per vector (32768 coordinates each at the maximum)
constexpr size_t kStaticStatPart = (size_t)kStaticMaxN * kStaticSlots * 4 * sizeof(double);
constexpr size_t kStaticStats = (size_t)kStaticMaxN * 4 * sizeof(double);
constexpr size_t kStaticQParams = (size_t)kStaticMaxN * sizeof(QParams);
constexpr size_t kStaticClipped = (size_t)kStaticMaxN * sizeof(uint32_t);
constexpr size_t kStaticFlags = 256;
constexpr size_t kStaticBytes = kStaticStatPart + kStaticStats + kStaticQParams + kStaticClipped + kStaticFlags;
static_assert(kStaticStatPart % 256 == 0 && kStaticStats % 256 == 0 && kStaticQParams % 256 == 0 &&
              kStaticClipped % 256 == 0, "every part of the static scratch starts 256-byte aligned");

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

constexpr int kMaxDevices = 64;
std::mutex static_mu;
unsigned char *static_ptr[kMaxDevices];  // the array's device address, per device; nullptr = not looked up yet

// Device address of `scratch` on the current device (looked up once per device; its flag word is cleared then).
lpc_status static_scratch(hipStream_t st, unsigned char **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LPC_EDEVICE;
  std::lock_guard<std::mutex> lock(static_mu);
  if (!static_ptr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LPC_EDEVICE;
    // a fill kernel, not a memset: the caller may be capturing the stream
    unsigned char *base = static_cast<unsigned char *>(p);
    if (launch_fill_u32(reinterpret_cast<uint32_t *>(base + kStaticBytes - kStaticFlags), 0u, kStaticFlags / 4, st) !=
        hipSuccess)
      return LPC_EDEVICE;
    static_ptr[dev] = base;
  }
  *out = static_ptr[dev];
  return LPC_OK;
}
}  // namespace

lpc_status lpc_exchange_static(int64_t d, int32_t N, int32_t bits, int32_t clip_mode, float clip, uint64_t seed,
                               const float *U, uint32_t epoch, uint32_t iter, uint32_t *packed, float *delta_out,
                               float *u_avg, uint32_t *flags_out, void *stream) {
  if (!U || !packed || !delta_out || !u_avg) return LPC_ENULL;
  if (d <= 0 || N <= 0) return LPC_ESHAPE;
  if (d > kStaticMaxD || N > kStaticMaxN) return LPC_EWORKSPACE;  // beyond what the static scratch holds
  if (bits < 2 || bits > 16) return LPC_EINVAL;
  if (clip_mode != LPC_CLIP_LAMBDA && clip_mode != LPC_CLIP_CSIGMA) return LPC_EINVAL;
  if (!(clip > 0.0f) || (clip_mode == LPC_CLIP_LAMBDA && clip > 1.0f)) return LPC_EINVAL;
  if (!aligned(U, 16) || !aligned(packed, 16) || !aligned(u_avg, 16) || !aligned(delta_out, 4) ||
      (flags_out && !aligned(flags_out, 4)))
    return LPC_ESHAPE;
  hipStream_t st = as_stream(stream);
  unsigned char *base = nullptr;
  LPC_TRY(static_scratch(st, &base));
  // a context on the stack that owns nothing: only the fields the exchange's launchers read
  lpc_ctx c{};
  c.cfg.N = N; c.cfg.B = 1; c.cfg.m = 1; c.cfg.bits = bits; c.cfg.clip_mode = clip_mode; c.cfg.clip = clip;
  c.cfg.seed = seed; c.cfg.scheme = LPC_SCHEME_A;
  c.d = d; c.d_pad = lpc_d_pad(d); c.W = lpc_words_per_msg(d, bits);
  c.quant = true; c.cus = 256; c.stat_slots = kStaticSlots;
  Scratch &s = c.s;
  s.stat_part = reinterpret_cast<double *>(base);
  s.stats = reinterpret_cast<double *>(base + kStaticStatPart);
  s.qparams = reinterpret_cast<QParams *>(base + kStaticStatPart + kStaticStats);
  s.n_clipped = reinterpret_cast<uint32_t *>(base + kStaticStatPart + kStaticStats + kStaticQParams);
  s.flags = flags_out ? flags_out : reinterpret_cast<uint32_t *>(base + kStaticBytes - kStaticFlags);
  const StreamKey key = key_of(&c, epoch, iter);
  if (fused_exchange_supported(&c)) {
    int32_t slots = 0;
    LPC_TRY_HIP(launch_vector_stats(&c, U, c.d_pad, 0, N, nullptr, kStatsPartial, &slots, st));
    LPC_TRY_HIP(launch_fused_exchange(&c, U, slots, key, packed, delta_out, nullptr, 0.0f, nullptr, u_avg, st));
    return LPC_OK;
  }
  LPC_TRY_HIP(launch_vector_stats(&c, U, c.d_pad, 0, N, nullptr, kStatsFinal, nullptr, st));
  LPC_TRY_HIP(launch_quantize(&c, U, key, packed, delta_out, s.n_clipped, st));
  LPC_TRY_HIP(launch_dequantize_avg(&c, packed, delta_out, u_avg, st));
  return LPC_OK;
}

lpc_status lpc_prox_step(lpc_ctx *ctx, float *w, const float *u_avg, const float *mu, float step, void *stream) {
  if (!ctx || !w || !u_avg || !mu) return LPC_ENULL;
  if (!(step > 0.0f)) return LPC_EINVAL;
  return dev(launch_prox(ctx, w, u_avg, mu, step, as_stream(stream)));
}

lpc_status lpc_epoch(lpc_ctx *ctx, float *w_snap, float *y, float *z, uint32_t epoch, void *stream) {
  if (!ctx || !w_snap) return LPC_ENULL;
  if (!aligned(w_snap, 16)) return LPC_ESHAPE;
  lpc_ctx *c = ctx;
  Scratch &s = c->s;
  hipStream_t st = as_stream(stream);
  const lpc_config &g = c->cfg;
  // evaluation runs take the unfused launches, whose quantizer reports the clip counts
  const bool tracing = c->trace_delta || c->trace_nclip || c->count_clipped || c->trace_coded_host;
  // communication step 1
  LPC_TRY(full_grad_impl(c, w_snap, s.mu, s.z_snap, nullptr, c->n_full, st));
  const float *zs = (c->n_full == c->n) ? s.z_snap : nullptr;  // margins cached only when every row was visited
  if (g.algo == LPC_ALGO_LPC) {
    LPC_TRY_HIP(launch_copy(s.w, w_snap, c->d, st));  // x_0 = x~
    const bool fused = fused_exchange_supported(c) && g.scheme == LPC_SCHEME_A && !tracing;
    const bool two = fused && c->iter_form == 1 && c->iter2_capable;
    const bool cols = fused && c->iter_form == 2 && c->cols_capable && zs != nullptr;
    const bool sparse = c->csr_sparse && !tracing;
    if (fused && c->iter_form == 3 && c->res_capable && zs != nullptr) {
      // all m inner iterations in one resident launch
      ResidentStep rs{};
      rs.z_snap = zs; rs.mu = s.mu; rs.w_snap = w_snap; rs.w = s.w; rs.alpc = false;
      rs.key = key_of(c, epoch, 0); rs.step = g.eta; rs.theta = 1.0f;
      rs.tag0 = c->res_tag; c->res_tag += (uint32_t)g.m + 1u;
      {
        ProfScope ps(c, LPC_PROF_RESIDENT, st);
        LPC_TRY_HIP(launch_resident_epoch(c, rs, st));
      }
      LPC_TRY_HIP(launch_copy(w_snap, s.w, c->d, st));  // x~ <- x_m
      return LPC_OK;
    }
    if (two) LPC_TRY_HIP(launch_fused_iter_reset(c, st));
    if (sparse) {
      // the sparse passes rely on U, the bitmap and the packed words being zero where nothing was written
      LPC_TRY_HIP(launch_zero(s.U, (int64_t)g.N * c->d_pad, st));
      if (csr_sparse_parts(g.B) > 1) {
        LPC_TRY_HIP(launch_zero(s.sparse_planes, (int64_t)g.N * (csr_sparse_parts(g.B) - 1) * c->d_pad, st));
        LPC_TRY_HIP(launch_fill_u32(s.touched_parts, 0u, (int64_t)g.N * (csr_sparse_parts(g.B) - 1) * c->bitmap_words, st));
      }
      LPC_TRY_HIP(launch_fill_u32(s.touched, 0u, (int64_t)g.N * c->bitmap_words, st));
      LPC_TRY_HIP(launch_fill_u32(s.packed, 0u, (int64_t)g.N * c->W, st));
      // the epoch's draws with each row's extent, label and snapshot margin, looked up once
      LPC_TRY_HIP(launch_csr_plan(c, zs, key_of(c, epoch, 0), false, st));
    }
    if (cols) {
      // two launches per inner iteration: column tiles of u^i from the partial dots; exchange + prox + the next
      // iteration's partial dots.  The iterate alternates between two buffers.
      float *wa = s.w, *wb = s.w2;
      const size_t pd_set = (size_t)(g.N + 1) * g.B * dense_cols_tiles(c);
      LPC_TRY_HIP(launch_dense_dots(c, wa, key_of(c, epoch, 0), 0, g.N, false, kTagBatch, s.pd, st));
      for (int32_t t = 0; t < g.m; ++t) {
        const StreamKey key = key_of(c, epoch, (uint32_t)t);
        float *pd_cur = s.pd + (size_t)(t & 1) * pd_set;
        float *pd_next = t + 1 < g.m ? s.pd + (size_t)((t + 1) & 1) * pd_set : nullptr;
        {
          ProfScope ps(c, LPC_PROF_VR_ROWS, st, true);
          c->at_snapshot = t == 0;  // x_0 = x~: u_0 is exactly zero
          const hipError_t e = launch_dense_cols(c, zs, pd_cur, key, kTagBatch, 0, g.N, false, s.U, c->d_pad, true, 0, st);
          c->at_snapshot = false;
          LPC_TRY_HIP(e);
        }
        ProfScope ps(c, LPC_PROF_EXCHANGE, st, true);
        LPC_TRY_HIP(launch_cols_exchange(c, s.U, key, s.packed, s.delta, s.mu, g.eta, wa, wb, nullptr, nullptr, pd_next,
                                         st));
        float *tmp = wa; wa = wb; wb = tmp;
      }
      LPC_TRY_HIP(launch_copy(w_snap, wa, c->d, st));  // x~ <- x_m
      return LPC_OK;
    }
    for (int32_t t = 0; t < g.m; ++t) {
      const StreamKey key = key_of(c, epoch, (uint32_t)t);
      if (sparse) {
        {
          ProfScope ps(c, LPC_PROF_VR_ROWS, st);
          LPC_TRY_HIP(launch_csr_vr_sparse(c, s.w, w_snap, zs, key, s.csr_plan + (int64_t)t * g.N * g.B, g.N, st));
        }
        {
          ProfScope ps(c, LPC_PROF_VR_FOLD, st);
          LPC_TRY_HIP(launch_sparse_stats(c, g.N, st));
        }
        ProfScope ps(c, LPC_PROF_EXCHANGE, st);
        if (g.scheme == LPC_SCHEME_A) {
          LPC_TRY_HIP(launch_sparse_quantize(c, key, false, st));
          LPC_TRY_HIP(launch_sparse_receive_prox(c, s.mu, g.eta, s.w, st));
        } else {
          // schemes (b), (c): one scale factor for all workers, integer sums at the receiver (and eq. (5) for (c));
          // the receiver is the dense one, so the consumed words and the bitmap are cleared by fills
          LPC_TRY_HIP(launch_sparse_quantize(c, key, true, st));
          LPC_TRY_HIP(launch_dequantize_shared(c, s.packed, s.delta, g.scheme == LPC_SCHEME_C, key, s.u_avg, st));
          LPC_TRY_HIP(launch_prox(c, s.w, s.u_avg, s.mu, g.eta, st));
          LPC_TRY_HIP(launch_fill_u32(s.packed, 0u, (int64_t)g.N * c->W, st));
          LPC_TRY_HIP(launch_fill_u32(s.touched, 0u, (int64_t)g.N * c->bitmap_words, st));
        }
      } else if (two) {
        // two launches per inner iteration: rows; fold + exchange + prox
        {
          ProfScope ps(c, LPC_PROF_VR_ROWS, st, true);
          LPC_TRY_HIP(launch_dense_vr_grad(c, s.w, w_snap, zs, key, kTagBatch, 0, g.N, false, st));
        }
        ProfScope ps(c, LPC_PROF_EXCHANGE, st, true);
        LPC_TRY_HIP(launch_fused_iter(c, key, s.packed, s.delta, s.mu, g.eta, s.w, nullptr, st));
      } else if (fused) {
        // three launches per inner iteration: rows, fold (+ statistic partials), exchange + prox
        int32_t slots = 0;
        LPC_TRY(vr_grad_impl(c, s.w, w_snap, zs, key, kTagBatch, 0, g.N, s.U, nullptr, kStatsPartial, st, &slots));
        ProfScope ps(c, LPC_PROF_EXCHANGE, st, true);
        LPC_TRY_HIP(launch_fused_exchange(c, s.U, slots, key, s.packed, s.delta, s.mu, g.eta, s.w, nullptr, st));
      } else {
        c->at_snapshot = t == 0;  // x_0 = x~ (only the column-tile worker pass needs telling)
        const lpc_status rc = vr_grad_impl(c, s.w, w_snap, zs, key, kTagBatch, 0, g.N, s.U, nullptr,
                                           c->quant ? kStatsFinal : kStatsNone, st);
        c->at_snapshot = false;
        LPC_TRY(rc);
        LPC_TRY(exchange_and_prox(c, key, s.w, tracing, st));
        if (tracing) LPC_TRY(record_iteration(c, t, st));
      }
    }
    LPC_TRY_HIP(launch_copy(w_snap, s.w, c->d, st));  // x~ <- x_m
    return LPC_OK;
  }
  if (!y || !z) return LPC_ENULL;
  if (!aligned(y, 16) || !aligned(z, 16)) return LPC_ESHAPE;
  AlpcParams ap;
  LPC_TRY(alpc_params(c, epoch, &ap));
  const float step_y = (float)(1.0 / (4.0 * (double)g.L));
  double weight = 1.0, wsum = 0.0;
  float *u_hat = s.U + (int64_t)g.N * c->d_pad;
  if (!c->csr && !c->mlp && fused_exchange_supported(c) && g.scheme == LPC_SCHEME_A && !tracing) {
    // three launches per inner iteration: the rows of the N workers AND of the shared batch J, their fold
    // (+ statistic partials), and the exchange with Alg. 2 steps 13-15 and the next step 6 as its epilogue
    LPC_TRY_HIP(launch_alpc_couple(c, z, w_snap, y, ap.tau1, ap.tau2, s.w, st));
    if (c->iter_form == 3 && c->res_capable && zs != nullptr) {
      // all m inner iterations in one resident launch; the weights of Alg. 2 step 15 follow the same recurrence there
      ResidentStep rs{};
      rs.z_snap = zs; rs.mu = s.mu; rs.w_snap = w_snap; rs.w = s.w; rs.y = y; rs.z = z; rs.ysum = s.ysum; rs.alpc = true;
      rs.key = key_of(c, epoch, 0); rs.step_y = step_y; rs.alpha = ap.alpha; rs.tau1 = ap.tau1; rs.tau2 = ap.tau2;
      rs.theta = ap.theta;
      rs.tag0 = c->res_tag; c->res_tag += (uint32_t)g.m + 1u;
      {
        ProfScope ps(c, LPC_PROF_RESIDENT, st);
        LPC_TRY_HIP(launch_resident_epoch(c, rs, st));
      }
      for (int32_t t = 0; t < g.m; ++t) {
        wsum += weight;
        weight *= (double)ap.theta;
      }
      LPC_TRY_HIP(launch_scale_to(c, s.ysum, (float)(1.0 / wsum), w_snap, st));
      return LPC_OK;
    }
    if (c->iter_form == 2 && c->cols_capable && zs != nullptr) {
      // two launches per inner iteration, as for Alg. 1; x and z alternate between two buffers each
      float *xa = s.w, *xb = s.w2, *za = z, *zb = s.z2;
      const size_t pd_set = (size_t)(g.N + 1) * g.B * dense_cols_tiles(c);
      LPC_TRY_HIP(launch_dense_dots(c, xa, key_of(c, epoch, 0), 0, g.N + 1, true, kTagBatch, s.pd, st));
      for (int32_t t = 0; t < g.m; ++t) {
        const StreamKey key = key_of(c, epoch, (uint32_t)t);
        float *pd_cur = s.pd + (size_t)(t & 1) * pd_set;
        float *pd_next = t + 1 < g.m ? s.pd + (size_t)((t + 1) & 1) * pd_set : nullptr;
        {
          ProfScope ps(c, LPC_PROF_VR_ROWS, st, true);
          LPC_TRY_HIP(launch_dense_cols(c, zs, pd_cur, key, kTagBatch, 0, g.N + 1, true, s.U, c->d_pad, true, 0, st));
        }
        AlpcStep al{};
        al.x = xa; al.u_hat = u_hat; al.w_snap = w_snap; al.mu = s.mu;
        al.y = y; al.z = zb; al.ysum = s.ysum; al.x_next = xb;
        al.step_y = step_y; al.alpha = ap.alpha; al.weight = (float)weight; al.tau1 = ap.tau1; al.tau2 = ap.tau2;
        al.first = t == 0 ? 1 : 0;
        ProfScope ps(c, LPC_PROF_EXCHANGE, st, true);
        LPC_TRY_HIP(launch_cols_exchange(c, s.U, key, s.packed, s.delta, nullptr, 0.0f, nullptr, nullptr, &al, za,
                                         pd_next, st));
        float *tmp = xa; xa = xb; xb = tmp;
        tmp = za; za = zb; zb = tmp;
        wsum += weight;
        weight *= (double)ap.theta;
      }
      if (za != z) LPC_TRY_HIP(launch_copy(z, za, c->d, st));
      LPC_TRY_HIP(launch_scale_to(c, s.ysum, (float)(1.0 / wsum), w_snap, st));
      return LPC_OK;
    }
    const bool two_alpc = c->iter_form == 1 && c->iter2_capable;
    if (two_alpc) LPC_TRY_HIP(launch_fused_iter_reset(c, st));
    for (int32_t t = 0; t < g.m; ++t) {
      const StreamKey key = key_of(c, epoch, (uint32_t)t);
      {
        ProfScope ps(c, LPC_PROF_VR_ROWS, st, true);
        LPC_TRY_HIP(launch_dense_vr_grad(c, s.w, w_snap, zs, key, kTagBatch, 0, g.N, true, st));
      }
      if (two_alpc) {
        // two launches per inner iteration: the rows above; fold + exchange + Alg. 2 steps 13-15 + next step 6
        AlpcStep al{};
        al.x = s.w; al.u_hat = nullptr; al.w_snap = w_snap; al.mu = s.mu;
        al.y = y; al.z = z; al.ysum = s.ysum; al.x_next = s.w;
        al.step_y = step_y; al.alpha = ap.alpha; al.weight = (float)weight; al.tau1 = ap.tau1; al.tau2 = ap.tau2;
        al.first = t == 0 ? 1 : 0;
        ProfScope ps(c, LPC_PROF_EXCHANGE, st, true);
        LPC_TRY_HIP(launch_fused_iter(c, key, s.packed, s.delta, nullptr, 0.0f, nullptr, &al, st));
        wsum += weight;
        weight *= (double)ap.theta;
        continue;
      }
      {
        ProfScope ps(c, LPC_PROF_VR_FOLD, st, true);
        LPC_TRY_HIP(launch_reduce_parts(c, s.part, c->vr_parts, (float)(1.0 / (double)g.B), s.U, c->d_pad, 0,
                                        g.N + 1, kStatsPartial, nullptr, st));
      }
      AlpcStep al{};
      al.x = s.w; al.u_hat = u_hat; al.w_snap = w_snap; al.mu = s.mu;
      al.y = y; al.z = z; al.ysum = s.ysum; al.x_next = s.w;
      al.step_y = step_y; al.alpha = ap.alpha; al.weight = (float)weight; al.tau1 = ap.tau1; al.tau2 = ap.tau2;
      al.first = t == 0 ? 1 : 0;
      ProfScope ps(c, LPC_PROF_EXCHANGE, st, true);
      LPC_TRY_HIP(launch_fused_exchange_alpc(c, s.U, (int32_t)((c->d_pad + 63) / 64), key, s.packed, s.delta, al,
                                             st));
      wsum += weight;
      weight *= (double)ap.theta;
    }
    LPC_TRY_HIP(launch_scale_to(c, s.ysum, (float)(1.0 / wsum), w_snap, st));
    return LPC_OK;
  }
  if (c->csr_sparse && !tracing) {
    // Sparse inner iteration for Alg. 2 / 3: the N workers' vectors and the shared batch's full-precision difference
    // (vector N) stay sparse through the worker and statistics passes; the workers' are quantized (own scale
    // factors, or the shared one of schemes (b), (c)), the receiver is the dense one, and one pass over d takes
    // Alg. 2 steps 13-15 with the next step 6 and clears the shared batch's vector.
    const int32_t nvec = g.N + 1;
    const int32_t extra = csr_sparse_parts(g.B) - 1;
    LPC_TRY_HIP(launch_zero(s.U, (int64_t)nvec * c->d_pad, st));
    if (extra > 0) {
      LPC_TRY_HIP(launch_zero(s.sparse_planes, (int64_t)nvec * extra * c->d_pad, st));
      LPC_TRY_HIP(launch_fill_u32(s.touched_parts, 0u, (int64_t)nvec * extra * c->bitmap_words, st));
    }
    LPC_TRY_HIP(launch_fill_u32(s.touched, 0u, (int64_t)nvec * c->bitmap_words, st));
    LPC_TRY_HIP(launch_fill_u32(s.packed, 0u, (int64_t)g.N * c->W, st));
    LPC_TRY_HIP(launch_csr_plan(c, zs, key_of(c, epoch, 0), true, st));
    LPC_TRY_HIP(launch_alpc_couple(c, z, w_snap, y, ap.tau1, ap.tau2, s.w, st));
    for (int32_t t = 0; t < g.m; ++t) {
      const StreamKey key = key_of(c, epoch, (uint32_t)t);
      {
        ProfScope ps(c, LPC_PROF_VR_ROWS, st);
        LPC_TRY_HIP(launch_csr_vr_sparse(c, s.w, w_snap, zs, key, s.csr_plan + (int64_t)t * nvec * g.B, nvec, st));
      }
      {
        ProfScope ps(c, LPC_PROF_VR_FOLD, st);
        LPC_TRY_HIP(launch_sparse_stats(c, nvec, st));
      }
      ProfScope ps(c, LPC_PROF_EXCHANGE, st);
      LPC_TRY_HIP(launch_sparse_quantize(c, key, g.scheme != LPC_SCHEME_A, st));
      if (g.scheme == LPC_SCHEME_A) LPC_TRY_HIP(launch_dequantize_avg(c, s.packed, s.delta, s.u_avg, st));
      else LPC_TRY_HIP(launch_dequantize_shared(c, s.packed, s.delta, g.scheme == LPC_SCHEME_C, key, s.u_avg, st));
      AlpcStep al{};
      al.x = s.w; al.u_hat = u_hat; al.w_snap = w_snap; al.mu = s.mu;
      al.y = y; al.z = z; al.ysum = s.ysum; al.x_next = s.w;
      al.step_y = step_y; al.alpha = ap.alpha; al.weight = (float)weight; al.tau1 = ap.tau1; al.tau2 = ap.tau2;
      al.first = t == 0 ? 1 : 0;
      LPC_TRY_HIP(launch_alpc_update_couple(c, al, st));
      // the consumed words and all bitmaps (the shared batch's included) start the next iteration at zero
      LPC_TRY_HIP(launch_fill_u32(s.packed, 0u, (int64_t)g.N * c->W, st));
      LPC_TRY_HIP(launch_fill_u32(s.touched, 0u, (int64_t)nvec * c->bitmap_words, st));
      wsum += weight;
      weight *= (double)ap.theta;
    }
    LPC_TRY_HIP(launch_scale_to(c, s.ysum, (float)(1.0 / wsum), w_snap, st));
    return LPC_OK;
  }
  for (int32_t t = 0; t < g.m; ++t) {
    const StreamKey key = key_of(c, epoch, (uint32_t)t);
    LPC_TRY_HIP(launch_alpc_couple(c, z, w_snap, y, ap.tau1, ap.tau2, s.w, st));
    LPC_TRY(vr_grad_impl(c, s.w, w_snap, zs, key, kTagBatch, 0, g.N, s.U, nullptr,
                         c->quant ? kStatsFinal : kStatsNone, st));
    {
      ProfScope ps(c, LPC_PROF_EXCHANGE, st);
      if (c->quant && g.scheme != LPC_SCHEME_A) {
        LPC_TRY_HIP(launch_share_delta(c, g.N, nullptr, st));
        LPC_TRY_HIP(launch_quantize(c, s.U, key, s.packed, s.delta, s.n_clipped, st));
        LPC_TRY_HIP(launch_dequantize_shared(c, s.packed, s.delta, g.scheme == LPC_SCHEME_C, key, s.u_avg, st));
      } else if (c->quant) {
        LPC_TRY_HIP(launch_quantize(c, s.U, key, s.packed, s.delta, s.n_clipped, st));
        LPC_TRY_HIP(launch_dequantize_avg(c, s.packed, s.delta, s.u_avg, st));
      } else {
        LPC_TRY_HIP(launch_plain_avg(c, s.U, s.u_avg, st));
      }
    }
    if (tracing) LPC_TRY(record_iteration(c, t, st));
    // double sampling: the shared batch J, full precision
    LPC_TRY(vr_grad_impl(c, s.w, w_snap, zs, key, kTagShared, 0, 1, u_hat, nullptr, kStatsNone, st));
    LPC_TRY_HIP(launch_alpc_update(c, s.w, s.u_avg, u_hat, s.mu, step_y, ap.alpha, (float)weight, t == 0, y, z,
                                   s.ysum, st));
    wsum += weight;
    weight *= (double)ap.theta;
  }
  LPC_TRY_HIP(launch_scale_to(c, s.ysum, (float)(1.0 / wsum), w_snap, st));
  return LPC_OK;
}

lpc_status lpc_epoch_traced(lpc_ctx *ctx, float *w_snap, float *y, float *z, uint32_t epoch, float *delta_trace,
                            uint32_t *nclip_trace, uint64_t *coded_bits_host, void *stream) {
  if (!ctx) return LPC_ENULL;
  if (!delta_trace && !nclip_trace && !coded_bits_host) return lpc_epoch(ctx, w_snap, y, z, epoch, stream);
  ctx->trace_delta = delta_trace;
  ctx->trace_nclip = nclip_trace;
  ctx->trace_coded_host = coded_bits_host;
  const lpc_status rc = lpc_epoch(ctx, w_snap, y, z, epoch, stream);
  ctx->trace_delta = nullptr;
  ctx->trace_nclip = nullptr;
  ctx->trace_coded_host = nullptr;
  return rc;
}

lpc_status lpc_epoch_report(lpc_ctx *ctx, float *w_snap, float *y, float *z, uint32_t epoch,
                            lpc_epoch_stats *stats_out_host, void *stream) {
  if (!ctx || !stats_out_host) return LPC_ENULL;
  lpc_ctx *c = ctx;
  hipStream_t st = as_stream(stream);
  LPC_TRY(lpc_epoch_traced(c, w_snap, y, z, epoch, c->s.report_delta, c->s.report_nclip, nullptr, stream));
  const int64_t cnt = (int64_t)c->cfg.m * c->cfg.N;
  LPC_TRY_HIP(launch_epoch_report(c->s.report_delta, c->s.report_nclip, cnt, c->s.report_out, st));
  unsigned long long out[2] = {0, 0};
  LPC_TRY_HIP(hipMemcpyAsync(out, c->s.report_out, sizeof(out), hipMemcpyDeviceToHost, st));
  const lpc_status flags = lpc_take_device_flags(c, stream);  // synchronises the stream
  if (flags != LPC_OK && flags != LPC_ENONFINITE) return flags;
  uint64_t per_iter = 0;
  LPC_TRY(lpc_bits_per_iteration(c->d, c->cfg.bits, c->cfg.N, c->cfg.scheme, &per_iter));
  stats_out_host->bits_sent = per_iter * (uint64_t)c->cfg.m;
  stats_out_host->messages = (uint64_t)cnt;
  stats_out_host->clipped = out[0];
  const uint32_t mb = (uint32_t)out[1];
  std::memcpy(&stats_out_host->max_delta, &mb, sizeof(float));
  stats_out_host->nonfinite = flags == LPC_ENONFINITE ? 1 : 0;
  return LPC_OK;
}

lpc_status lpc_clip_sweep(lpc_ctx *ctx, const float *w0, int32_t n_clip, const float *clips_host, int32_t epochs,
                          uint32_t epoch0, float *w_work, float *y_work, float *z_work, double *P_out_host,
                          uint64_t *clipped_out_host, void *stream) {
  if (!ctx || !w0 || !clips_host || !w_work || !P_out_host) return LPC_ENULL;
  lpc_ctx *c = ctx;
  if (!c->quant || n_clip < 1 || epochs < 1) return LPC_EINVAL;
  const bool alpc = c->cfg.algo != LPC_ALGO_LPC;
  if (alpc && (!y_work || !z_work)) return LPC_ENULL;
  for (int32_t k = 0; k < n_clip; ++k) {
    if (!(clips_host[k] > 0.0f)) return LPC_EINVAL;
    if (c->cfg.clip_mode == LPC_CLIP_LAMBDA && clips_host[k] > 1.0f) return LPC_EINVAL;
  }
  hipStream_t st = as_stream(stream);
  const float clip_before = c->cfg.clip;
  lpc_status rc = LPC_OK;
  for (int32_t k = 0; k < n_clip && rc == LPC_OK; ++k) {
    c->cfg.clip = clips_host[k];
    c->count_clipped = clipped_out_host != nullptr;
    rc = [&]() -> lpc_status {
      LPC_TRY_HIP(launch_copy(w_work, w0, c->d, st));
      if (alpc) {
        LPC_TRY_HIP(launch_copy(y_work, w0, c->d, st));
        LPC_TRY_HIP(launch_copy(z_work, w0, c->d, st));
      }
      if (clipped_out_host) LPC_TRY_HIP(launch_fill_u32(reinterpret_cast<uint32_t *>(c->s.clip_total), 0u, 2, st));
      for (int32_t e = 0; e < epochs; ++e) LPC_TRY(lpc_epoch(c, w_work, y_work, z_work, epoch0 + (uint32_t)e, stream));
      if (clipped_out_host)
        LPC_TRY_HIP(hipMemcpyAsync(&clipped_out_host[k], c->s.clip_total, sizeof(uint64_t), hipMemcpyDeviceToHost, st));
      c->count_clipped = false;
      return lpc_objective(c, w_work, &P_out_host[k], stream);  // synchronises the stream
    }();
  }
  c->count_clipped = false;
  c->cfg.clip = clip_before;
  return rc;
}

lpc_status lpc_objective(lpc_ctx *ctx, const float *w, double *P_out_host, void *stream) {
  if (!ctx || !w || !P_out_host) return LPC_ENULL;
  hipStream_t st = as_stream(stream);
  LPC_TRY(full_grad_impl(ctx, w, nullptr, nullptr, ctx->s.f_scalar, ctx->n, st));
  LPC_TRY_HIP(launch_objective_reg(ctx, w, ctx->s.f_scalar, st));
  LPC_TRY_HIP(hipMemcpyAsync(P_out_host, ctx->s.f_scalar, sizeof(double), hipMemcpyDeviceToHost, st));
  LPC_TRY_HIP(hipStreamSynchronize(st));
  return LPC_OK;
}

lpc_status lpc_gradient_mapping(lpc_ctx *ctx, const float *w, float eta, double *gm2_out_host, void *stream) {
  if (!ctx || !w || !gm2_out_host) return LPC_ENULL;
  if (!(eta > 0.0f)) return LPC_EINVAL;
  hipStream_t st = as_stream(stream);
  float *grad = ctx->s.u_avg;   // free outside an epoch
  LPC_TRY(full_grad_impl(ctx, w, grad, nullptr, nullptr, ctx->n, st));
  LPC_TRY_HIP(launch_gradient_mapping(ctx, w, grad, (double)eta, ctx->s.f_scalar, st));
  LPC_TRY_HIP(hipMemcpyAsync(gm2_out_host, ctx->s.f_scalar, sizeof(double), hipMemcpyDeviceToHost, st));
  LPC_TRY_HIP(hipStreamSynchronize(st));
  return LPC_OK;
}

lpc_status lpc_code_histogram(lpc_ctx *ctx, const uint32_t *packed, uint64_t *counts, void *stream) {
  if (!ctx || !packed || !counts) return LPC_ENULL;
  if (!ctx->quant) return LPC_EINVAL;
  LPC_TRY_HIP(launch_code_histogram(packed, ctx->d, ctx->cfg.bits, counts, as_stream(stream)));
  return LPC_OK;
}

lpc_status lpc_huffman_encode(lpc_ctx *ctx, const uint32_t *packed, const int32_t *lens_host, uint32_t *out_words,
                              int64_t capacity_words, uint64_t *total_bits_out_host, void *stream) {
  if (!ctx || !packed || !lens_host || !total_bits_out_host) return LPC_ENULL;
  if (!ctx->quant || capacity_words < 0 || (capacity_words > 0 && !out_words)) return LPC_EINVAL;
  hipStream_t st = as_stream(stream);
  const int32_t nsym = 1 << ctx->cfg.bits;
  std::vector<HuffEntry> table((size_t)nsym);
  if (huffman_canonical_table(lens_host, nsym, table.data()) != 0) return LPC_EINVAL;
  LPC_TRY_HIP(hipMemcpyAsync(ctx->s.huff_table, table.data(), sizeof(HuffEntry) * (size_t)nsym, hipMemcpyHostToDevice,
                             st));
  LPC_TRY_HIP(launch_huffman_measure(ctx, packed, st));
  unsigned long long meta[2] = {0, 0};
  LPC_TRY_HIP(hipMemcpyAsync(meta, ctx->s.huff_meta, sizeof(meta), hipMemcpyDeviceToHost, st));
  LPC_TRY_HIP(hipStreamSynchronize(st));  // also: the table has left the host vector
  if (meta[1]) return LPC_EINVAL;         // a coordinate whose symbol has no codeword
  *total_bits_out_host = meta[0];
  const int64_t need = (int64_t)((meta[0] + 31) / 32);
  if (need > capacity_words) return LPC_ESHAPE;
  if (need == 0) return LPC_OK;
  LPC_TRY_HIP(launch_huffman_emit(ctx, packed, out_words, need, st));
  return LPC_OK;
}

lpc_status lpc_take_device_flags(lpc_ctx *ctx, void *stream) {
  if (!ctx) return LPC_ENULL;
  hipStream_t st = as_stream(stream);
  uint32_t flags[4] = {0, 0, 0, 0};
  LPC_TRY_HIP(hipMemcpyAsync(flags, ctx->s.flags, sizeof(flags), hipMemcpyDeviceToHost, st));
  LPC_TRY_HIP(hipStreamSynchronize(st));
  LPC_TRY_HIP(launch_fill_u32(ctx->s.flags, 0u, 4, st));
  if (flags[0] & 2u) return LPC_EDEVICE;  // a workgroup of the two-launch iteration gave up waiting for the others
  return (flags[0] & 1u) ? LPC_ENONFINITE : LPC_OK;
}

}  // extern "C"
