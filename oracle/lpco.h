/*
 * lpco.h -- CPU oracle for the LPC-SVRG / ALPC-SVRG hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, single-threaded-by-default
 * reference written from the paper (Yu, Wu, Huang, arXiv 1901.08924).  It
 * shares no code, header, table or helper with the HIP library; nothing in the
 * product path may include, link or call it.  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg use it.
 *
 * All pointers are HOST pointers.  Vectors that the paper treats as
 * "full precision" are stored as 32-bit floats (the paper's full precision is
 * the 32-bit float); every reduction (dot products, gradient sums, objective)
 * is accumulated in double.  The quantizer arithmetic is fixed in float,
 * step by step, because it decides integer codes.
 *
 * Parity pins (see tests/test_oracle_*.py):
 *   philox            : published known-answer vectors of Philox4x32-10
 *   quantizer         : unbiasedness and exact variance (x-z)(z+delta-x)
 *                       (Sec. 3.2, Lemma 1 and its proof), Lemma 4 of the
 *                       supplement, grid/end-point/out-of-hull cases, ternary
 *                       special case (Sec. 4.1 "Unbiased quantization")
 *   pack              : exhaustive round trip, size 32 + b*d bits (Sec. 4.2)
 *   prox              : brute-force argmin of the definition (Sec. 3.3)
 *   full gradient     : finite differences, library least squares / logistic
 *   LPC-SVRG loop     : quantization off == separately written prox-SVRG
 *                       (Theorem 1 setting); minimiser vs library solvers
 *   ALPC-SVRG         : ridge closed form, m=1 snapshot rule, unbiased v-hat
 *   MLP               : autograd of the same network (library routine); the
 *                       ReLU-margin helper on a hand-built network with known
 *                       pre-activations
 *   parity unpinned   : the c*sigma clip convention, the choice of eta, and the
 *                       softmax-MLP gradient beyond finite differences
 */
#ifndef LPCO_H
#define LPCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { LPCO_OK = 0, LPCO_EINVAL = -1, LPCO_ENULL = -2, LPCO_ESHAPE = -3, LPCO_ENONFINITE = -5,
       LPCO_EUNSUPPORTED = -7 };
enum { LPCO_LOSS_LOGISTIC = 0, LPCO_LOSS_SQUARED = 1, LPCO_LOSS_MLP_SOFTMAX = 2 };
enum { LPCO_ALGO_LPC = 0, LPCO_ALGO_ALPC_SC = 1, LPCO_ALGO_ALPC_GC = 2 };
enum { LPCO_CLIP_LAMBDA = 0, LPCO_CLIP_CSIGMA = 1 };
/* stream tags of the counter-based generator */
enum { LPCO_TAG_QUANT = 0, LPCO_TAG_BATCH = 1, LPCO_TAG_SHARED = 2, LPCO_TAG_REQUANT = 3 };
/* communication step 2 variants (Sec. 4.2): (a) per-worker delta; (b) shared delta,
 * integer sum; (c) shared delta + unbiased re-quantization of the average (eq. 5) */
enum { LPCO_SCHEME_A = 0, LPCO_SCHEME_B = 1, LPCO_SCHEME_C = 2 };

/* The finite-sum problem of eq. (1):  P(w) = (1/n) sum_i f_i(w) + h(w),
 * h(w) = lambda1*|w|_1 + (lambda2/2)*|w|^2.  Exactly one of X (dense,
 * row-major, leading dimension ldx) or (row_ptr, col_idx, vals) (CSR) is set.
 * For the MLP loss, X holds the inputs (n x mlp_dims[0]), y the class ids and
 * d is the total parameter count. */
typedef struct {
  int64_t n, d;
  int32_t loss;
  const float *X;
  int64_t ldx;
  const int32_t *row_ptr;
  const int32_t *col_idx;
  const float *vals;
  int64_t nnz;
  const float *y;
  const int32_t *mlp_dims;
  int32_t mlp_nlayers; /* number of weight layers; mlp_dims has mlp_nlayers+1 entries */
  float lambda1, lambda2;
} lpco_problem;

typedef struct {
  int32_t algo;
  int32_t N, B, m, bits; /* bits >= 32: quantization off */
  int32_t clip_mode;
  float clip; /* the paper's lambda in (0,1], or c of c*sigma */
  int32_t scheme;
  float eta, L, sigma, tau1, tau2, alpha; /* ALPC: 0 means "derive" */
  uint64_t seed;
  int64_t n_full; /* rows used by the snapshot gradient; 0 means all n */
} lpco_config;

/* ---- counter-based generator (Philox4x32-10, Salmon et al. SC'11) ---- */
void lpco_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
/* word `index` of the stream (seed, epoch, iter, tag, worker) */
uint32_t lpco_stream_word(uint64_t seed, uint32_t epoch, uint32_t iter, uint32_t tag, uint32_t worker,
                          uint64_t index);
/* Alg. 1 step 6 / Alg. 2 step 11: B indices, uniform, independent, with
 * replacement.  tag = LPCO_TAG_BATCH (per worker) or LPCO_TAG_SHARED (J). */
int lpco_sample_batch(uint64_t seed, uint32_t epoch, uint32_t iter, uint32_t tag, uint32_t worker, int32_t B,
                      int64_t n, int64_t *idx_out);

/* ---- quantizer (Sec. 3.2 rules (1),(2); eq. (3)) ---- */
int64_t lpco_d_pad(int64_t d);                     /* 32 * ceil(d/32) */
int64_t lpco_words_per_msg(int64_t d, int32_t b);  /* ceil(d/32) * b  */
/* stats[4] = { max|u_j|, sum u_j, sum u_j^2, #non-finite } over the d true coordinates */
int lpco_vector_stats(const float *u, int64_t d, double stats[4]);
/* eq. (3) with lambda given directly or derived from c*sigma; returns delta and
 * the positive clip threshold t = lambda*|u|_inf (float arithmetic). */
int lpco_delta_from_stats(const double stats[4], int64_t d, int32_t bits, int32_t clip_mode, float clip,
                          float *delta_out, float *thresh_out);
/* codes k_j in [-2^(b-1), 2^(b-1)-1] for one vector, given delta; thresh is used
 * only to count clipped coordinates (pass +inf to count nothing on the positive side). */
int lpco_quantize_codes(const float *u, int64_t d, int32_t bits, float delta, float thresh, uint64_t seed,
                        uint32_t epoch, uint32_t iter, uint32_t tag, uint32_t worker, int32_t *codes_out,
                        uint32_t *n_clipped);
int lpco_pack(const int32_t *codes, int64_t d, int32_t bits, uint32_t *words /* lpco_words_per_msg */);
int lpco_unpack(const uint32_t *words, int64_t d, int32_t bits, int32_t *codes_out);
/* all N workers at once: U is [N][d_pad]; packed is [N][W]; stats may be NULL
 * (then computed here); delta_in may be NULL (then eq. (3) is applied). */
int lpco_quantize_clip(int64_t d, int32_t N, int32_t bits, int32_t clip_mode, float clip, uint64_t seed,
                       uint32_t epoch, uint32_t iter, const float *U, const double *stats, const float *delta_in,
                       uint32_t *packed, float *delta_out, uint32_t *n_clipped);
/* eq. (4): u_avg_j = (1/N) sum_i delta_i * k^i_j, fixed worker order, float fma */
int lpco_dequantize_avg(int64_t d, int32_t N, int32_t bits, const uint32_t *packed, const float *delta,
                        float *u_avg);
/* quantization off: u_avg = (1/N) sum_i u^i (float adds in worker order) */
int lpco_plain_avg(int64_t d, int32_t N, const float *U, float *u_avg);
/* schemes (b)/(c): shared delta = max_i delta_i, integer code sums, optional eq. (5) */
int lpco_dequantize_shared(int64_t d, int32_t N, int32_t bits, const uint32_t *packed, float delta_shared,
                           int32_t requantize, uint64_t seed, uint32_t epoch, uint32_t iter, float *u_avg,
                           int32_t *code_sums /* [d] or NULL */);

/* ---- prox (Sec. 3.3) and gradient oracles ---- */
/* w <- prox_{step*h}(w - step*(u_avg + mu)) ; Alg. 1 steps 9-10 */
int lpco_prox_step(int64_t d, float *w, const float *u_avg, const float *mu, float step, float lambda1,
                   float lambda2);
/* Alg. 1 step 4: z = Xw (n, may be NULL), mu = grad f(w) (d), f_out = f(w) (may be NULL).
 * Uses the first n_rows rows (0 = all). */
int lpco_full_grad(const lpco_problem *p, const float *w, int64_t n_rows, float *mu, float *z, double *f_out);
/* Alg. 1 step 6 for workers [worker_begin, worker_end): U row i = u^i (d_pad
 * floats, padding zero); stats row i as lpco_vector_stats.  tag selects the
 * per-worker stream or the shared batch J (then the single row "worker_begin"
 * is written and the stream's worker field is the shared one). */
int lpco_worker_vr_grad(const lpco_problem *p, const lpco_config *c, const float *w, const float *w_snap,
                        uint32_t epoch, uint32_t iter, uint32_t tag, int32_t worker_begin, int32_t worker_end,
                        float *U, double *stats);
/* MLP only: the smallest |pre-activation| of a hidden ReLU unit over the B given rows (the gradient is
 * discontinuous at zero, so parity with a float implementation is only meaningful away from it) */
int lpco_mlp_relu_margin(const lpco_problem *p, const float *w, const int64_t *idx, int32_t B, double *margin_out);
/* P(w) of eq. (1) */
int lpco_objective(const lpco_problem *p, const float *w, double *P_out);

/* ---- the loops ---- */
/* resolved ALPC parameters for epoch s (Theorem 3 / Alg. 3 schedules) */
int lpco_alpc_params(const lpco_problem *p, const lpco_config *c, uint32_t epoch, float *tau1, float *tau2,
                     float *alpha, float *theta);
/* One epoch of Alg. 1 (algo LPC: y, zacc ignored) or Alg. 2 / Alg. 3.
 * w_snap: in x~^s, out x~^(s+1).  y, zacc: ALPC state, in/out (d each). */
int lpco_epoch(const lpco_problem *p, const lpco_config *c, float *w_snap, float *y, float *zacc, uint32_t epoch,
               uint64_t *bits_sent /* may be NULL; communication step 2 only, Table 1 */);
/* The same epoch, also recording per inner iteration t and worker i the scale factor delta_t^i (eq. (3);
 * the shared one under schemes (b), (c); 0 with quantization off) and the number of clipped coordinates
 * d_lambda of that message (Sec. 3.2), and the size in bits of its d codes after entropy coding (Sec. 6.1;
 * 32*d with quantization off): delta_trace, nclip_trace, coded_trace are [m][N], each may be NULL. */
int lpco_epoch_traced(const lpco_problem *p, const lpco_config *c, float *w_snap, float *y, float *zacc,
                      uint32_t epoch, float *delta_trace, uint32_t *nclip_trace, uint64_t *coded_trace);

/* ---- evaluators ---- */
/* |G_eta(w)|^2, the gradient-mapping metric of Sec. 3.3 */
int lpco_gradient_mapping(const lpco_problem *p, const float *w, float eta, double *gm2_out);
/* left-hand side of eq. (6) (schemes a, b) / eq. (7) (scheme c) of Theorem 2 */
double lpco_theorem2_lhs(int64_t d, int32_t bits, double lambda, int64_t d_lambda, int32_t N, int32_t B, int32_t m,
                         double rho, int32_t scheme);
/* entropy (Huffman) coding of the code stream, Sec. 6.1: optimal prefix-code lengths from the counts
 * of the 2^b code values; returns the encoded size in bits */
uint64_t lpco_huffman_bits(const uint64_t *counts, int32_t nsym, int32_t *lens_out);
int lpco_code_histogram(const uint32_t *words, int64_t d, int32_t bits, uint64_t *counts);
/* The entropy-coded stream of one packed message under the canonical prefix code of the given lengths
 * (symbols ordered by (length, bin index); codewords most significant bit first; stream bit p in word p/32
 * at bit p%32), and its inverse. */
int lpco_huffman_encode(const uint32_t *words, int64_t d, int32_t bits, const int32_t *lens, uint32_t *out_words,
                        int64_t capacity_words, uint64_t *total_bits_out);
int lpco_huffman_decode(const uint32_t *stream, uint64_t total_bits, int64_t d, int32_t bits, const int32_t *lens,
                        int32_t *codes_out);

/* ---- message accounting (Table 1) ---- */
uint64_t lpco_bits_per_message(int64_t d, int32_t bits);
uint64_t lpco_bits_per_iteration(int64_t d, int32_t bits, int32_t N, int32_t scheme);

void lpco_set_threads(int32_t nthreads); /* cpu_baseline timing only; default 1 */

#ifdef __cplusplus
}
#endif
#endif
