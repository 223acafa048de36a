/*
 * lpc.h -- C ABI of the MI355X (gfx950) implementation of the data-parallel
 * hot path of LPC-SVRG / ALPC-SVRG (Yu, Wu, Huang, arXiv 1901.08924).
 *
 * The library solves the finite-sum composite problem of eq. (1),
 *     min_w P(w) = (1/n) sum_i f_i(w) + h(w),   h(w) = lambda1*|w|_1 + (lambda2/2)*|w|^2,
 * with N data-parallel workers simulated as shards on ONE GPU: the snapshot
 * full-gradient pass (communication step 1), the workers' variance-reduced
 * minibatch differences, the clipped low-precision stochastic quantizer with
 * bit-packing, the receiver-side dequantize-and-average (communication step 2)
 * and the proximal step, plus ALPC-SVRG's double sampling.
 *
 * Conventions
 *  - Every pointer named "device" below is a DEVICE pointer owned by the caller
 *    (for instance memory of a torch tensor); the library only borrows it.
 *    Float/uint32 buffers must be 16-byte aligned, double buffers 8-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Every call except lpc_create, lpc_destroy, lpc_objective,
 *    lpc_gradient_mapping and lpc_take_device_flags only enqueues work: no host synchronisation, no
 *    allocation.  Scratch memory comes from the workspace given to lpc_create.
 *  - Calls on one context must be issued on one stream at a time: they share
 *    the context's scratch.
 *  - Every call returns an lpc_status; nothing throws or aborts across the ABI.
 *  - Results are a function of (problem, config, inputs, epoch, iter) only: all
 *    randomness comes from a counter-based Philox4x32-10 stream with
 *    key = (seed low, seed high) and counter = (index >> 2, tag << 24 | worker,
 *    iter, epoch); word (index & 3) of the block belongs to `index`.
 *  - d_pad = 32*ceil(d/32); a packed message has W = ceil(d/32)*bits 32-bit words.
 */
#ifndef LPC_H
#define LPC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lpc_ctx lpc_ctx; /* opaque host object */

typedef enum {
  LPC_OK = 0,
  LPC_EINVAL = -1,      /* a scalar argument or config field is out of range */
  LPC_ENULL = -2,       /* a required pointer is NULL */
  LPC_ESHAPE = -3,      /* sizes / leading dimensions / alignment do not fit */
  LPC_EWORKSPACE = -4,  /* workspace missing, misaligned or too small */
  LPC_ENONFINITE = -5,  /* a vector handed to the quantizer held NaN/Inf (see lpc_take_device_flags) */
  LPC_EDEVICE = -6,     /* a HIP call failed */
  LPC_EUNSUPPORTED = -7 /* valid in the paper, not built here */
} lpc_status;

typedef enum { LPC_LOSS_LOGISTIC = 0, LPC_LOSS_SQUARED = 1, LPC_LOSS_MLP_SOFTMAX = 2 } lpc_loss;
typedef enum { LPC_ALGO_LPC = 0, LPC_ALGO_ALPC_SC = 1, LPC_ALGO_ALPC_GC = 2 } lpc_algo; /* Alg. 1 / 2 / 3 */
typedef enum { LPC_CLIP_LAMBDA = 0, LPC_CLIP_CSIGMA = 1 } lpc_clip_mode;
typedef enum { LPC_SCHEME_A = 0, LPC_SCHEME_B = 1, LPC_SCHEME_C = 2 } lpc_scheme; /* Sec. 4.2 (a), (b), (c) */
typedef enum { LPC_BATCH_WORKER = 1, LPC_BATCH_SHARED = 2 } lpc_batch_kind;

/* The data of eq. (1).  Exactly one of X (dense row-major, leading dimension
 * ldx floats) or (row_ptr, col_idx, vals) (CSR, sorted int32 indices) is set.
 * Losses: logistic f_i = log(1+exp(-y_i x_i'w)), y_i = +-1; squared
 * f_i = (x_i'w - y_i)^2/2; MLP = ReLU multi-layer perceptron with softmax
 * cross-entropy, X = inputs [n][mlp_dims[0]], y = class ids stored as floats,
 * d = total parameter count, parameters laid out layer by layer as the weight
 * matrix [in][out] row-major followed by the bias [out]. */
typedef struct {
  int64_t n, d;
  int32_t loss;            /* lpc_loss */
  const float *X;          /* device */
  int64_t ldx;
  const int32_t *row_ptr;  /* device, n+1 entries */
  const int32_t *col_idx;  /* device */
  const float *vals;       /* device */
  int64_t nnz;
  const float *y;          /* device, n entries */
  const int32_t *mlp_dims; /* HOST, mlp_nlayers+1 entries (read during lpc_create only) */
  int32_t mlp_nlayers;
  float lambda1, lambda2;
} lpc_problem;

/* Inputs of Alg. 1 (S, m, lambda, B, eta) and Alg. 2/3 (tau1, tau2, alpha).
 * bits in [2,16], or >= 32 for "quantization off" (u~ = plain average).
 * clip: the paper's clipping parameter lambda in (0,1] (LPC_CLIP_LAMBDA), or c
 * of the [-c*sigma, c*sigma] rule (LPC_CLIP_CSIGMA: lambda = min(1, c*sigma/|u|_inf),
 * sigma = population standard deviation of the coordinates of u).
 * ALPC fields left at 0 are derived: Theorem 3 for Alg. 2
 * (tau1 = sqrt(m*sigma/(6L)) <= 1/2, alpha = 1/(6*tau1*L), tau2 = min(1/2, 5*zeta/3 + 1/(2B))),
 * Alg. 3 step 3 for Alg. 3 (tau1 = 2/(s+4), alpha = 1/(6*L*tau1), or alpha/tau1 if alpha is given). */
typedef struct {
  int32_t algo;      /* lpc_algo */
  int32_t N, B, m, bits;
  int32_t clip_mode; /* lpc_clip_mode */
  float clip;
  int32_t scheme;    /* lpc_scheme: per-worker delta (a), or shared delta with integer sums (b) / re-quantizing (c) */
  float eta, L, sigma, tau1, tau2, alpha;
  uint64_t seed;
  int64_t n_full;    /* rows used by the snapshot gradient (0 = all n) */
} lpc_config;

/* ---- context ------------------------------------------------------------ */

/* Bytes of device scratch the context needs for this problem/config. */
size_t lpc_workspace_bytes(const lpc_problem *problem, const lpc_config *config);

/* Validates problem and config, copies both, and lays the scratch buffers out
 * in `workspace` (device, 256-byte aligned, at least lpc_workspace_bytes long,
 * owned by the caller and alive until lpc_destroy).  Clears the scratch's
 * counters and, for CSR data, builds a column-major copy of the rarely used
 * columns' entries in the scratch, on the default stream, and waits for that.  Errors: LPC_ENULL,
 * LPC_EINVAL (bits = 1 divides by zero in eq. (3); N*B > n contradicts
 * Theorem 1's N*B <= n), LPC_ESHAPE, LPC_EWORKSPACE, LPC_EUNSUPPORTED. */
lpc_status lpc_create(lpc_ctx **ctx_out, const lpc_problem *problem, const lpc_config *config, void *workspace,
                      size_t workspace_bytes);
void lpc_destroy(lpc_ctx *ctx);
const char *lpc_status_string(lpc_status s);
int64_t lpc_d_pad(int64_t d);
int64_t lpc_words_per_msg(int64_t d, int32_t bits);

/* ---- the steps of Alg. 1 -------------------------------------------------- */

/* Alg. 1 step 4 / Alg. 2 step 3 (communication step 1): the snapshot gradient
 *   z = X w (n floats, may be NULL), mu = grad f(w) = (1/n) X' l'(z, y) (d floats),
 *   f_out = f(w) (one device double, may be NULL),
 * over the first n_full rows.  X is read from HBM once. */
lpc_status lpc_full_grad(lpc_ctx *ctx, const float *w, float *mu, float *z, double *f_out, void *stream);

/* Alg. 1 step 6 (Alg. 2 steps 7 and 11): for each worker i in
 * [worker_begin, worker_end) draw B row indices uniformly, independently, with
 * replacement from the worker's stream (kind = LPC_BATCH_WORKER) and form
 *   u^i = (1/B) sum_{a in batch} [ grad f_a(w) - grad f_a(w_snap) ]
 * into row i of U ([N][d_pad] floats, padding written as zero), with
 * stats[i] = { |u^i|_inf, sum_j u_j, sum_j u_j^2, number of non-finite u_j }
 * (4 doubles per worker, may be NULL).  kind = LPC_BATCH_SHARED draws the one
 * batch J that ALPC-SVRG's double sampling shares between all workers and
 * writes row worker_begin only.  z_snap (n floats: X w_snap, as produced by
 * lpc_full_grad) lets each sampled row be read once; NULL recomputes it. */
lpc_status lpc_worker_vr_grad(lpc_ctx *ctx, const float *w, const float *w_snap, const float *z_snap,
                              uint32_t epoch, uint32_t iter, int32_t kind, int32_t worker_begin, int32_t worker_end,
                              float *U, double *stats, void *stream);

/* stats[v] (4 doubles, as above) for each of nvec rows of U ([nvec][d_pad]). */
lpc_status lpc_vector_stats(lpc_ctx *ctx, const float *U, int32_t nvec, double *stats, void *stream);

/* Alg. 1 step 7 (quantization step), Sec. 3.2 and eq. (3), all N workers:
 *   delta_i = lambda*|u^i|_inf/(2^(bits-1)-1)  (or delta_in[i] if delta_in != NULL),
 *   code_j  = stochastic rounding of u_j/delta_i onto {-2^(bits-1),...,2^(bits-1)-1}
 *             after projection onto that range (gradient clipping),
 * codes packed as bits-wide two's-complement fields of a little-endian bit
 * stream (coordinate j in stream bits [j*bits, (j+1)*bits)), padding coded 0.
 * stats may be NULL only if delta_in is given.  Outputs: packed [N][W],
 * delta_out [N] (0 for an all-zero vector), n_clipped [N] (coordinates outside
 * dom(delta,b): above lambda*|u|_inf or below -2^(bits-1)*delta; may be NULL). */
lpc_status lpc_quantize_clip(lpc_ctx *ctx, const float *U, const double *stats, const float *delta_in,
                             uint32_t epoch, uint32_t iter, uint32_t *packed, float *delta_out, uint32_t *n_clipped,
                             void *stream);

/* Communication step 2, scheme (a), eq. (4): u_avg_j = (1/N) sum_i delta_i*code^i_j,
 * accumulated in worker order with one fused multiply-add per worker. */
lpc_status lpc_dequantize_avg(lpc_ctx *ctx, const uint32_t *packed, const float *delta, float *u_avg, void *stream);

/* Communication step 2, schemes (b) and (c) of Sec. 4.2: all N messages were quantized with the same
 * scale factor delta[0] = max_i delta_i (pass that value as every entry of delta_in to lpc_quantize_clip),
 * so the receiver adds the codes as integers and scales once: u_avg_j = delta * (sum_i code^i_j)/N.  With
 * requantize != 0 the average is rounded once more, without bias, onto dom(delta, bits) (eq. (5)) using
 * stream tag 3.  lpc_epoch applies (b)/(c) when config.scheme says so. */
lpc_status lpc_dequantize_shared(lpc_ctx *ctx, const uint32_t *packed, const float *delta, int32_t requantize,
                                 uint32_t epoch, uint32_t iter, float *u_avg, void *stream);

/* Alg. 1 steps 7-8 in one call (quantization step + communication step 2, scheme (a)): statistics of
 * the N rows of U, eq. (3), quantize + pack into packed [N][W] with delta_out [N], and the receiver's
 * average u_avg (d floats) of eq. (4).  Same results, bit for bit, as lpc_vector_stats +
 * lpc_quantize_clip + lpc_dequantize_avg in LPC_CLIP_LAMBDA mode; for small d it runs as two launches. */
lpc_status lpc_exchange(lpc_ctx *ctx, const float *U, uint32_t epoch, uint32_t iter, uint32_t *packed,
                        float *delta_out, float *u_avg, void *stream);

/* lpc_exchange for callers that cannot allocate device memory or hold a context's workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  It takes no context: the configuration
 * comes as arguments, and the scratch lpc_exchange keeps in a workspace (statistic partials, statistics,
 * quantizer parameters, clip counts; about 0.6 MB) lives in a device array inside the library, of which every
 * GPU the library runs on holds one copy until the process ends.  The call allocates and frees nothing and only
 * enqueues kernels on `stream` (its first call on a device also looks the array's address up).  Same outputs, bit
 * for bit, as lpc_exchange with the same d, N, bits, clip mode, clip and seed: packed [N][W], delta_out [N],
 * u_avg [d].  Limits: d <= 8388608 (2^23) coordinates and N <= 64 vectors; beyond either the call returns
 * LPC_EWORKSPACE (the static scratch is too small) and does nothing.  flags_out (device, one uint32, may be NULL):
 * bit 0 is OR-ed in when a vector held a NaN or Inf; the caller clears it.  All calls on one GPU share the one
 * array, which keeps the previous call's contents (each call overwrites what it reads): calls that overlap on
 * one GPU (different streams, no ordering between them) race and must be serialised by the caller. */
lpc_status lpc_exchange_static(int64_t d, int32_t N, int32_t bits, int32_t clip_mode, float clip, uint64_t seed,
                               const float *U, uint32_t epoch, uint32_t iter, uint32_t *packed, float *delta_out,
                               float *u_avg, uint32_t *flags_out, void *stream);

/* Alg. 1 steps 9-10: v = u_avg + mu;  w <- prox_{step*h}(w - step*v), in place,
 * prox(p)_j = sign(p_j)*max(|p_j| - step*lambda1, 0)/(1 + step*lambda2) (Sec. 3.3). */
lpc_status lpc_prox_step(lpc_ctx *ctx, float *w, const float *u_avg, const float *mu, float step, void *stream);

/* One epoch of Alg. 1 (algo LPC; y, z ignored) or of Alg. 2 / Alg. 3:
 * snapshot gradient, m inner iterations, snapshot update.  w_snap: in x~^s, out
 * x~^(s+1).  y, z: ALPC-SVRG's auxiliary iterates, in/out (d floats each; start
 * them equal to x~^0).  epoch = s selects the random streams and Alg. 3's schedule. */
lpc_status lpc_epoch(lpc_ctx *ctx, float *w_snap, float *y, float *z, uint32_t epoch, void *stream);

/* P(w) of eq. (1) over all n rows, returned to the HOST (synchronises the stream). */
lpc_status lpc_objective(lpc_ctx *ctx, const float *w, double *P_out_host, void *stream);

/* Reads and clears the context's device-side flags (synchronises the stream):
 * returns LPC_ENONFINITE if any vector seen by the statistics pass since the last
 * call held a NaN or Inf; LPC_EDEVICE if a workgroup of the two-launch inner iteration gave up
 * waiting for the others (the iterates since then are not to be trusted); else LPC_OK. */
lpc_status lpc_take_device_flags(lpc_ctx *ctx, void *stream);

/* ---- evaluators (outside the timed path) --------------------------------------------------
 * |G_eta(w)|^2 with G_eta(w) = (w - prox_{eta*h}(w - eta*grad f(w)))/eta, the convergence metric
 * of Sec. 3.3 (Theorems 1 and 2 bound its expectation), over all n rows; fp64 accumulation.
 * w: device, d floats.  Returned to the HOST (synchronises the stream).  Uses the context's
 * scratch; the snapshot state kept by lpc_epoch is not touched.  eta > 0 else LPC_EINVAL. */
lpc_status lpc_gradient_mapping(lpc_ctx *ctx, const float *w, float eta, double *gm2_out_host, void *stream);

/* lpc_epoch that also records, for every inner iteration t and worker i, the scale factor delta_t^i the
 * worker quantized with (eq. (3); the shared max_i delta_t^i under schemes (b), (c)) and the number of
 * clipped coordinates d_lambda of its message (Sec. 3.2; the quantity Lemma 2 and Theorem 2 are stated in):
 * delta_trace (floats) and nclip_trace (uint32) are device arrays [m][N], zero with quantization off.
 * coded_bits_host is a HOST array [m][N] that receives the size in bits of each message's d codes after
 * entropy coding (Sec. 6.1: the optimal prefix code of that message's own histogram; 32*d with
 * quantization off; add 32 bits for delta and Table 1's fan-out for a total as in Sec. 6.1's table of
 * communication costs); asking for it synchronises the stream once per message.  Each of the three may be
 * NULL; all NULL is lpc_epoch.  The traced epoch takes the unfused launches
 * (statistics, quantizer, receiver, prox as separate kernels) for every data kind; for Alg. 1 in
 * LPC_CLIP_LAMBDA mode on dense data its iterates equal lpc_epoch's bit for bit, elsewhere to rounding.
 * Asynchronous unless coded_bits_host is given. */
lpc_status lpc_epoch_traced(lpc_ctx *ctx, float *w_snap, float *y, float *z, uint32_t epoch, float *delta_trace,
                            uint32_t *nclip_trace, uint64_t *coded_bits_host, void *stream);

/* Table 1 (Sec. 4.2): bits transmitted per inner iteration by communication step 2 for d coordinates, `bits` bits
 * per coordinate and N workers: scheme (a) (32 + b d) N (N - 1); (b) N (64 + 2 b d + d ceil(log2 N)); (c)
 * N (64 + 2 b d).  bits >= 32 (quantization off): 32 d N (N - 1).  Host arithmetic only.  LPC_EINVAL for bits
 * outside [2,16] and below 32, N < 1 or an unknown scheme. */
lpc_status lpc_bits_per_iteration(int64_t d, int32_t bits, int32_t N, int32_t scheme, uint64_t *out_host);

/* One epoch as lpc_epoch, with a summary returned to the HOST (synchronises the stream): bits_sent = m times the
 * Table 1 figure of the context's scheme; messages = m*N; clipped = the coordinates outside dom(delta, b) summed
 * over all messages (Sec. 3.2's d_lambda, the quantity Lemma 2 bounds the error with); max_delta = the largest
 * scale factor any message was quantized with (eq. (3)); nonfinite = 1 if a vector handed to the quantizer held a
 * NaN or Inf (the context's flag is cleared).  The epoch takes the unfused launches, as lpc_epoch_traced does. */
typedef struct {
  uint64_t bits_sent, messages, clipped;
  float max_delta;
  int32_t nonfinite;
} lpc_epoch_stats;
lpc_status lpc_epoch_report(lpc_ctx *ctx, float *w_snap, float *y, float *z, uint32_t epoch,
                            lpc_epoch_stats *stats_out_host, void *stream);

/* Selection of the clipping parameter (Sec. 6.1 picks lambda by cross-validation, once): for each of the
 * n_clip candidates clips_host[k] (lambda in (0,1] or c > 0, in the context's clip mode) the method is run
 * for `epochs` epochs numbered epoch0, epoch0+1, ... from the same start w0 (ALPC-SVRG: y = z = w0) with
 * the same random streams, and P_out_host[k] receives the objective P of eq. (1) at the final snapshot;
 * clipped_out_host[k] (may be NULL) the clipped coordinates summed over all messages of the run.  The
 * caller picks the candidate with the smallest P.  w0: device, d floats, not modified.  w_work (and
 * y_work, z_work for ALPC-SVRG, else NULL): device scratch, d floats each; w_work ends as the last
 * candidate's snapshot.  The context's clip value is restored on return.  Synchronises the stream.
 * LPC_EINVAL with quantization off or a candidate outside the mode's range. */
lpc_status lpc_clip_sweep(lpc_ctx *ctx, const float *w0, int32_t n_clip, const float *clips_host, int32_t epochs,
                          uint32_t epoch0, float *w_work, float *y_work, float *z_work, double *P_out_host,
                          uint64_t *clipped_out_host, void *stream);

/* Left-hand side of Theorem 2's step-size condition,
 *   8 m^2 rho^2 [ c*d*lambda^2/(2^(bits-1)-1)^2 + d_lambda*(1-lambda)^2 + 1/(N*B) ] + rho,
 * c = 1/4 for schemes (a), (b) (eq. (6)) and 3/8 for scheme (c) (eq. (7)); rho = eta*L, d_lambda =
 * the number of clipped coordinates (Sec. 3.2).  The theorem needs the value <= 1 and rho < 1/2.
 * Host arithmetic only; out_host receives the value.  LPC_EINVAL for bits outside [2,16]. */
lpc_status lpc_theorem2_lhs(int64_t d, int32_t bits, double lambda, int64_t d_lambda, int32_t N, int32_t B,
                            int32_t m, double rho, int32_t scheme, double *out_host);

/* Entropy coding of the messages (Sec. 6.1 applies Huffman coding to the code stream).
 * lpc_code_histogram: counts[k] = number of the first d coordinates of ONE packed message whose
 * code is k - 2^(bits-1); packed: device, W words; counts: device, 2^bits uint64, overwritten.
 * lpc_huffman_bits: HOST arithmetic; from nsym counts, the lengths of an optimal prefix code
 * (lens_out_host, nsym int32, may be NULL; unused symbols get 0; a lone used symbol gets 1) and
 * the encoded size sum_k counts[k]*len[k] in bits (bits_out_host).  The size is unique; the
 * lengths are one valid optimum when weights tie. */
lpc_status lpc_code_histogram(lpc_ctx *ctx, const uint32_t *packed, uint64_t *counts, void *stream);
lpc_status lpc_huffman_bits(const uint64_t *counts_host, int32_t nsym, int32_t *lens_out_host,
                            uint64_t *bits_out_host);

/* The entropy-coded message itself.  The paper names the code (Huffman), not a format; this one is fixed here:
 * the CANONICAL prefix code of the given lengths -- symbols (bin index k = code + 2^(bits-1)) ordered by
 * (length, k), the first codeword all zeros, each next one the previous plus one, shifted left where the
 * length grows -- with the codewords of coordinates 0..d-1 of ONE packed message (device, W words) written
 * one after the other, most significant bit first; stream bit p is bit p%32 of out_words[p/32] (device),
 * unused high bits of the last word are zero.  lens_host: 2^bits lengths in [0, 32] as returned by
 * lpc_huffman_bits (0 = symbol without codeword).  *total_bits_out_host receives the stream length.
 * LPC_EINVAL: quantization off, lengths that are no prefix code, or a coordinate whose symbol has length
 * 0.  LPC_ESHAPE: the stream needs more than capacity_words words (total_bits_out_host is still set, so
 * capacity_words = 0 asks for the size only).  Uses the context's scratch; synchronises the stream once,
 * the emitting launches are left in flight. */
lpc_status lpc_huffman_encode(lpc_ctx *ctx, const uint32_t *packed, const int32_t *lens_host, uint32_t *out_words,
                              int64_t capacity_words, uint64_t *total_bits_out_host, void *stream);

/* ---- measurement aid (benchmarks; no passage of the paper) ------------------------------
 * While enabled, every launch of the kernel classes below made by this context is bracketed by
 * two HIP events on its stream (this allocates events and perturbs the pipeline slightly, so it
 * is off by default).  Where a class is a single kernel launch the two events ride on that launch
 * itself, so their interval is the dispatch's own begin-to-end time (what a kernel trace reports);
 * where it is several launches the events are recorded before and after them, which adds a few
 * microseconds of event handling.  lpc_profile_read synchronises the stream, returns per class the
 * summed duration in milliseconds, the number of records since the last read and (exact, may be NULL)
 * whether every record of the class was of the first kind (three HOST arrays of LPC_PROF_NCLASS
 * entries), and clears the records. */
typedef enum {
  LPC_PROF_FULL_ROWS = 0, /* snapshot pass: rows kernel                         */
  LPC_PROF_FULL_FOLD = 1, /* snapshot pass: fold of the partial gradient rows   */
  LPC_PROF_VR_ROWS = 2,   /* worker pass: rows kernel (all workers, one launch) */
  LPC_PROF_VR_FOLD = 3,   /* worker pass: fold + statistics                     */
  LPC_PROF_EXCHANGE = 4,  /* quantize/pack + dequantize/average + prox          */
  LPC_PROF_RESIDENT = 5,  /* all inner iterations of an epoch in one launch     */
  LPC_PROF_NCLASS = 6
} lpc_prof_class;
lpc_status lpc_profile_enable(lpc_ctx *ctx, int32_t on);
/* Phase time stamps of the resident inner loop (LPC_TUNE_ITER_FORM 3).  While switched on, every resident launch of
 * the context leaves, per inner iteration, 11 readings of the device's constant 100 MHz counter taken by one
 * workgroup at its phase boundaries (iteration start; rows done; partial vectors stored; first barrier of its die
 * passed; fold done; statistics published; flags of the eight dies seen; operands and scale factors ready; codes
 * ready; update stored; second barrier passed).  stamps_out_host (may be NULL): receives the last launch's stamps,
 * m rows of 16 words (words 11-15 unused), after synchronising the stream.  `on` then switches the recording
 * on or off for the launches that follow.  LPC_EUNSUPPORTED where the context cannot run that form. */
lpc_status lpc_resident_trace(lpc_ctx *ctx, int32_t on, uint64_t *stamps_out_host, void *stream);
lpc_status lpc_profile_read(lpc_ctx *ctx, double *ms_total, int64_t *launches, int32_t *exact, void *stream);

/* ---- unit-test and benchmark entry of the MLP instance's contraction kernel (no passage of the paper) ----
 * C (M x N, row-major, leading dimension ldc) = [C +] alpha * op(A) * op(B) [+ bias[n]] [then ReLU] in fp32 on
 * the matrix cores (output widths of at most 16 columns take the vector units): op(A) is M x K, stored
 * [M][K] (lda >= K), or [K][M] with transA (lda >= M); op(B) is K x N, stored [K][N] (ldb >= N), or [N][K]
 * with transB (ldb >= K).  bias: N floats or NULL.  All pointers are device pointers.  Only enqueues. */
lpc_status lpc_debug_gemm(const float *A, const float *B, float *C, int32_t M, int32_t N, int32_t K, int64_t lda,
                          int64_t ldb, int64_t ldc, int32_t transA, int32_t transB, float alpha, const float *bias,
                          int32_t relu, int32_t accumulate, void *stream);

/* ---- tuning and test aid (no passage of the paper) -----------------------------------------
 * Form and launch shape of the inner iteration on small dense problems (d_pad <= 16384, N <= 64).
 *   LPC_TUNE_ITER_FORM:
 *     0 (default): three launches: the workers' rows (whole rows per workgroup, partial gradient rows out), their
 *       fold, the exchange.
 *     1: two launches: the workers' rows, then fold + exchange in one launch whose workgroups wait, for a bounded
 *       number of polls, for each other's statistics.
 *     2: two launches with nothing but the launch boundary between them.  The workers' pass runs in 128-column
 *       tiles: a workgroup completes one tile of one u^i, taking each sampled row's margin as the sum of partial
 *       dot products that the previous launch left; the exchange launch then also leaves the partial dots of
 *       the next iteration's rows with the new iterate.
 *     3: one cooperative launch for all m inner iterations of an epoch (Alg. 1 steps 5-11 or Alg. 2 steps 5-15
 *       with scheme (a), a dense generalized linear model with n_full == n, d a multiple of 4, 16-byte aligned
 *       rows, a chip of 256 compute units).  256 workgroups stay resident; worker i's rows are read by the
 *       compute units of die i mod 8; partial vectors, folded slices, statistics and iterates pass between
 *       workgroups through device memory as (value, tag) words; one barrier per die and iteration.  Every wait is
 *       bounded by LPC_TUNE_SPIN_LIMIT; a wait that gives up raises an abort word that all workgroups see, the
 *       launch ends, the iterate is unspecified and lpc_take_device_flags reports LPC_EDEVICE.
 *     Measured on MI355X forms 1-3 are slower than form 0 (form 1 pays for device-scope atomics, form 2 for reading
 *     the sampled rows twice, form 3 for dependent instruction chains that a single resident workgroup per compute
 *     unit cannot overlap); they are kept as tested alternatives.
 *     Forms 0 and 1 give the same bits as each other; forms 2 and 3 add the same numbers in another order, so
 *     their u^i differ in the last bits.  Every form gives the same bits from run to run.
 *   LPC_TUNE_ITER_TILE: form 1: coordinates per workgroup of the second launch, 64 or 128;
 *   LPC_TUNE_ITER_THREADS: form 1: its threads per workgroup, 256 or 512;
 *   LPC_TUNE_SPIN_LIMIT: form 1: polls before a workgroup gives up waiting (it then finishes normally with what it
 *     has and lpc_take_device_flags reports LPC_EDEVICE); 0 makes every wait give up at once (tests of that path).
 * LPC_EINVAL for an unknown key or value, LPC_EUNSUPPORTED where the context cannot run the form. */
typedef enum {
  LPC_TUNE_ITER_FORM = 0,
  LPC_TUNE_ITER_TILE = 1,
  LPC_TUNE_ITER_THREADS = 2,
  LPC_TUNE_SPIN_LIMIT = 3
} lpc_tune_key;
lpc_status lpc_tune(lpc_ctx *ctx, int32_t key, int64_t value);

#ifdef __cplusplus
}
#endif
#endif
