/*
 * sv.h - C ABI of the MI355X (gfx950) Speculative Verification hot path.
 *
 * One decode step of Speculative Verification (arxiv 2509.24328) over
 * B sequences x k drafted positions x V vocabulary entries:
 *
 *   sv_row_stats        draft/companion indicators S and A      (Sec. 4.2; appendix defs of S and A)
 *   sv_accept_estimate  binned estimate P^(T_i | S, A)           (appendix def. of the observed probability)
 *   sv_select_length    verification length per sequence         (Sec. 5: E(N|gamma), goodput, batch greedy)
 *   sv_verify_sample    speculative-sampling verification        (Sec. 4.2 last paragraph; Leviathan et al.)
 *
 * The same step in three calls: sv_row_stats, sv_estimate_select (the second and
 * third call in one launch), sv_verify_sample_chained (takes the draft rows'
 * normalisers over from sv_row_stats through the workspace and sweeps the
 * target rows only).  Further down: the profile-construction pass that
 * produces the table, the sampling warps (temperature, top-k, top-p,
 * repetition penalty) with dense and compacted forms of the step, and helpers.
 *
 * Conventions common to all calls
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates, frees or synchronises: each call only enqueues kernels
 *     on `stream` (a hipStream_t passed as void*; NULL = the default stream)
 *     and returns.  Results are valid once the stream has reached that point.
 *   - Tensors are dense row-major with the vocabulary innermost.  Logits are
 *     SV_F32 (IEEE binary32) or SV_BF16 (bfloat16, the upper 16 bits of a
 *     binary32).  Base pointers need only element alignment; rows that start
 *     on a 16-byte boundary (always the case when V*elem_size is a multiple of
 *     16 and the base is 16-byte aligned) take the vector-load path.
 *   - Return value: SV_OK or a negative SV_ERR_* for argument errors detected
 *     on the host (nothing is enqueued then).  Data-dependent conditions (NaN
 *     rows, token ids out of range, near-ties) are never errors: they set
 *     SV_FLAG_* bits in the flags outputs.
 *   - Range of the logits: with y = z * log2(e) / T (T = 1 unless an entry
 *     point takes a temperature), an entry with y < -2^30 - a finite stand-in
 *     for -inf such as -1e30 or the lowest finite number of the type - carries
 *     no probability mass, exactly like -inf; a row whose largest entry is below
 *     that, or has y > 2^30, is reported as a bad row.
 *   - `ws` is caller-provided device scratch of at least
 *     sv_workspace_bytes(B, k, V, dtype) bytes, 256-byte aligned, which may be
 *     reused by the next call on the same stream.  Calls that share a
 *     workspace must not overlap in time.  Its contents mean nothing to the
 *     caller and need no initialisation; the one thing that survives a call is
 *     what sv_row_stats leaves for sv_verify_sample_chained.
 */
#ifndef SV_H_
#define SV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef void* sv_stream_t;

enum { SV_F32 = 0, SV_BF16 = 1 };
enum { SV_BATCH_GREEDY = 0, SV_PER_SEQUENCE = 1 };

enum {
  SV_OK = 0,
  SV_ERR_INVALID_ARG = -1, /* a size is out of range / inconsistent            */
  SV_ERR_NULL = -2,        /* a required pointer is NULL                       */
  SV_ERR_DTYPE = -3,       /* dtype is neither SV_F32 nor SV_BF16              */
  SV_ERR_ALIGN = -4,       /* a pointer is not aligned to its element type     */
  SV_ERR_WORKSPACE = -5,   /* ws is NULL, misaligned or smaller than required  */
  SV_ERR_LAUNCH = -6,      /* the HIP runtime rejected a launch                */
  SV_ERR_TOO_LARGE = -7    /* problem exceeds a documented library limit       */
};

/* Condition bits written to flags outputs. */
enum {
  SV_FLAG_BAD_ROW = 1,            /* a needed row holds NaN/+inf or no entry in range         */
  SV_FLAG_NEAR_TIE = 2,           /* |u - min(1, ratio)| < 1e-6 at an evaluated position      */
  SV_FLAG_RESIDUAL_FALLBACK = 4,  /* residual without mass (exactly 0 / non-finite) or bad
                                     draft row: drawn from the target distribution instead    */
  SV_FLAG_NEAR_CDF_EDGE = 8,      /* sampling threshold within 1e-6 * W (+ 1e-6 absolute on
                                     the dense paths, whose probabilities are float32) of an
                                     edge of the drawn token's CDF interval                   */
  SV_FLAG_BAD_TOKEN = 16,         /* drafted token id outside [0, V)                          */
  SV_FLAG_NOT_COMPACT = 32,       /* a needed row has no compact support (count < 0): the
                                     result is not valid, use the dense warped entry points   */
  SV_FLAG_NO_CHAIN = 64           /* sv_verify_sample_chained: the workspace does not hold the
                                     draft normalisers of these arguments (no sv_row_stats call
                                     on it, or one with another z_d, x, shape, dtype, draft
                                     temperature or draft cutoffs): the draft rows count as bad   */
};

/* Largest B*k accepted by sv_select_length (keys are sorted in one workgroup). */
#define SV_SELECT_MAX_KEYS 8192
/* Largest k accepted by sv_verify_sample. */
#define SV_MAX_K 64
/* Largest number of tensors one sv_warp_*_multi call takes. */
#define SV_WARP_MAX_TENSORS 8
/* Largest history (context + drafted prefix) one sv_repetition_penalty call takes per row. */
#define SV_PENALTY_MAX_TOKENS 4096
/* Largest per-row capacity of a compacted support (sv_warp_compact). */
#define SV_SUPPORT_MAX_CAP 1024

/* Device scratch that sv_verify_sample_static holds on every GPU it runs on. */
#define SV_STATIC_SCRATCH_BYTES (1 << 20)

/* Kernels of the library, for sv_set_timing_events. */
enum {
  SV_KERNEL_ROW_STATS = 0,
  SV_KERNEL_ACCEPT_ESTIMATE = 1,
  SV_KERNEL_SELECT_LENGTH = 2,
  SV_KERNEL_VERIFY_ROWS = 3,    /* first kernel of sv_verify_sample: row normalisers          */
  SV_KERNEL_VERIFY_MASS = 4,    /* second: accept decision, chunk masses of the sampled row    */
  SV_KERNEL_VERIFY_PICK = 5,    /* third: chunk scan, LDS prefix scan, token                   */
  SV_KERNEL_COUNT = 6
};

/* Human-readable name of a status code (static string, never NULL). */
const char* sv_strerror(int status);

/* Bytes of device scratch sv_row_stats / sv_verify_sample need for this shape
 * (0 if the shape is invalid).  sv_row_stats leaves the normalisers of the draft
 * rows in it (see sv_verify_sample_chained); nothing else survives a call. */
size_t sv_workspace_bytes(int B, int k, int V, int dtype);

/*
 * Indicators between draft and companion distributions (Sec. 4.2):
 *   P_d = softmax(z_d[b,i,:]),  P_c = softmax(z_c[b,i,:])
 *   S[b,i] = sum_v min(P_d(v), P_c(v))
 *   A[b,i] = min(1, P_c(x[b,i]) / P_d(x[b,i]))          (1 when P_d(x) = 0)
 * plus the row log-sum-exps and, optionally, KL(P_d || P_c), the draft entropy
 * H(P_d) in nats and the draft's probability of its own token P_d(x) (the signals
 * of the entropy- and probability-based predictors the paper compares with,
 * Sec. 2 "Predicting Speculation Accuracy").
 *   z_d, z_c   [B,k,V] dtype        in
 *   x          [B,k]   int32        in   drafted token ids
 *   lse_d, lse_c, S, A [B,k] float  out  (NaN for bad rows; A NaN for bad tokens)
 *   kl_or_null, entropy_d_or_null, pd_x_or_null [B,k] float   out  optional
 *   flags_or_null [B,k] uint32      out  optional, SV_FLAG_BAD_ROW / SV_FLAG_BAD_TOKEN
 * B, k, V >= 1.  B = 0 is accepted and does nothing.
 * The call also leaves, in ws, the normalisers of the draft rows and the draft
 * logits of the drafted tokens under a header naming its arguments: what
 * sv_verify_sample_chained picks up.  Nothing else reads them.
 */
int sv_row_stats(const void* z_d, const void* z_c, const int32_t* x,
                 int B, int k, int V, int dtype,
                 float* lse_d, float* lse_c, float* S, float* A,
                 float* kl_or_null, float* entropy_d_or_null, float* pd_x_or_null,
                 uint32_t* flags_or_null,
                 void* ws, size_t ws_bytes, sv_stream_t stream);

/*
 * Binned acceptance estimate (appendix definition of P(T_i | S, A)):
 *   p_hat[j] = table[bin(S[j]; edges_s), bin(A[j]; edges_a)]
 * Bins are half-open [e_i, e_{i+1}) over ascending edges, the top bin closed,
 * values outside the edges clamped to the first/last bin, NaN -> bin 0.
 *   S, A        [n] float           in
 *   edges_s     [n_s+1] float, edges_a [n_a+1] float, table [n_s,n_a] float   in
 *   p_hat       [n] float           out
 *   edge_flag_or_null [n] uint8     out  1 when S or A is NaN or lies within 1e-5
 *                                        (float32 |v - e| <= 1e-5f) of an interior edge
 * n >= 0, n_s, n_a >= 1.
 */
int sv_accept_estimate(const float* S, const float* A, int n,
                       const float* edges_s, int n_s,
                       const float* edges_a, int n_a,
                       const float* table,
                       float* p_hat, uint8_t* edge_flag_or_null, sv_stream_t stream);

/*
 * Verification length per sequence (Sec. 5).  With c[b,j] = prod_{i<=j} p_hat[b,i]
 * (estimates clamped to [0,1], NaN -> 0; float64, left to right) the expected
 * accepted length of verifying gamma tokens of b is sum_{j<gamma} c[b,j].
 * SV_BATCH_GREEDY: order all (b,j) by c descending (ties: b, then j, ascending);
 * E_M = sum of the first M keys, accumulated in that order in float64;
 * estimated goodput G_M = E_M / latency[M], G_0 = 0; M* = the largest M such
 * that G_1 < G_2 < ... < G_M* keeps strictly improving from G_0 (first peak);
 * gamma[b] = number of selected keys of sequence b.
 * SV_PER_SEQUENCE: the same search on every sequence alone with latency[0..k].
 *   p_hat   [B,k] float     in
 *   latency [n_latency] float, > 0   in   n_latency >= B*k+1 (batch) or k+1 (per sequence)
 *   gamma   [B] int32       out  0..k
 *   t_offsets [B+1] int32   out  exclusive scan of gamma[b] + 1
 *   total_M [1] int32       out  sum_b gamma[b]
 * Limit: B*k <= SV_SELECT_MAX_KEYS, else SV_ERR_TOO_LARGE.  B = 0 is accepted and
 * does nothing (no output is written), as in the other calls.
 */
int sv_select_length(const float* p_hat, int B, int k,
                     const float* latency, int n_latency, int mode,
                     int32_t* gamma, int32_t* t_offsets, int32_t* total_M,
                     sv_stream_t stream);

/*
 * sv_accept_estimate and sv_select_length in one launch (same sources): the
 * estimates of the B*k positions are looked up from (S, A) by the rule of
 * sv_accept_estimate, written to p_hat, and the lengths are selected from them
 * by the rule of sv_select_length.  Results are those of the two calls; the
 * launch in between is saved, which is what a small batch's step is made of.
 *   S, A [B,k] float in;  edges_s [n_s+1], edges_a [n_a+1], table [n_s,n_a] float in
 *   p_hat [B,k] float out;  edge_flag_or_null [B,k] uint8 out
 *   latency, mode, gamma, t_offsets, total_M, limits and errors as for sv_select_length.
 */
int sv_estimate_select(const float* S, const float* A, int B, int k,
                       const float* edges_s, int n_s, const float* edges_a, int n_a,
                       const float* table, const float* latency, int n_latency, int mode,
                       float* p_hat, uint8_t* edge_flag_or_null,
                       int32_t* gamma, int32_t* t_offsets, int32_t* total_M,
                       sv_stream_t stream);

/*
 * Speculative-sampling verification of the first gamma[b] drafted tokens of
 * each sequence (Sec. 4.2, last paragraph; the rule itself is Leviathan et al.'s):
 * for i < gamma[b] accept x[b,i] iff u_i < p_t(x)/p_d(x); n = leading accepts;
 * then draw one token at position n: from the normalised residual
 * max(0, p_t - p_d) if n < gamma[b], whatever its mass W > 0 (from p_t itself,
 * with SV_FLAG_RESIDUAL_FALLBACK, only when W is exactly 0 or not finite), else
 * from the target distribution of position gamma[b] (bonus token / position
 * the target generates itself).  The probabilities are float32 numbers, so a
 * cumulative weight carries an absolute error of up to 5e-7: when the threshold
 * u' * W lies within 1e-6 * W + 1e-6 of an edge of the drawn token's interval
 * the token next to it may be the exact one, and SV_FLAG_NEAR_CDF_EDGE says so
 * (always the case for residuals of mass below 2e-6, which float32
 * probabilities do not resolve; the emitted law is within that mass of exact).
 * Draws are inverse-CDF over ascending token id: the smallest v whose
 * inclusive cumulative weight exceeds u' * W.
 * Uniforms: Philox-4x32-10, key = (seed lo, seed hi), counter = (i, b, 0, step);
 * word 0 -> u_i, word 1 -> u' for sampling at position i; value ((w>>8)+0.5)*2^-24.
 *   z_t   dense [B,k+1,V] when t_offsets_or_null is NULL, else packed
 *         [n_t_rows,V] with the target row of (b,i), i <= gamma[b], at row t_offsets[b]+i
 *   t_offsets_or_null [B+1] int32   in   optional
 *   n_t_rows          rows in packed z_t (ignored when dense); rows addressed
 *                     beyond it are treated as bad rows, never read
 *   z_d   [B,k,V] dtype, x [B,k] int32                       in
 *   gamma_or_null [B] int32          in   optional (NULL: gamma[b] = k); clamped to 0..k
 *   out_tokens [B,k+1] int32         out  accepted tokens, the drawn token, then -1
 *   n_accept   [B] int32             out
 *   flags      [B] uint32            out  SV_FLAG_* bits
 *   ratio_or_null [B,k] float        out  optional: p_t/p_d at evaluated positions, NaN elsewhere
 * Limits: k <= SV_MAX_K, V <= 16777216.
 */
int sv_verify_sample(const void* z_t, const int32_t* t_offsets_or_null, int n_t_rows,
                     const void* z_d, const int32_t* x, const int32_t* gamma_or_null,
                     int B, int k, int V, int dtype,
                     uint64_t seed, uint32_t step,
                     int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                     float* ratio_or_null,
                     void* ws, size_t ws_bytes, sv_stream_t stream);

/*
 * sv_verify_sample for the step as it runs in serving (Sec. 5 and 6: S and A are
 * computed from the draft and companion logits, the lengths are chosen, the
 * target runs, then verification): the draft rows that verification needs the
 * normalisers of are the rows sv_row_stats has already swept in this step.
 * sv_row_stats (and sv_row_stats_warped) leave those normalisers - row maximum
 * and sum of exponentials in float64, and the draft logit of each drafted token -
 * in the workspace; this call takes them from there and sweeps only the target
 * rows, i.e. sum_b (gamma[b] + 1) rows instead of sum_b (2 gamma[b] + 1).
 * Same arguments, outputs, flags, limits and errors as sv_verify_sample.
 * Requirements: the same ws, z_d, x, B, k, V and dtype as the latest
 * sv_row_stats call on that workspace, which must precede this call on the same
 * stream (or be ordered before it by the caller), and z_d unchanged in between.
 * The kernels check the names (addresses, shape, dtype, draft temperature and
 * cutoff pointer) against a header the statistics pass leaves beside the
 * normalisers; on a mismatch every sequence gets SV_FLAG_NO_CHAIN, its draft
 * rows count as bad rows (SV_FLAG_BAD_ROW: no token accepted) and its token is
 * drawn from the target distribution.  Whether z_d still holds what
 * sv_row_stats read cannot be checked.
 */
int sv_verify_sample_chained(const void* z_t, const int32_t* t_offsets_or_null, int n_t_rows,
                             const void* z_d, const int32_t* x, const int32_t* gamma_or_null,
                             int B, int k, int V, int dtype,
                             uint64_t seed, uint32_t step,
                             int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                             float* ratio_or_null,
                             void* ws, size_t ws_bytes, sv_stream_t stream);

/*
 * sv_verify_sample for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc) and
 * so have no workspace to pass: the same kernels run on a scratch array of
 * SV_STATIC_SCRATCH_BYTES that the library holds in device memory on every GPU
 * it is used on, until the process ends.  Arguments, outputs, flags and errors
 * are those of sv_verify_sample without ws / ws_bytes.  The call itself
 * allocates and frees nothing.
 * Limit: sv_workspace_bytes(B, k, V, dtype) <= SV_STATIC_SCRATCH_BYTES (the
 * headline shape B=64, k=8, V=152064 needs 135 KB), else SV_ERR_TOO_LARGE.
 * All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (two streams, two host threads) race and give undefined results;
 * calls that follow each other on one stream are fine, nothing in the array
 * has to survive from one call to the next or to start at zero.
 */
int sv_verify_sample_static(const void* z_t, const int32_t* t_offsets_or_null, int n_t_rows,
                            const void* z_d, const int32_t* x, const int32_t* gamma_or_null,
                            int B, int k, int V, int dtype,
                            uint64_t seed, uint32_t step,
                            int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                            float* ratio_or_null, sv_stream_t stream);

/* ------------------------------------------------------------------------
 * Profile construction and information gain: the offline pass that produces
 * the table sv_accept_estimate looks up (appendix definition of the observed
 * P(T_i | S, A); Sec. 7.3 "Information Gain from S and A", Table 1).
 * ------------------------------------------------------------------------ */

/*
 * Acceptance ratio p_t(x)/p_d(x) of EVERY drafted position (no early stop, no
 * sampling); X = min(1, ratio) is the acceptance probability the profile bins.
 *   z_t   dense [B, t_rows_per_seq, V], t_rows_per_seq = k or k+1 (a bonus row,
 *         if present, is not read);  z_d [B,k,V];  x [B,k] int32        in
 *   ratio [B,k] float                out  NaN for bad rows / tokens
 *   flags_or_null [B,k] uint32       out  SV_FLAG_BAD_ROW / SV_FLAG_BAD_TOKEN
 * Same workspace as sv_verify_sample.
 */
int sv_accept_ratio(const void* z_t, int t_rows_per_seq, const void* z_d, const int32_t* x,
                    int B, int k, int V, int dtype,
                    float* ratio, uint32_t* flags_or_null,
                    void* ws, size_t ws_bytes, sv_stream_t stream);

/*
 * Equal-count ("adaptive": smaller bins where samples are denser) edges of one
 * axis: edges[0] = lo, edges[n_bins] = hi, edges[j] = the floor(j*m/n_bins)-th
 * smallest (0-based) of the m non-NaN samples (lo when m = 0).
 *   values [n] float   in;   edges [n_bins+1] float   out.   Limit: n <= 8192.
 */
int sv_quantile_edges(const float* values, int n, int n_bins, float lo, float hi,
                      float* edges, sv_stream_t stream);

/*
 * Add n samples to the joint histogram counts[n_s, n_a, n_x] (uint32) and to
 * the per-cell sums sum_x[n_s, n_a] (double) of X = clip(ratio, 0, 1).  Cells
 * follow the bin rule of sv_accept_estimate; the X bin is
 * min(n_x-1, floor(X * n_x)) in float32.  Samples with a NaN in S, A or ratio
 * are skipped.  The caller zeroes counts and sum_x before the first batch.
 * Limit: n_x <= 1024.
 */
int sv_profile_accumulate(const float* S, const float* A, const float* ratio, int n,
                          const float* edges_s, int n_s, const float* edges_a, int n_a, int n_x,
                          uint32_t* counts, double* sum_x, sv_stream_t stream);

/*
 * table[n_s, n_a] (float) = mean X of each cell, empty cells = the global mean
 * (0 when there is no sample); info[0..2] (double) = H(X), H(X | S,A) and the
 * information gain I(X; S,A) = H(X) - H(X | S,A), in bits, over the binned
 * variables.
 */
int sv_profile_finalize(const uint32_t* counts, const double* sum_x, int n_s, int n_a, int n_x,
                        float* table, double* info, sv_stream_t stream);

/* ------------------------------------------------------------------------
 * Sampling warps (appendix table "Sampling hyperparameters for each model
 * series": temperature, top-k, top-p; applied in that order).
 * ------------------------------------------------------------------------ */

/*
 * Per-row cutoff such that the warped distribution is soft-max(z / temperature)
 * restricted to {v : z_v >= cutoff[row]}.  top-k keeps the entries at least as
 * large as the K-th largest value; top-p then keeps, over those, whole groups of
 * equal value from the top until their mass reaches top_p.  top_k <= 0 or >= V
 * and top_p >= 1 switch the respective warp off (cutoff = -inf keeps all).
 *   z       [rows, V] dtype    in
 *   cutoff  [rows] float       out  a value of the row, -inf, or NaN for a bad row
 *   flags_or_null [rows] uint32 out SV_FLAG_BAD_ROW; SV_FLAG_NEAR_TIE when the top-p
 *                                   decision lies within 3e-6 of top_p
 * temperature in [1e-3, 1e3], top_p > 0; otherwise SV_ERR_INVALID_ARG.
 */
int sv_warp_cutoffs(const void* z, int rows, int V, int dtype,
                    float temperature, int top_k, float top_p,
                    float* cutoff, uint32_t* flags_or_null, sv_stream_t stream);

/*
 * sv_warp_cutoffs for up to SV_WARP_MAX_TENSORS logit tensors of one vocabulary size
 * and dtype in one launch (the draft, companion and target logits of a step, each
 * with the sampling hyper-parameters of its model series).  The rows are independent,
 * so the results are those of one sv_warp_cutoffs call per tensor; one launch over
 * all rows keeps the memory system busy while some rows are being decided.
 *   n                         number of tensors
 *   z, rows, temperature, top_k, top_p, cutoff, flags_or_null
 *                             HOST arrays of length n holding, per tensor, the
 *                             arguments of sv_warp_cutoffs (z[t], cutoff[t],
 *                             flags_or_null[t] are device pointers; flags_or_null
 *                             itself, or single entries of it, may be NULL)
 */
int sv_warp_cutoffs_multi(int n, const void* const* z, const int* rows, int V, int dtype,
                          const float* temperature, const int* top_k, const float* top_p,
                          float* const* cutoff, uint32_t* const* flags_or_null, sv_stream_t stream);

/*
 * Repetition penalty (appendix table of sampling hyper-parameters; the usual
 * logits processor), in place, to be applied before the other warps: for every
 * row (b, i) and every distinct token t of its history, z[t] becomes z[t] / penalty
 * if z[t] > 0, else z[t] * penalty.  History of row (b, i): history[b, :], plus
 * x[b, 0 .. min(i, k) - 1] when x is given (the tokens drafted before position i).
 * Token ids outside [0, V) (padding: -1) are ignored.  float32 arithmetic (the
 * division correctly rounded); bfloat16 logits are rounded to nearest-even.
 *   z        dense [B, rows_per_seq, V], or packed [n_rows, V] with
 *            row_offsets_or_null [B+1] int32: sequence b owns rows
 *            row_offsets[b] .. row_offsets[b+1]-1 (at most rows_per_seq of them are
 *            touched; a range outside [0, n_rows] is skipped)          in/out
 *   history  [B, n_hist] int32 (may be NULL when n_hist = 0)            in
 *   x_or_null [B, k] int32                                              in
 * penalty > 0.  Limits: n_hist (+ k with x) <= SV_PENALTY_MAX_TOKENS; B,
 * rows_per_seq <= 65535.  Calls on tensors that share rows must not overlap.
 */
int sv_repetition_penalty(void* z, const int32_t* row_offsets_or_null, int n_rows, int B, int rows_per_seq,
                          int V, int dtype, const int32_t* history, int n_hist,
                          const int32_t* x_or_null, int k, float penalty, sv_stream_t stream);

/*
 * sv_repetition_penalty on up to SV_WARP_MAX_TENSORS logit tensors of one batch in
 * one launch (the draft, companion and target logits of a step share B, V, dtype,
 * the history and the drafted tokens; they differ in their rows per sequence and
 * in whether they are packed).
 *   z, row_offsets_or_null, n_rows_or_null, rows_per_seq   HOST arrays of length n with the
 *        per-tensor arguments of sv_repetition_penalty (row_offsets_or_null itself, or
 *        single entries of it, may be NULL = dense; n_rows_or_null may be NULL when
 *        row_offsets_or_null is)
 */
int sv_repetition_penalty_multi(int n, void* const* z, const int32_t* const* row_offsets_or_null,
                                const int* n_rows_or_null, int B, const int* rows_per_seq, int V, int dtype,
                                const int32_t* history, int n_hist, const int32_t* x_or_null, int k,
                                float penalty, sv_stream_t stream);

/*
 * sv_row_stats on warped distributions: P_d = soft-max(z_d / temperature_d) over
 * {v : z_d[v] >= cutoff_d[row]}, P_c likewise with its own temperature and
 * cutoffs (the draft and the companion are run with the sampling
 * hyper-parameters of their model series; Sec. 4.2 for S and A, the appendix
 * table of sampling hyper-parameters for the warps).  Everything else - shapes,
 * outputs, flags, workspace, errors - is as for sv_row_stats; lse_d / lse_c are
 * the normalisers of the warped rows z / T.
 *   cutoff_d_or_null, cutoff_c_or_null  [B*k] float in  one cutoff per logit row as
 *        written by sv_warp_cutoffs on the same tensor (NaN or -inf: keep every
 *        entry); NULL = no cutoff for that tensor
 * A drafted token outside the draft's support has P_d(x) = 0 and gives A = 1,
 * as an entry at -inf does in sv_row_stats; KL is +inf when the companion's
 * support misses part of the draft's.
 * Temperatures must lie in [1e-3, 1e3], else SV_ERR_INVALID_ARG.
 */
int sv_row_stats_warped(const void* z_d, const void* z_c, const int32_t* x,
                        int B, int k, int V, int dtype,
                        float temperature_d, const float* cutoff_d_or_null,
                        float temperature_c, const float* cutoff_c_or_null,
                        float* lse_d, float* lse_c, float* S, float* A,
                        float* kl_or_null, float* entropy_d_or_null, float* pd_x_or_null,
                        uint32_t* flags_or_null,
                        void* ws, size_t ws_bytes, sv_stream_t stream);

/*
 * sv_verify_sample on warped distributions (same sources as above; the
 * accept / residual / bonus rule is unchanged and acts on the warped target and
 * draft distributions).
 *   cutoff_t_or_null  [rows of z_t] float in  one cutoff per logit row of z_t, indexed
 *        like z_t itself (dense: b * (k+1) + i; packed: t_offsets[b] + i)
 *   cutoff_d_or_null  [B*k] float in
 * Everything else is as for sv_verify_sample.  Temperatures in [1e-3, 1e3].
 */
int sv_verify_sample_warped(const void* z_t, const int32_t* t_offsets_or_null, int n_t_rows,
                            const void* z_d, const int32_t* x, const int32_t* gamma_or_null,
                            int B, int k, int V, int dtype,
                            float temperature_t, const float* cutoff_t_or_null,
                            float temperature_d, const float* cutoff_d_or_null,
                            uint64_t seed, uint32_t step,
                            int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                            float* ratio_or_null, void* ws, size_t ws_bytes, sv_stream_t stream);

/*
 * sv_verify_sample_chained on warped distributions: the draft normalisers are
 * those sv_row_stats_warped left in the workspace, so temperature_d and
 * cutoff_d_or_null must be the draft temperature and cutoff array that call was
 * given (checked by value and by address; SV_FLAG_NO_CHAIN otherwise).
 */
int sv_verify_sample_warped_chained(const void* z_t, const int32_t* t_offsets_or_null, int n_t_rows,
                                    const void* z_d, const int32_t* x, const int32_t* gamma_or_null,
                                    int B, int k, int V, int dtype,
                                    float temperature_t, const float* cutoff_t_or_null,
                                    float temperature_d, const float* cutoff_d_or_null,
                                    uint64_t seed, uint32_t step,
                                    int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                                    float* ratio_or_null, void* ws, size_t ws_bytes, sv_stream_t stream);

/*
 * sv_accept_ratio on warped distributions, on the logits themselves (for rows
 * whose support does not compact, and for profiles built without compaction):
 * X = P_t(x) / P_d(x) of every drafted position with P_t = soft-max(z_t / T_t) over
 * {v : z_t[v] >= cutoff_t[row]} and P_d likewise.
 *   cutoff_t_or_null  [B * t_rows_per_seq] float in  one cutoff per row of z_t (dense
 *        layout b * t_rows_per_seq + i), as written by sv_warp_cutoffs on z_t
 *   cutoff_d_or_null  [B*k] float in
 * +inf where the draft's support misses the token but the target's holds it, NaN
 * where neither holds it.  Everything else is as for sv_accept_ratio.
 */
int sv_accept_ratio_warped(const void* z_t, int t_rows_per_seq, const void* z_d, const int32_t* x,
                           int B, int k, int V, int dtype,
                           float temperature_t, const float* cutoff_t_or_null,
                           float temperature_d, const float* cutoff_d_or_null,
                           float* ratio, uint32_t* flags_or_null,
                           void* ws, size_t ws_bytes, sv_stream_t stream);

/* ------------------------------------------------------------------------
 * The step on compacted supports.  With the paper's sampling hyper-parameters
 * (top-k 20, or top-p 0.6-0.9 at temperature 0.6-0.95) a warped distribution
 * lives on a few dozen tokens, so one pass per logit tensor that writes each
 * row's support replaces every later sweep over the vocabulary.
 * ------------------------------------------------------------------------ */

/*
 * sv_warp_cutoffs plus the support of every warped row:
 *   count  [rows] int32        out  number of kept tokens n_r; 0 for a bad row; -1 when the
 *                                   support is wider than cap or could not be settled on the
 *                                   kernel's candidate list (flat rows): use the dense path
 *   token  [rows, cap] int32   out  kept token ids, ascending, entries 0..n_r-1
 *   prob   [rows, cap] double  out  their probabilities under soft-max(z / T) restricted to
 *                                   the kept set (entries of zero probability are not listed)
 *   lse    [rows] float        out  log-sum-exp of z / T over the kept set (NaN: bad row / -1)
 *   cutoff_or_null, flags_or_null   as in sv_warp_cutoffs
 * 1 <= cap <= SV_SUPPORT_MAX_CAP.  Entries beyond n_r are left untouched.
 * Rows are independent, so tensors that share the hyper-parameters and lie one
 * after the other in memory (draft and companion logits, say) can go through
 * one call with rows = the sum: a launch with more than two rows per compute
 * unit overlaps the decisions of some rows with the sweeps of others.
 */
int sv_warp_compact(const void* z, int rows, int V, int dtype,
                    float temperature, int top_k, float top_p, int cap,
                    int32_t* count, int32_t* token, double* prob, float* lse,
                    float* cutoff_or_null, uint32_t* flags_or_null, sv_stream_t stream);

/*
 * sv_warp_compact for up to SV_WARP_MAX_TENSORS tensors in one launch: HOST arrays of
 * length n as in sv_warp_cutoffs_multi, plus the per-tensor output arrays of
 * sv_warp_compact (one capacity for all).
 */
int sv_warp_compact_multi(int n, const void* const* z, const int* rows, int V, int dtype,
                          const float* temperature, const int* top_k, const float* top_p, int cap,
                          int32_t* const* count, int32_t* const* token, double* const* prob,
                          float* const* lse, float* const* cutoff_or_null,
                          uint32_t* const* flags_or_null, sv_stream_t stream);

/*
 * sv_row_stats on compacted supports (draft and companion, one support per
 * (b, i) as written by sv_warp_compact with the same cap): S, A and the optional
 * KL, entropy and P_d(x), in fp64 over the listed tokens.  Outputs and flags as in
 * sv_row_stats; lse_d / lse_c are copied from the supports.  A pair with a count
 * of -1 on either side gets NaN outputs and SV_FLAG_NOT_COMPACT.
 *   V  vocabulary size, only to range-check the drafted tokens
 */
int sv_row_stats_sparse(const int32_t* count_d, const int32_t* token_d, const double* prob_d, const float* lse_d_in,
                        const int32_t* count_c, const int32_t* token_c, const double* prob_c, const float* lse_c_in,
                        int cap, const int32_t* x, int B, int k, int V,
                        float* lse_d, float* lse_c, float* S, float* A,
                        float* kl_or_null, float* entropy_d_or_null, float* pd_x_or_null,
                        uint32_t* flags_or_null, sv_stream_t stream);

/*
 * sv_verify_sample on compacted supports: same rule, same Philox addressing,
 * same outputs and flags.  The target supports are indexed like the rows of z_t
 * (dense: b * (k+1) + i; packed: t_offsets[b] + i, with n_t_rows rows in all),
 * the draft supports by b * k + i.  A sequence that needs a row with a count of
 * -1 gets SV_FLAG_NOT_COMPACT | SV_FLAG_BAD_ROW and must be redone densely.
 */
int sv_verify_sample_sparse(const int32_t* count_t, const int32_t* token_t, const double* prob_t,
                            const int32_t* t_offsets_or_null, int n_t_rows,
                            const int32_t* count_d, const int32_t* token_d, const double* prob_d,
                            int cap, const int32_t* x, const int32_t* gamma_or_null,
                            int B, int k, int V, uint64_t seed, uint32_t step,
                            int32_t* out_tokens, int32_t* n_accept, uint32_t* flags,
                            float* ratio_or_null, sv_stream_t stream);

/*
 * sv_accept_ratio on compacted supports: X = P_t(x) / P_d(x) of every drafted
 * position under the warped distributions (profile construction with the sampling
 * hyper-parameters in force).  Target supports: t_rows_per_seq (k or k+1) rows per
 * sequence.  NaN with SV_FLAG_BAD_ROW / SV_FLAG_BAD_TOKEN / SV_FLAG_NOT_COMPACT where
 * the ratio is not available; +inf where the draft gives the token no mass.
 */
int sv_accept_ratio_sparse(const int32_t* count_t, const int32_t* token_t, const double* prob_t,
                           int t_rows_per_seq, const int32_t* count_d, const int32_t* token_d,
                           const double* prob_d, int cap, const int32_t* x, int B, int k, int V,
                           float* ratio, uint32_t* flags_or_null, sv_stream_t stream);

/*
 * The uniforms sv_verify_sample draws (for tests and for callers that want to
 * replay a step): Philox-4x32-10 with counter (i, b, 0, step) and key (seed low,
 * seed high); output word 0 -> accept uniform of drafted position i, word 1 ->
 * sampling uniform of position i; value ((w >> 8) + 0.5) * 2^-24.
 *   u_accept, u_sample  [B, n_pos] double  out
 */
int sv_uniforms(uint64_t seed, uint32_t step, int B, int n_pos, double* u_accept, double* u_sample,
                sv_stream_t stream);

/*
 * Timing taps for benchmarks (not part of the method): while a pair of
 * hipEvent_t handles is set for `kernel`, every launch of that kernel records
 * `start_event` immediately before and `stop_event` immediately after it on the
 * launch stream, so that hipEventElapsedTime(start, stop) brackets that kernel
 * alone.  Pass NULLs to clear.  The setting is process-wide (it applies to the
 * launches of every thread) and may be changed from any thread at any time: a
 * launch sees either the old pair or the new one.  The events must outlive the
 * launches.  Returns SV_ERR_INVALID_ARG for an
 * unknown kernel id or when only one of the two events is given.
 */
int sv_set_timing_events(int kernel, void* start_event, void* stop_event);

#ifdef __cplusplus
}
#endif
#endif /* SV_H_ */
