/* tslt.h -- C ABI of the MI355X (gfx950) hot path of Truncated Sparse Logits Transmission.
 *
 * The operations are the per-position probability steps of the paper "Fast Collaborative Inference
 * via Distributed Speculative Decoding":
 *   device side  -- truncated sampling on the draft logits (Section 3.1: Top-K, Top-rho, the
 *                   renormalisation equation) and "sparsify-then-sample" (Solution 1, Section 3.2);
 *   server side  -- token-sequence verification (Algorithm 3), multi-candidate verification
 *                   (Algorithm 5 and its residual-update equation) and token-tree verification with
 *                   the new-sequence search (Algorithm 8; tree layout of Section 4.1).
 *
 * Conventions that hold for every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller unless it is marked "host".  The library
 *     allocates nothing: scratch memory comes from a caller-provided workspace sized by
 *     tslt_workspace_bytes() and aligned to 256 bytes (tslt_verify_static alone uses an array of its own).
 *   - `stream` is a hipStream_t passed as void*.  Calls enqueue kernels on it and return without
 *     synchronising; outputs are valid once the stream has reached that point.
 *   - Return value: TSLT_OK, or a negative code for an error found on the host (bad argument,
 *     workspace too small, launch failure).  Nothing is enqueued when a negative code is returned.
 *     tslt_last_error() gives a message for the calling thread.
 *   - Data-dependent problems never abort.  They set bits in the optional per-row / per-sequence
 *     `status` array (TSLT_ROW_*) and give the defined fallback (count 0, token -1).
 *   - Logit rows are row-major with `row_stride` elements between rows; any alignment of the element
 *     type is accepted.  A row must be shorter than 4 GiB, and V below 2^31 (TSLT_ERR_UNSUPPORTED otherwise).  dtype is fp32, bf16 or binary16 (16-bit elements are widened exactly to fp32 on load).
 *   - Temperature (not in the paper): s = fl32(z * fl32(1/T)), one fp32 multiplication per logit.
 *     The SCALED values are what a truncated set carries, so the server needs no draft-side
 *     parameter: q_hat is the plain softmax of the received values.  T must be > 0.
 *   - Order of a truncated set ("canonical order"): raw logit descending, ties by ascending token
 *     index.  Logits equal to -inf have probability 0 and are never selected; NaN or +inf marks the
 *     row TSLT_ROW_NONFINITE.
 *   - A truncated set handed to the server side (q_idx, q_logit, q_count) must hold DISTINCT token indices in
 *     [0, V) and finite values, none more than 700 above the first (tslt_truncate writes them in descending
 *     order, so its sets always qualify).  A value that is not finite or an index outside the vocabulary is
 *     found and reported as TSLT_ROW_BAD_SET; repeated indices are not looked for (they would be counted twice).
 *   - Sampling is inverse-CDF with caller-supplied uniforms u in [0,1): the first bucket whose
 *     cumulative weight exceeds u * total, accumulated in fp64.  Dense distributions are scanned in
 *     ascending token index, sparse ones in canonical order.  Uniforms are indexed by position /
 *     node, never by control flow, so results do not depend on evaluation order.
 */
#ifndef TSLT_H
#define TSLT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element type of logit rows, and format of travelling values: fp32, bfloat16, IEEE binary16 */
typedef enum { TSLT_F32 = 0, TSLT_BF16 = 1, TSLT_F16 = 2 } tslt_dtype;

enum {
  TSLT_OK = 0,
  TSLT_ERR_INVALID_ARG = -1,
  TSLT_ERR_UNSUPPORTED = -2,  /* a size beyond what the kernels are built for (see TSLT_MAX_K_CAP) */
  TSLT_ERR_WORKSPACE = -3,    /* workspace missing, misaligned or smaller than tslt_workspace_bytes() */
  TSLT_ERR_HIP = -4           /* a HIP runtime call failed */
};

/* bits of the per-row / per-sequence status words */
enum {
  TSLT_ROW_NONFINITE = 1,        /* NaN or +inf among the logits of a row that was needed */
  TSLT_ROW_EMPTY = 2,            /* no logit above -inf, or an empty sparse set */
  TSLT_ROW_TOKEN_NOT_IN_SET = 4, /* a draft token / candidate that is not in its sparse set: rejected */
  TSLT_ROW_BAD_SET = 8,          /* a received set with a value that is not finite or an index outside [0, V): the
                                    position counts as unusable (as for TSLT_ROW_NONFINITE) */
  TSLT_ROW_EXACT_PATH = 256      /* informational: the row took the multi-pass selection path */
};

enum {
  TSLT_OP_TRUNCATE = 0,
  TSLT_OP_SAMPLE = 1,
  TSLT_OP_VERIFY = 2,
  TSLT_OP_VERIFY_TREE = 3,      /* tslt_verify_tree with node outputs: every node is evaluated */
  TSLT_OP_VERIFY_TREE_PATH = 4  /* tslt_verify_tree without node outputs: only the verified path is sampled */
};

#define TSLT_MAX_K_CAP 1024   /* largest width of a sparse set */
#define TSLT_MAX_TREE_DEPTH 16
#define TSLT_MAX_BRANCH 16    /* largest k_l of an expansion configuration */

/* Library version (major*10000 + minor*100 + patch). */
int tslt_version(void);

/* Message of the last error returned to the calling thread ("" if none).  Host pointer, valid until
 * the next failing call on this thread. */
const char* tslt_last_error(void);

/* Bytes of workspace an operation needs.  `n_outer` is the number of rows (truncate, sample) or of
 * sequences B (verify, verify_tree); `n_inner` is gamma (verify) or N_nodes (verify_tree), ignored
 * otherwise.  Returns 0 when the operation uses none. */
size_t tslt_workspace_bytes(int op, int64_t n_outer, int64_t n_inner, int64_t V, int32_t k_cap);

/* Truncated sampling on logits (Section 3.1; Solution 1 of Section 3.2), one draft row per position.
 *
 *   logits      [rows, row_stride] draft logits z
 *   temperature T > 0
 *   top_k       K of Top-K; 0 = off.  Effective selection size is min(K, k_cap, #logits > -inf)
 *   top_p       rho of Top-rho in (0,1); 0 or >= 1 = off.  The kept set is the smallest prefix of the
 *               canonical order whose mass, measured against the FULL-vocabulary normaliser, is
 *               >= rho; it is cut at the selection size above without changing that test
 *   k_cap       width of the outputs, 1..TSLT_MAX_K_CAP
 *   payload     format in which the kept values will travel (Section 2.2's b_prob bits per value):
 *               TSLT_F32 the scaled logits as computed; TSLT_BF16 / TSLT_F16 each value rounded to nearest-
 *               even to that format (clamped to its finite range).  The kept set, its count and out_mass do
 *               not depend on it; out_logit, out_prob and (tslt_truncate_sample) the draws do: q_hat is the
 *               softmax of the values as the receiver will decode them
 *   out_idx     [rows, k_cap] int32 token ids in canonical order; -1 beyond count
 *   out_logit   [rows, k_cap] fp32 scaled logits s of the kept tokens (the payload; exactly representable
 *               in the payload format); -inf beyond count
 *   out_prob    [rows, k_cap] fp32 q_hat = q / sum_{kept} q (renormalisation equation); 0 beyond
 *               count; may be NULL
 *   out_count   [rows] int32 size of the kept set
 *   out_mass    [rows] fp32 rho-mass of the kept set, sum_{kept} q (sigma of Theorem 1 = 1 - mass);
 *               may be NULL
 *   status      [rows] int32 TSLT_ROW_* bits (written, not accumulated); may be NULL
 * Workspace: none (ws may be NULL).
 */
int tslt_truncate(const void* logits, tslt_dtype dt, int64_t rows, int64_t V, int64_t row_stride,
                  float temperature, int32_t top_k, float top_p, int32_t k_cap, tslt_dtype payload,
                  int32_t* out_idx, float* out_logit, float* out_prob, int32_t* out_count,
                  float* out_mass, int32_t* status, void* ws, size_t ws_bytes, void* stream);

/* Sample from truncated distributions (the sample step of Algorithm 2; Algorithm 4 for k candidates).
 *
 *   idx, logit, count   a truncated set per row as written by tslt_truncate ([rows, k_cap], [rows])
 *   u                   [rows, n_samples] fp32 uniforms in [0,1)
 *   without_replacement 0: the n_samples draws are i.i.d. from q_hat (Algorithm 4);
 *                       1: each drawn slot is removed and the rest renormalised before the next draw
 *   out_token           [rows, n_samples] int32 sampled token ids (-1 if the set is empty or exhausted)
 *   out_slot            [rows, n_samples] int32 position of the token inside its set; may be NULL
 * Workspace: none.
 */
int tslt_sample(const int32_t* idx, const float* logit, const int32_t* count, int64_t rows,
                int32_t k_cap, const float* u, int32_t n_samples, int32_t without_replacement,
                int32_t* out_token, int32_t* out_slot, void* stream);

/* "Sparsify-then-sample" (Solution 1 of Section 3.2) in one launch: tslt_truncate followed by n_samples
 * draws from each row's q_hat (Algorithm 4's candidate draws; n_samples = 1 for a chain), with the same
 * results as tslt_truncate followed by tslt_sample with the same without_replacement.
 *
 *   arguments up to `status`   as for tslt_truncate
 *   u           [rows, n_samples] fp32 uniforms in [0,1)
 *   n_samples   1..TSLT_MAX_BRANCH
 *   without_replacement   as for tslt_sample
 *   out_token   [rows, n_samples] int32 sampled token ids (-1 if the row's set is empty or used up)
 *   out_slot    [rows, n_samples] int32 position of the token inside its set; may be NULL
 * Workspace: none.
 */
int tslt_truncate_sample(const void* logits, tslt_dtype dt, int64_t rows, int64_t V, int64_t row_stride,
                         float temperature, int32_t top_k, float top_p, int32_t k_cap, tslt_dtype payload,
                         int32_t* out_idx, float* out_logit, float* out_prob, int32_t* out_count,
                         float* out_mass, int32_t* status,
                         const float* u, int32_t n_samples, int32_t without_replacement,
                         int32_t* out_token, int32_t* out_slot, void* ws, size_t ws_bytes, void* stream);

/* Wire format of truncated sets (Section 2.2 fixes the size of the payload, K pairs of a b_idx-bit token id
 * and a b_prob-bit value per position; the layout is defined here).  The stream of one row, least significant
 * bit first: 16 bits count, then per kept entry, in canonical order, b_idx = ceil(log2 V) bits of token id
 * followed by the 16 bits of the value (bfloat16 or binary16; values are rounded as by tslt_truncate's
 * `payload`, so sets truncated with the same format pack without loss).  Rows are padded with zero bits to
 * whole 32-bit words and concatenated.  Bit p of a row's stream is bit p % 32 of its word p / 32.
 *
 *   tslt_pack_bound_words  host function: the words tslt_pack can need for `rows` rows (every row full)
 *   idx, logit, count      truncated sets as written by tslt_truncate ([rows, k_cap], [rows])
 *   payload                TSLT_BF16 or TSLT_F16
 *   out_words              [out_capacity_words] uint32; out_capacity_words >= tslt_pack_bound_words(...)
 *   out_row_offset         [rows + 1] int64: first word of every row; entry `rows` is the total, so that
 *                          32 * out_row_offset[rows] bits travel, of which sum_r count_r * (b_idx + 16) are
 *                          Section 2.2's D
 * tslt_unpack is the inverse: out_idx / out_logit / out_count as tslt_truncate writes them (-1 / -inf beyond
 * count).  A count that exceeds k_cap, or what its row's words hold, is cut to that.
 * Workspace: none.
 */
int64_t tslt_pack_bound_words(int64_t rows, int32_t k_cap, int64_t V);
int tslt_pack(const int32_t* idx, const float* logit, const int32_t* count, int64_t rows, int32_t k_cap, int64_t V,
              tslt_dtype payload, uint32_t* out_words, int64_t out_capacity_words, int64_t* out_row_offset,
              void* stream);
int tslt_unpack(const uint32_t* words, const int64_t* row_offset, int64_t rows, int32_t k_cap, int64_t V,
                tslt_dtype payload, int32_t* out_idx, float* out_logit, int32_t* out_count, void* stream);

/* Token-sequence verification (Algorithm 3) for B sequences of gamma draft positions.
 *
 *   target_logits [B, gamma+1, row_stride] target logits; row gamma is the bonus row P_{L+1}
 *   target_temperature  T_p > 0 applied to the target rows as in tslt_truncate
 *   q_idx, q_logit [B, gamma, k_cap], q_count [B, gamma]  the received truncated sets
 *   draft_tokens  [B, gamma] int32 the drafted x_j
 *   u_accept      [B, gamma], u_resample [B, gamma+1] fp32 uniforms in [0,1)
 *   out_accept_len [B] int32 number of accepted draft tokens n in 0..gamma: x_j is accepted iff
 *                 u_accept[j] < min(1, p_j(x_j) / q_hat_j(x_j)) and every earlier one was
 *   out_tokens    [B, gamma+1] int32: the n accepted tokens, then the token resampled from
 *                 norm(max(0, p - q_hat)) at the first rejected position (uniform u_resample[n]), or,
 *                 if n = gamma, the bonus token drawn from p_{gamma+1} (u_resample[gamma]); -1 after
 *   out_ratio     [B, gamma] fp32 p/q_hat for every position (all are evaluated, as the algorithm
 *                 verifies in parallel); -1 where the token is not in its set; may be NULL
 *   out_beta      [B, gamma] fp32 sum_x min(q_hat, p) per position (Lemma 1's acceptance rate); may
 *                 be NULL
 *   status        [B] int32; may be NULL
 * Workspace: tslt_workspace_bytes(TSLT_OP_VERIFY, B, gamma, V, k_cap).
 */
int tslt_verify(const void* target_logits, tslt_dtype dt, int64_t B, int32_t gamma, int64_t V,
                int64_t row_stride, float target_temperature,
                const int32_t* q_idx, const float* q_logit, const int32_t* q_count, int32_t k_cap,
                const int32_t* draft_tokens, const float* u_accept, const float* u_resample,
                int32_t* out_accept_len, int32_t* out_tokens, float* out_ratio, float* out_beta,
                int32_t* status, void* ws, size_t ws_bytes, void* stream);

/* The two halves of tslt_verify as separate calls, for callers that want to put work (or timing
 * events) between them; same arguments, same workspace.  tslt_verify_accept evaluates the acceptance
 * tests of Algorithm 3 for every position (writes out_ratio, out_beta and the decisions, into the
 * workspace); tslt_verify_resample then finds the first rejection, draws the replacement or bonus
 * token and writes out_accept_len, out_tokens and status.  tslt_verify == accept followed by resample
 * on the same stream with the same workspace. */
int tslt_verify_accept(const void* target_logits, tslt_dtype dt, int64_t B, int32_t gamma, int64_t V,
                       int64_t row_stride, float target_temperature,
                       const int32_t* q_idx, const float* q_logit, const int32_t* q_count, int32_t k_cap,
                       const int32_t* draft_tokens, const float* u_accept, const float* u_resample,
                       int32_t* out_accept_len, int32_t* out_tokens, float* out_ratio, float* out_beta,
                       int32_t* status, void* ws, size_t ws_bytes, void* stream);
int tslt_verify_resample(const void* target_logits, tslt_dtype dt, int64_t B, int32_t gamma, int64_t V,
                         int64_t row_stride, float target_temperature,
                         const int32_t* q_idx, const float* q_logit, const int32_t* q_count, int32_t k_cap,
                         const int32_t* draft_tokens, const float* u_accept, const float* u_resample,
                         int32_t* out_accept_len, int32_t* out_tokens, float* out_ratio, float* out_beta,
                         int32_t* status, void* ws, size_t ws_bytes, void* stream);

/* tslt_verify with the acceptance tests taken in stages (Algorithm 3 stops at the first rejection: the
 * positions after it need not be looked at).  Stage 0 covers the first `first_stage` positions of every
 * sequence, stage 1 the next `first_stage`, and every later stage twice as many as the one before it; a
 * stage is one launch, and a sequence that an earlier stage has rejected is skipped in it, so the target
 * rows of its remaining positions are never read.  accept_len, tokens and status are those of
 * tslt_verify; out_ratio and out_beta are NaN at the positions of skipped stages (positions of the stage
 * that holds the first rejection are all evaluated).  first_stage = 0 or >= gamma is tslt_verify itself.
 * Pays when B * first_stage rows fill the GPU (B in the thousands); at a few hundred sequences the
 * stages are too small to reach the memory bandwidth and the single launch is faster.
 * tslt_verify_accept_staged is the staged counterpart of tslt_verify_accept; it is followed by
 * tslt_verify_resample. */
int tslt_verify_staged(const void* target_logits, tslt_dtype dt, int64_t B, int32_t gamma, int64_t V,
                       int64_t row_stride, float target_temperature,
                       const int32_t* q_idx, const float* q_logit, const int32_t* q_count, int32_t k_cap,
                       const int32_t* draft_tokens, const float* u_accept, const float* u_resample,
                       int32_t* out_accept_len, int32_t* out_tokens, float* out_ratio, float* out_beta,
                       int32_t* status, void* ws, size_t ws_bytes, void* stream, int32_t first_stage);
int tslt_verify_accept_staged(const void* target_logits, tslt_dtype dt, int64_t B, int32_t gamma, int64_t V,
                              int64_t row_stride, float target_temperature,
                              const int32_t* q_idx, const float* q_logit, const int32_t* q_count, int32_t k_cap,
                              const int32_t* draft_tokens, const float* u_accept, const float* u_resample,
                              int32_t* out_accept_len, int32_t* out_tokens, float* out_ratio, float* out_beta,
                              int32_t* status, void* ws, size_t ws_bytes, void* stream, int32_t first_stage);

/* tslt_verify for callers that cannot allocate or bring a workspace: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments as tslt_verify without `ws` / `ws_bytes`, same
 * kernels, same results; the per-position decisions and status words (8 bytes per draft position) live in an
 * array that is part of the library's device image (TSLT_STATIC_MAX_POSITIONS positions, 2 MiB per GPU, held
 * until the process ends).  The call allocates nothing and calls no allocating routine.
 *   - B * gamma above TSLT_STATIC_MAX_POSITIONS returns TSLT_ERR_UNSUPPORTED (use tslt_verify and a workspace).
 *   - The first call on a device looks up the array's address on that device (hipGetSymbolAddress) and keeps
 *     it; make that first call outside a stream capture.
 *   - Every call on one GPU uses that GPU's one array, and the array keeps what the last call left in it
 *     (each call overwrites every word it reads later, nothing needs clearing).  Two calls that overlap in time
 *     on one GPU -- on different streams, or from different threads -- race: serialise them, or use tslt_verify
 *     with one workspace per call in flight. */
#define TSLT_STATIC_MAX_POSITIONS 262144
int tslt_verify_static(const void* target_logits, tslt_dtype dt, int64_t B, int32_t gamma, int64_t V,
                       int64_t row_stride, float target_temperature,
                       const int32_t* q_idx, const float* q_logit, const int32_t* q_count, int32_t k_cap,
                       const int32_t* draft_tokens, const float* u_accept, const float* u_resample,
                       int32_t* out_accept_len, int32_t* out_tokens, float* out_ratio, float* out_beta,
                       int32_t* status, void* stream);

/* Measurement aid, not part of the method: one read-only streaming launch over `bytes` bytes of `src` with
 * the load shape of the dense passes (n_blocks workgroups of 256 threads, each reading one contiguous chunk
 * with 16-byte nontemporal loads, four in flight per thread).  Timed by the caller, it gives the read
 * bandwidth this chip delivers to a kernel that only reads: the practical ceiling beside the published peak.
 *   src     device, 16-byte aligned;  bytes a positive multiple of n_blocks * 16384
 *   sink    device, one uint32 (written only if the xor-sum of the data equals a fixed constant) */
int tslt_calibrate_read(const void* src, size_t bytes, int32_t n_blocks, uint32_t* sink, void* stream);

/* What truncation to K entries does to the acceptance rate (Section 3.2).  A set is in canonical order, so
 * its first K entries are the Top-K set of the same draft distribution; for every K of k_list and every
 * row, against that row's dense target distribution p:
 *   out_keep[row, j]  sum of q_hat over the first K entries, q_hat the softmax of the received values over
 *                     the WHOLE set (times tslt_truncate's out_mass: rho of Theorem 1, the Top-K probability
 *                     mass of the draft distribution; sigma = 1 - rho)
 *   out_beta[row, j]  sum_x min(q_hat_K(x), p(x)), q_hat_K the first K entries renormalised: the acceptance
 *                     rate under truncation, 1 - TV(q_hat_K, p) by Lemma 1; Theorem 1 bounds its distance
 *                     from the rate under the untruncated q by sigma
 * K below 1 counts as 1, K above the set's size as the whole set.  A row that is unusable (status bits as for
 * tslt_verify), or whose set is empty, gives NaN.
 *   target_logits  [rows, row_stride] device;  q_idx, q_logit [rows, k_cap], q_count [rows] device
 *   k_list         HOST pointer, n_k values (1 <= n_k <= 32), read before the call returns
 *   out_keep, out_beta  [rows, n_k] fp32 device;  status [rows] int32 device, may be NULL
 * No workspace. */
int tslt_truncation_stats(const void* target_logits, tslt_dtype dt, int64_t rows, int64_t V, int64_t row_stride,
                          float target_temperature, const int32_t* q_idx, const float* q_logit, const int32_t* q_count,
                          int32_t k_cap, const int32_t* k_list, int32_t n_k, float* out_keep, float* out_beta,
                          int32_t* status, void* stream);

/* Acceptance rates of multi-candidate verification with k candidates per position (Section 4.3), for Algorithm 5
 * as printed (candidates i.i.d. from q_hat, the same q_hat at every stage).  P^(1) = P and the residual update
 * p^(j+1) = norm(max(0, p^(j) - q_hat)) do not depend on which tokens were drawn, so for every row, against
 * that row's dense target distribution p:
 *   out_beta[row, j]  beta^(j+1) = sum_x min(q_hat(x), p^(j+1)(x)), the rate at which candidate j+1 is accepted
 *                     given that the ones before it were rejected (the lemma of Section 4.3); NaN for the
 *                     stages behind one whose residual is empty (beta = 1: they are never reached)
 *   out_theta[row]    theta = beta^(1) + sum_{i=2..k} beta^(i) prod_{j<i} (1 - beta^(j)): the rate at which one
 *                     of the k candidates is accepted
 * A row that is unusable (status bits as for tslt_verify), or whose set is empty, gives NaN.
 *   target_logits  [rows, row_stride] device;  q_idx, q_logit [rows, k_cap], q_count [rows] device
 *   k              1..TSLT_MAX_BRANCH
 *   out_beta       [rows, k] fp32 device;  out_theta [rows] fp32 device;  status [rows] int32 device, may be NULL
 * No workspace. */
int tslt_multicandidate_stats(const void* target_logits, tslt_dtype dt, int64_t rows, int64_t V, int64_t row_stride,
                              float target_temperature, const int32_t* q_idx, const float* q_logit,
                              const int32_t* q_count, int32_t k_cap, int32_t k, float* out_beta, float* out_theta,
                              int32_t* status, void* stream);

/* Token-tree verification (Algorithm 8 with Algorithm 5 at every non-leaf node) for B trees.
 *
 * Nodes are stored breadth-first (Section 4.1): layer l has W_l = k_1*...*k_l nodes, the i-th node of
 * layer l (0-based) owns nodes i*k_{l+1} .. (i+1)*k_{l+1}-1 of layer l+1.  N_nodes = sum_l W_l,
 * N_int = N_nodes - W_L.
 *
 *   target_logits [B, N_nodes, row_stride] target logits of every node
 *   depth, expansion   L and the HOST array k_1..k_L (1 <= k_l <= TSLT_MAX_BRANCH)
 *   q_idx, q_logit [B, N_int, k_cap], q_count [B, N_int]  truncated draft set of every non-leaf node
 *   cand_tokens   [B, N_nodes-1] int32: entry n-1 is the token of node n (n >= 1); -1 = absent
 *   u_accept      [B, N_nodes-1] fp32 one uniform per candidate node (entry n-1 for node n)
 *   u_resample    [B, N_nodes] fp32 one uniform per node
 *   without_replacement  how the candidates of a node were drawn, which fixes the proposal q^(i) of stage i:
 *                 0: i.i.d. from q_hat (Algorithm 4) -- q^(i) = q_hat at every stage, Algorithm 5 as printed;
 *                 1: one after the other without replacement -- q^(i) = q_hat with the earlier candidates
 *                 removed and the rest renormalised (each stage is single-candidate speculative sampling
 *                 against that proposal, which keeps the output distributed as P; Section 4.2 only cites
 *                 this direction).  Candidate i is accepted iff u < min(1, p^(i)(x_i) / q^(i)(x_i)), else
 *                 p^(i+1) = norm(max(0, p^(i) - q^(i)))
 *   out_node_token, out_node_slot [B, N_nodes] int32: output of every node -- for a non-leaf node the
 *                 accepted candidate and its child number 0..k-1, or, after k rejections, a sample of
 *                 P^(k+1) and -1;
 *                 for a leaf a sample of its target distribution and -1.  Both may be NULL: then only
 *                 the nodes on the verified path are evaluated (depth+1 target rows are read per tree
 *                 instead of N_nodes; same out_seq, as the uniforms are indexed by node).
 *   out_seq       [B, depth+1] int32 verified sequence: walk from the root, append the node's output,
 *                 descend into the accepted child, stop at the first node without one; -1 after
 *   out_len       [B] int32 length of that sequence, 1..depth+1
 *   out_ratio     [B, N_nodes-1] fp32 p^(i)/q^(i) of every candidate that was tested (NaN if an
 *                 earlier sibling was accepted first or its parent was not evaluated, -1 if not in the
 *                 set); may be NULL
 *   out_beta      [B, N_nodes-1] fp32 stage acceptance rate beta^(i) = sum_x min(q^(i)(x), p^(i)(x)) of
 *                 Section 4.3 for every candidate that was tested (NaN otherwise); may be NULL
 *   status        [B] int32 TSLT_ROW_* bits of the nodes that were evaluated (every node, or only those
 *                 on the verified path, see out_node_token); may be NULL
 * Workspace: tslt_workspace_bytes(TSLT_OP_VERIFY_TREE, B, N_nodes, V, k_cap) when node outputs are
 * requested, tslt_workspace_bytes(TSLT_OP_VERIFY_TREE_PATH, ...) (much smaller) when both are NULL.
 */
int tslt_verify_tree(const void* target_logits, tslt_dtype dt, int64_t B, int64_t V, int64_t row_stride,
                     float target_temperature, int32_t depth, const int32_t* expansion,
                     const int32_t* q_idx, const float* q_logit, const int32_t* q_count, int32_t k_cap,
                     const int32_t* cand_tokens, const float* u_accept, const float* u_resample,
                     int32_t without_replacement,
                     int32_t* out_node_token, int32_t* out_node_slot, int32_t* out_seq, int32_t* out_len,
                     float* out_ratio, float* out_beta, int32_t* status, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TSLT_H */
