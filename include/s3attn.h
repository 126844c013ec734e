/* s3attn.h -- C ABI of the MI355X (gfx950) hot path of S3-Attention:
 *
 *   sae_encode_topk : key/query chunk -> Top-k SAE feature ids + activations   (Sec. 3.3)
 *   index_*         : feature ids -> feature -> token-position inverted index   (Sec. 3.4)
 *   coactivate_score: query features + index -> position scores -> Top-B spans  (Sec. 3.5, App. D.2, App. E)
 *
 * Conventions
 *   - Every array pointer is a DEVICE pointer owned by the caller unless marked "host".
 *   - Every call is asynchronous on `stream` (a hipStream_t passed as void*; NULL = the null
 *     stream); outputs are valid once the stream has reached the call.  No call synchronises
 *     the host with the device and no call after s3_index_create / workspace set-up allocates.
 *   - Inputs are never modified.  Outputs must not alias inputs.
 *   - Return value: S3_OK (0) or a negative S3_E* code; s3_last_error() gives the message.
 *     Arguments are validated on the host before anything is launched; on error nothing has
 *     been launched.
 *   - One GPU: the device that is current when s3_index_create / a call is made.
 */
#ifndef S3ATTN_H
#define S3ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    S3_OK = 0,
    S3_EINVAL = -1,    /* null pointer, shape or parameter outside the supported range */
    S3_ESTATE = -2,    /* call not allowed in the index's current state */
    S3_ECAPACITY = -3, /* more tokens than the index was created for, or workspace too small */
    S3_EHIP = -4       /* a HIP runtime call failed */
};

enum { S3_BF16 = 0, S3_FP32 = 1 };

#define S3_MAX_K 128         /* largest supported Top-k */
#define S3_MAX_FEAT 65536    /* largest supported SAE width */

/* Message of the last error on this host thread (valid until the next failing call). */
const char* s3_last_error(void);

/* ------------------------------------------------------------------------------------------
 * Sec. 3.3, encoder equation z = ReLU(W_enc (x - b_dec) + b_enc) followed by the Top-K
 * equation, for a batch of independent (layer, head) SAEs.  The same call encodes key chunks
 * (Sec. 3.4, per-chunk feature extraction) and query vectors (Sec. 3.5 "Query Decoding"); the
 * caller passes the same w_enc/b_enc for both (shared codebook, Alg. 1 Phase 0).
 *
 *   x      [n_heads, T, d_head]       bf16 or fp32 (dtype), row-major, 16-byte aligned
 *   w_enc  [n_heads, n_feat, d_head]  same dtype, feature-major (one feature's vector contiguous)
 *   b_enc  [n_heads, n_feat]          fp32; b_dec must be folded in by the caller:
 *                                     b_enc_eff = b_enc - W_enc b_dec
 *   ids    [n_heads, T, k] int32, vals [n_heads, T, k] fp32 (outputs)
 *
 * Per row the k features with the largest pre-activation z are selected (ties: lower id), so a
 * row always has exactly k distinct ids; vals = max(z, 0).  Within a row the order is
 * (z descending, id ascending).  z is accumulated in fp32 and never written to memory.
 * Inputs are assumed finite.
 * Limits: d_head in {64, 128, 256}; 1 <= k <= min(n_feat, S3_MAX_K); the candidate lists must
 * fit the 160 KB of LDS beside two 32-feature tiles of W_enc, which leaves k <= 128 for bf16 with
 * d_head <= 128 and fp32 with d_head 64, k <= 121 for bf16 with d_head 256 and fp32 with d_head
 * 128, k <= 78 for fp32 with d_head 256 (k = 128 is the sparsity the paper trains its SAEs with,
 * App. B.3); n_feat <= S3_MAX_FEAT; T >= 0 (T == 0 is a no-op); n_heads >= 1.  Otherwise S3_EINVAL.
 * bf16 with d_head 128, k <= 64 and n_feat a multiple of 128 takes the fast kernel.
 * No workspace is needed (so there is no workspace query for this call).
 */
int s3_sae_encode_topk(const void* x, int dtype, int T, int d_head, const void* w_enc,
                       const float* b_enc, int n_feat, int k, int n_heads, int32_t* ids,
                       float* vals, void* stream);

/* The same operation for the chunks of one stream (Alg. 1, Phase 1: the prefill walks the context
 * chunk by chunk with the same encoder), with a selection threshold carried from chunk to chunk.
 * Results are identical to s3_sae_encode_topk for ANY contents of tau_hint: the carried values
 * only set where the exact Top-K selection (Sec. 3.3) of a token starts; a token whose start was
 * too high (fewer than k pre-activations above it) is selected again from scratch inside the same
 * call.  The k-th largest pre-activation of a token scales with |x_t|, so the smallest
 * tau_t / |x_t| (and the smallest tau_t) of one chunk are good starts for the next one.
 *
 *   tau_hint [n_heads][2] fp32, device, read and overwritten: the smallest tau_t / |x_t| and the
 *            smallest tau_t over the tokens of the previous call; only the one that was the tighter
 *            predictor on that call is kept, the other is -INFINITY.  Fill with -INFINITY before
 *            the first chunk of a stream: a head without a bound has its first 256 tokens (128 for
 *            k > 32) selected from scratch first, and their thresholds start the rest of the chunk.
 *   ws       s3_sae_encode_topk_stream_workspace(n_heads, T) bytes, 256-byte aligned, device;
 *            scratch, contents meaningless between calls.
 * Shapes the threshold-carrying kernel is not built for (anything but bf16, d_head 128,
 * n_feat % 128 == 0) run exactly as s3_sae_encode_topk and leave tau_hint untouched.
 * Errors as s3_sae_encode_topk; S3_ECAPACITY if ws_bytes is too small. */
size_t s3_sae_encode_topk_stream_workspace(int n_heads, int T);
int s3_sae_encode_topk_stream(const void* x, int dtype, int T, int d_head, const void* w_enc,
                              const float* b_enc, int n_feat, int k, int n_heads, int32_t* ids,
                              float* vals, float* tau_hint, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Sec. 3.4, inverted semantic index: for all f in F_t, I[f] <- I[f] U {t}, held on the GPU in
 * the contiguous form the paper recommends (Sec. 3.4 "CPU Index Size"): per head a CSR with
 * offsets[n_feat + 1] and positions[P], lists in ascending feature id, positions inside a list
 * in the order the tokens were appended.  P = tokens * k per head (same section).
 *
 * s3_index_create allocates everything for n_heads independent indexes of up to max_tokens
 * tokens each (host call; the handle is library-owned; destroy with s3_index_destroy).
 * Limits: n_feat <= S3_MAX_FEAT, k <= S3_MAX_K, max_tokens * k < 2^31, max_tokens <= 2^24.
 * Beside the CSR the index holds the intermediate of the build (4 bytes per posting) and, for up
 * to 64 blocks of 16384 tokens, a table of where every block starts in every list
 * (4 * n_feat * (blocks - 1) bytes per head), which scoring reads instead of searching the lists.
 */
typedef struct s3_index s3_index;
int s3_index_create(int n_heads, int n_feat, int k, int64_t max_tokens, s3_index** out);
void s3_index_destroy(s3_index* idx);

/* Append one chunk (Alg. 1, Phase 1 inner loop "Update I with feats").
 *   ids [n_heads, T, k] int32 in [0, n_feat); positions [T] int32 absolute positions shared by
 *   all heads, or NULL for base_pos + row.  Chunks may have any length T >= 0.
 * S3_ESTATE after finalize; S3_ECAPACITY if the total would exceed max_tokens.
 * Ids outside [0, n_feat) are undefined behaviour (they are not checked on the device). */
int s3_index_append(s3_index* idx, const int32_t* ids, int T, const int32_t* positions,
                    int32_t base_pos, void* stream);

/* Turn everything appended so far into the CSR.  May be called once; appending afterwards is
 * S3_ESTATE.  The result does not depend on how the stream was cut into chunks. */
int s3_index_finalize(s3_index* idx, void* stream);

/* Borrowed device views of one head's CSR (valid until destroy): offsets [n_feat + 1] int32,
 * positions [*n_postings] int32.  Host call; S3_ESTATE before finalize. */
int s3_index_csr(const s3_index* idx, int head, const int32_t** offsets,
                 const int32_t** positions, int64_t* n_postings);

/* Copy one head's CSR into caller-owned device arrays offsets_out [n_feat + 1] and
 * positions_out [n_postings] (either may be NULL to skip it); asynchronous on `stream`. */
int s3_index_export(const s3_index* idx, int head, int32_t* offsets_out, int32_t* positions_out,
                    void* stream);

/* Forget everything appended (tokens = 0, not finalized) and keep the allocations, so that the
 * next context can be indexed without allocating (Alg. 1 "Initialize inverted index").  Work
 * already queued on a stream keeps reading the old contents: order the reset after it. */
int s3_index_reset(s3_index* idx);

/* Tokens appended so far (host value). */
int64_t s3_index_tokens(const s3_index* idx);

/* One-shot form for a single index with caller-owned outputs: offsets [n_feat + 1],
 * out_positions [T * k]; positions [T] or NULL (= row).  ws must hold
 * s3_index_build_workspace(T, k, n_feat) bytes (256-byte aligned). */
size_t s3_index_build_workspace(int T, int k, int n_feat);
int s3_index_build(const int32_t* ids, const int32_t* positions, int T, int k, int n_feat,
                   int32_t* offsets, int32_t* out_positions, void* ws, size_t ws_bytes,
                   void* stream);

/* s3_index_build for callers that cannot allocate and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * errors as s3_index_build without ws / ws_bytes: the workspace is a buffer of
 * S3_STATIC_SCRATCH_BYTES that is built into the library (static device memory, one copy per GPU,
 * held until the process ends).  The call allocates nothing, frees nothing and records no memset.
 * S3_ECAPACITY when s3_index_build_workspace(T, k, n_feat) exceeds S3_STATIC_SCRATCH_BYTES
 * (about T * k <= 4 M postings).  All calls on one GPU share the buffer: calls that overlap on
 * that GPU (different streams, or threads on different streams) race; serialise them. */
#define S3_STATIC_SCRATCH_BYTES (16u << 20)
int s3_index_build_static(const int32_t* ids, const int32_t* positions, int T, int k, int n_feat,
                          int32_t* offsets, int32_t* out_positions, void* stream);

/* ------------------------------------------------------------------------------------------
 * Sec. 3.5 scoring equation with App. D.2's weights:
 *     S[t] = sum over heads h, over query pairs (q, j) with f = qids[h, q, j]:
 *            qvals[h, q, j] * IDF_h(f) * 1[t in I_h[f]],   IDF(f) = 1 / (ln(1 + freq(f)) + 1),
 * freq(f) = length of I_h[f]; a feature with freq > max_freq is skipped when max_freq > 0
 * (App. E's hard threshold; the paper's value is 5000).  Then the smoothing and peak
 * selection of Sec. 3.5 "Adaptive Granularity", read as a box kernel and fixed-length spans:
 *     W[s] = sum_{t = s}^{s + span_len - 1} S[t],  s in [0, L - span_len]   (span_len clamped to L)
 *     repeat top_b times: best remaining window (ties: smallest s); if nms, drop every window
 *     overlapping it (|s' - s| < span_len); stop early if none is left.
 * L = n_positions: positions in the index must lie in [0, n_positions).
 *
 *   qids/qvals [n_heads, nq, k]  (the output layout of s3_sae_encode_topk on the query vectors;
 *                                 the caller has already mapped each Q head to its KV head)
 *   scores_out [n_positions] fp32 or NULL; span_start [top_b] int32; span_score [top_b] fp32;
 *   n_found [1] int32.  Entries past n_found are set to -1 / 0.
 *   ws: s3_coactivate_score_workspace(idx, n_positions) bytes, 256-byte aligned.
 * Sums are accumulated in 64-bit fixed point, so the result is independent of execution order
 * (bit-identical from run to run) and W[s] is exactly the sum of its members before the final
 * rounding to fp32.
 * Limits: 1 <= span_len; 1 <= top_b <= 1024; nq >= 0; nq * k <= 2^20; qvals finite and >= 0;
 * ceil(log2(n_heads * k)) + ceil(log2(min(span_len, n_positions))) <= 36, so that a window's
 * fixed-point sum cannot overflow 64 bits while weights keep at least 22 significant bits
 * (S3_EINVAL otherwise).
 */
size_t s3_coactivate_score_workspace(const s3_index* idx, int64_t n_positions);
int s3_coactivate_score(const s3_index* idx, const int32_t* qids, const float* qvals, int nq,
                        int64_t n_positions, int span_len, int top_b, int32_t max_freq, int nms,
                        float* scores_out, int32_t* span_start, float* span_score,
                        int32_t* n_found, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Sec. 3.4 "CPU Index Size": the compact form of a finalized index -- contiguous integer arrays
 * with delta encoding and optional stop-feature pruning -- and Sec. 3.5 scoring straight from it.
 * Positions are cut into blocks of 16384; a posting is stored as its 16-bit offset from the start
 * of its block, and the postings are ordered block by block, inside a block list by list
 * (ascending feature id), inside a list in list order:
 *     cstart [n_blocks * n_feat + 1] int32: entry b * n_feat + f is where the segment of (block b,
 *            feature f) starts in delta; the next entry is its end
 *     delta  [kept postings] uint16;  cfreq [n_feat] int32: length of each list (0: dropped)
 * A list with more than prune_freq postings is dropped whole when prune_freq > 0 (a stop feature;
 * scoring the compact index then equals scoring the plain one with max_freq = prune_freq).
 * 2 bytes per posting instead of 4, and everything a scoring workgroup reads for its block of
 * positions is one contiguous run of memory.
 *
 * s3_index_compact builds it on `stream` into `buf` (device, caller-owned, 256-byte aligned, at
 * least s3_index_compact_bytes(idx) bytes -- sized for no pruning); *out is a small host handle
 * (free with s3_cindex_destroy; the arrays live in buf and stay valid as long as buf does, also
 * after the plain index is destroyed).  Needs an index fed implicit, increasing positions that lie
 * below 64 * 16384 (S3_ESTATE otherwise, and before finalize).
 * s3_cindex_export copies one head's arrays (any may be NULL): cstart_out [n_blocks * n_feat + 1],
 * delta_out [max_postings] (only the first cstart[last] entries are meaningful), cfreq_out [n_feat];
 * s3_cindex_info gives n_blocks and max_postings (= tokens * k).
 * s3_coactivate_score_compact: as s3_coactivate_score, reading the compact index. */
typedef struct s3_cindex s3_cindex;
size_t s3_index_compact_bytes(const s3_index* idx);
int s3_index_compact(const s3_index* idx, int32_t prune_freq, void* buf, size_t buf_bytes, s3_cindex** out,
                     void* stream);
void s3_cindex_destroy(s3_cindex* cidx);
int s3_cindex_info(const s3_cindex* cidx, int* n_blocks, int64_t* max_postings);
int s3_cindex_export(const s3_cindex* cidx, int head, int32_t* cstart_out, uint16_t* delta_out,
                     int32_t* cfreq_out, void* stream);
size_t s3_coactivate_score_compact_workspace(const s3_cindex* cidx, int64_t n_positions);
int s3_coactivate_score_compact(const s3_cindex* cidx, const int32_t* qids, const float* qvals, int nq,
                                int64_t n_positions, int span_len, int top_b, int32_t max_freq, int nms,
                                float* scores_out, int32_t* span_start, float* span_score,
                                int32_t* n_found, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * Sec. 3.5 "Adaptive Granularity" and Alg. 1 Phase 2 (S' <- Conv1D(S); Idx <- NMS_Select(S', N)) with
 * a smoothing kernel of the caller's choice and variable-length spans.  The paper fixes the sizes
 * (App. B.3: kernel 48, 8 for QA; N = 40 centres) and leaves the weights, the suppression rule and
 * the span rule open; the readings taken:
 *     D[t] = sum_{j < K} kernel[j] * S[t + j - floor(K / 2)]        (zeros outside [0, L))
 *     repeat n_centers times: c = the remaining position of largest D (ties: smallest t); stop if
 *         D[c] <= 0; every position within nms_radius of c is suppressed
 *     span of c = [c - a, c + b], a and b the largest values <= max_half_len (and inside the context)
 *         such that D >= rel_threshold * D[c] at every position of the span
 * D is accumulated in fp64 from the fp32 inputs and rounded to fp32 once; all comparisons use
 * those fp32 values (threshold product in fp64), so the result does not depend on execution order.
 *
 *   scores [n_positions] fp32 (the scores_out of s3_coactivate_score); kernel [K] fp32, device;
 *   density_out [n_positions] fp32 or NULL; center / span_lo / span_hi [n_centers] int32,
 *   center_density [n_centers] fp32, n_found [1] int32; entries past n_found are -1 / 0.
 *   ws: s3_select_spans_workspace(n_positions) bytes, 256-byte aligned.
 * Limits: 1 <= K <= 4096; 1 <= n_centers <= 4096; nms_radius, max_half_len >= 0;
 * 0 <= rel_threshold <= 1.
 *
 * s3_smoothing_kernel fills a HOST array with the weights of a box (1/K each), triangular
 * (proportional to min(j + 1, K - j)) or Gaussian (centre (K - 1) / 2, sigma K / 6) kernel, each
 * normalised to sum 1; the caller copies them to the device. */
enum { S3_KERNEL_BOX = 0, S3_KERNEL_TRIANGULAR = 1, S3_KERNEL_GAUSSIAN = 2 };
int s3_smoothing_kernel(int kind, int K, float* weights);
size_t s3_select_spans_workspace(int64_t n_positions);
int s3_select_spans(const float* scores, int64_t n_positions, const float* kernel, int K, int n_centers,
                    int nms_radius, float rel_threshold, int max_half_len, float* density_out,
                    int32_t* center, float* center_density, int32_t* span_lo, int32_t* span_hi,
                    int32_t* n_found, void* ws, size_t ws_bytes, void* stream);

/* Sec. 3.6 / Alg. 1 Phase 3, Idx_final = Idx_S3 U Idx_lexical U LeadTail, as a set of positions:
 * the union of the spans [span_lo[i], span_hi[i]] (inclusive; i < min(*n_spans, max_spans), n_spans a
 * device pointer or NULL for max_spans), of the caller's index list `extra` (the lexical retriever's
 * output; entries outside [0, n_positions) are ignored, repeats are fine) and of the first `lead`
 * and last `tail` positions.
 *   mask [n_positions] uint8 (0 / 1); idx_out [n_positions] int32: the selected positions in
 *   ascending order; n_out [1] int32 their number.  ws: s3_fuse_indices_workspace(n_positions) bytes.
 * Limits: max_spans <= 65535; n_extra < 2^31. */
size_t s3_fuse_indices_workspace(int64_t n_positions);
int s3_fuse_indices(int64_t n_positions, const int32_t* span_lo, const int32_t* span_hi,
                    const int32_t* n_spans, int max_spans, const int32_t* extra, int64_t n_extra,
                    int lead, int tail, unsigned char* mask, int32_t* idx_out, int32_t* n_out, void* ws,
                    size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------
 * One training step of the Top-K SAE (Sec. 3.3: encoder, Top-K and decoder equations; App. B.3:
 * Adam, learning rate 1e-3, batches of 4096 tokens, expansion 128, k = 128).  The paper trains the
 * SAE by reconstruction and names no other term; the objective taken is the mean squared error
 *     L = sum_t |xhat_t - x_t|^2 / (B d),   u_t = x_t - b_dec,  (ids, zhat) = TopK(ReLU(W_enc u_t + b_enc), k),
 *     xhat_t = sum_i zhat_{t,i} W_dec[ids_{t,i}] + b_dec.
 * The encoder runs as in the retrieval path: on u and W_enc rounded to bf16 (round to nearest
 * even), fp32 accumulation, exact Top-K (ties: lower id).  The backward pass holds the selection
 * fixed, passes gradient only to selected entries with zhat > 0, and treats the rounding as the
 * identity (gradients use the rounded operands).  With g_t = 2 (xhat_t - x_t) / (B d) and
 * dz_{t,i} = (g_t . W_dec[id]) [zhat_{t,i} > 0]:
 *     dW_dec[f] = sum zhat g_t,  dW_enc[f] = sum dz u_t,  db_enc[f] = sum dz   (over the (t, i) with id = f),
 *     db_dec = sum_t (g_t - sum_i dz_{t,i} W_enc[id_{t,i}]).
 * Then Adam with bias correction on all parameters, step >= 1 (the caller counts the steps):
 *     m <- beta1 m + (1 - beta1) grad,  v <- beta2 v + (1 - beta2) grad^2,
 *     p <- p - lr (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps).
 * Every sum is taken in a fixed order (per feature in (token, slot) order through an inverted index
 * of the batch; no atomics): the step is bit-reproducible.
 *
 *   x [B, d_head] fp32, device, read only.
 *   w_enc, w_dec [n_feat, d_head], b_enc [n_feat], b_dec [d_head]: fp32, device, updated in place.
 *   adam_m, adam_v [P] fp32, device, P = 2 n_feat d_head + n_feat + d_head, in the order
 *            W_enc | b_enc | W_dec | b_dec; zero before the first step; updated in place.
 *   loss_out [1] fp32: L before the update.  ids_out [B, k] int32 or NULL: the selection.
 *   grads_out [P] fp32 or NULL: the gradients, packed like adam_m.
 *   ws: s3_sae_train_workspace(B, d_head, n_feat, k) bytes (0 for an unsupported shape), 256-byte
 *       aligned.
 * Limits: d_head = 128; n_feat a multiple of 128, <= 65536; 1 <= k <= min(128, n_feat);
 * B * k <= 2^24; lr >= 0; 0 <= beta1, beta2 < 1; eps > 0.  S3_EINVAL / S3_ECAPACITY as elsewhere. */
size_t s3_sae_train_workspace(int B, int d_head, int n_feat, int k);
int s3_sae_train_step(const float* x, int B, int d_head, int n_feat, int k, float* w_enc,
                      float* b_enc, float* w_dec, float* b_dec, float* adam_m, float* adam_v,
                      float lr, float beta1, float beta2, float eps, int step, float* loss_out,
                      int32_t* ids_out, float* grads_out, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* S3ATTN_H */
