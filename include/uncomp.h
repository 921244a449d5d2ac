/*
 * libuncomp -- UNComp's prefill-time KV-cache compression pass for AMD MI355X (gfx950).
 *
 * Four hot calls, in the order a caller enqueues them on one HIP stream:
 *
 *   uncomp_head_entropy    truncated matrix entropy of every token matrix
 *   uncomp_assign_budgets  entropies -> per-head token budgets and per-layer stages
 *   uncomp_window_score    observation-window attention score of every prefix token
 *   uncomp_select_gather   per-head top-k of the scores, compaction of K and V
 *
 * and, for the tokens generated afterwards:
 *
 *   uncomp_decode_init     cumulative scores of the compacted cache from the prefill score
 *   uncomp_decode_step     one token: attention over the cache, score update, eviction
 *
 * and, between the layers of the prefill where the token count drops:
 *
 *   uncomp_hidden_evict    last-token attention -> top-N rows of the hidden states
 *
 * and, before any inference, over a set of sampled prompts:
 *
 *   uncomp_prepare_*       running mean of erank and label votes per head -> group labels
 *   uncomp_budgets_from_labels   per-head budgets from stored labels
 *
 * Conventions that hold for every call:
 *   - Pointers named X, K, V, Qwin, *_out, entropy, score, budget are DEVICE pointers
 *     owned by the caller; the library never allocates, frees or keeps them.  The
 *     context, stride arrays and strings are HOST memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on it and never synchronise; outputs are valid once the stream has
 *     reached the end of the call's work.  What they enqueue is kernel launches (and, in
 *     uncomp_matrix_entropy, device-to-device copies): no allocation, no memset, no host
 *     wait, so with the profiler and the overlap mode off a sequence of calls can be
 *     captured into a HIP graph and replayed on new contents of the same buffers.
 *   - All temporary device memory comes from the context's workspace, allocated once in
 *     uncomp_create.  A call that needs more returns UNCOMP_ERR_WORKSPACE and launches
 *     nothing.  One context serves one stream at a time (calls on it share the workspace).
 *   - Arguments are validated on the host before anything is launched; a failing call
 *     returns a negative status, launches nothing and leaves outputs untouched.
 *     uncomp_last_error gives a one-line reason.
 *   - Supported: D == 128, and D == 64 in the four hot calls (64-wide heads run on the plain
 *     arithmetic units, not the matrix cores: correct, several times slower; every other call
 *     takes D == 128 only); dtype bf16 or fp32; 1 <= k_trunc; pool odd, 1 <= pool <= 15;
 *     0 < w < N; M >= 1 dividing H.  Anything else is UNCOMP_ERR_UNSUPPORTED.
 */
#ifndef UNCOMP_H
#define UNCOMP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct uncomp_ctx uncomp_ctx;

typedef enum {
    UNCOMP_OK = 0,
    UNCOMP_ERR_INVALID_ARG = -1,  /* NULL pointer, non-positive size, inconsistent sizes */
    UNCOMP_ERR_UNSUPPORTED = -2,  /* a value outside the supported set listed above      */
    UNCOMP_ERR_WORKSPACE = -3,    /* the context's workspace is too small for this call  */
    UNCOMP_ERR_HIP = -4           /* a HIP runtime call failed (text in uncomp_last_error) */
} uncomp_status;

typedef enum { UNCOMP_BF16 = 0, UNCOMP_F32 = 1 } uncomp_dtype;

enum {
    /* Sec. 3.1 Eq. 1: subtract the mean token before forming the covariance.  Without
     * it the uncentred form X^T X/(N-1) from the proof of Lemma 3 is used.             */
    UNCOMP_CENTER = 1u,
    /* Sec. 3.2 Eq. 5 summed over the top-k eigenvalues after rescaling THEM to sum to
     * one (so an isotropic matrix reaches the bound H_k = log k of Lemma 4).  Without
     * it the eigenvalues keep their share of the full unit trace, Eq. 5 as printed.    */
    UNCOMP_TRUNC_RENORM = 2u,
    /* Layer partition: count a boundary where erank rises by more than eps (the test in
     * Alg. 2's prefill loop) instead of where it falls by more than eps (Eq. 8-9).     */
    UNCOMP_LAYER_DELTA_INCREASE = 4u
};
#define UNCOMP_DEFAULT_FLAGS (UNCOMP_CENTER | UNCOMP_TRUNC_RENORM)

/* Creates a context on HIP device `device` with `workspace_bytes` of device scratch
 * (0 = a default of 64 MiB).  Sets *ctx_out; the caller destroys it with uncomp_destroy. */
uncomp_status uncomp_create(uncomp_ctx** ctx_out, int device, size_t workspace_bytes);
uncomp_status uncomp_destroy(uncomp_ctx* ctx);

/* Workspace (bytes) that one round of the four calls needs for the given problem:
 * n_mat token matrices of N rows in uncomp_head_entropy, and B*H KV heads with G query
 * heads each in uncomp_window_score / uncomp_select_gather.  Pass 0 for a call that will
 * not be made with this context. */
size_t uncomp_workspace_bytes(int n_mat, int N, int D, int B, int H, int G, int w);

/* Host string describing the last failing call on this context (never NULL, owned by
 * the context, valid until the next call on it).  With ctx == NULL: the calling thread's last
 * failing context-free call (uncomp_head_entropy_noalloc), "null context" if there was none. */
const char* uncomp_last_error(const uncomp_ctx* ctx);

/* Per-kernel timing for benchmarks (not a paper operation).  uncomp_profile(ctx, 1) makes
 * every later hot call bracket each of its kernel launches with two HIP events on the
 * caller's stream and clears earlier records; uncomp_profile(ctx, 0) stops it.  After the
 * caller has synchronised the stream, uncomp_profile_read copies up to max_records
 * (kernel name, milliseconds) pairs in launch order into the HOST arrays names / ms (either
 * may be NULL), clears the records and returns their count (negative = status).  At most
 * 1024 launches are kept between reads; later ones go untimed.  The events are created by
 * uncomp_profile(ctx, 1) itself, so a timed region creates nothing.  Names are static strings. */
uncomp_status uncomp_profile(uncomp_ctx* ctx, int on);
int uncomp_profile_read(uncomp_ctx* ctx, int max_records, const char** names, float* ms);

/* What the device sustains, measured on the spot (not a paper operation; the one call here that
 * WAITS for its kernels): read_GBps, the rate of a plain streaming read of `bytes` (>= 64 MiB) of
 * the caller's DEVICE memory at buf (16-byte aligned, contents irrelevant, not written);
 * mfma_TFLOPs_live / mfma_TFLOPs_zero, the rate of a loop of v_mfma_f32_32x32x16_bf16 at two waves per
 * SIMD on pseudo-random operands and on zeros (the chip lowers its clock under the switching
 * activity of live data, so kernels with real operands are bound by the first figure).  The three
 * results are HOST doubles.  Takes a few tens of milliseconds. */
uncomp_status uncomp_measure_peaks(uncomp_ctx* ctx, const void* buf, size_t bytes, double* read_GBps,
                                   double* mfma_TFLOPs_live, double* mfma_TFLOPs_zero, void* stream);

/* Overlap mode (default off).  With on != 0, uncomp_head_entropy runs only its Gram kernel on
 * the caller's stream and moves the eigen stage to a stream owned by the context (ordered
 * after the Gram kernel by an event); a following uncomp_assign_budgets goes to that stream
 * too, so both run beside the uncomp_window_score kernels of the caller's stream.  The next
 * uncomp_select_gather, or an explicit uncomp_join, makes the caller's stream wait for them.
 * Until then entropy_out / eig_out / the budget outputs are NOT ordered with the caller's
 * stream.  The workspace must hold the entropy and scoring regions side by side, which is
 * what uncomp_workspace_bytes reports.  Every other call that touches the workspace regions
 * of the side-stream work (a second uncomp_head_entropy, uncomp_decode_step,
 * uncomp_hidden_evict, uncomp_matrix_entropy, uncomp_prepare_accumulate) joins first by
 * itself, so calls may follow one another in any order. */
uncomp_status uncomp_set_overlap(uncomp_ctx* ctx, int on);
uncomp_status uncomp_join(uncomp_ctx* ctx, void* stream);

/* Kernel selection for testing: plain_alu != 0 makes the bf16 calls use the plain-ALU
 * kernels (the ones fp32 inputs always use) instead of the MFMA kernels, the eigen stage the
 * fp32 Jacobi iteration instead of the fp64 tridiagonalisation, uncomp_decode_step its
 * one-kernel path, and uncomp_select_gather the one-workgroup-per-head selection also for a
 * few long rows (which it otherwise splits over many workgroups).  Default 0. */
uncomp_status uncomp_set_kernel_path(uncomp_ctx* ctx, int plain_alu);

/*
 * Truncated matrix entropy (Sec. 3.1 Eq. 1 and Lemma 2; Sec. 3.2 Eq. 5-6; unit trace as
 * in the proof of Lemma 4).
 *
 * X holds n_mat token matrices; matrix m starts at element m*mat_stride, its token t at
 * element t*ldx further on, and the D features of a token are contiguous.  For each
 * matrix: covariance over the N tokens (centred unless UNCOMP_CENTER is cleared), scaled
 * to unit trace; eigenvalues sigma_1 >= ... >= sigma_D (negatives from rounding clamped to
 * zero); entropy_out[m] = - sum_{i <= min(k_trunc, D)} s_i ln s_i with s_i per
 * UNCOMP_TRUNC_RENORM; 0 ln 0 = 0; a zero covariance (e.g. N == 1) gives 0.
 * erank_k = exp(entropy).  eig_out, if not NULL, receives the D unit-trace eigenvalues of
 * each matrix in descending order ([n_mat][D] floats).
 * Requires ldx >= D, ldx and mat_stride multiples of 8 elements, X 16-byte aligned.
 */
uncomp_status uncomp_head_entropy(uncomp_ctx* ctx, const void* X, uncomp_dtype dtype,
                                  int n_mat, int N, int D, int64_t mat_stride, int64_t ldx,
                                  int k_trunc, unsigned flags,
                                  float* entropy_out, float* eig_out, void* stream);

/*
 * Truncated matrix entropy of wide token matrices (same definition as uncomp_head_entropy, for
 * D = 256 ... 16384 in multiples of 128: e.g. the hidden states H_m of Sec. 3.3.2, whose erank
 * the paper's layer analysis plots).  The D x D covariance is never formed: the k_trunc <= 128
 * largest eigenvalues are taken as the Ritz values of a 128-dimensional subspace after n_iter
 * rounds of block power iteration (each round reads X twice).  Their error falls like
 * (sigma_129 / sigma_k)^(2 n_iter): a few rounds when the spectrum drops before the 129th
 * eigenvalue, many when it is flat there.  For bf16 inputs the rounds multiply by factors rounded
 * to bf16 (the iterated block keeps 17 bits only in the last round and in the final projection):
 * the Ritz values change by the square of what a round gets wrong, below 2e-6 relative on the
 * tested spectra.
 * entropy_out [n_mat]; eig_out, if not NULL, receives
 * the 128 Ritz values of each matrix as shares of the full trace, descending ([n_mat][128]).
 * X as in uncomp_head_entropy (ldx >= D, strides multiples of 8 elements, 16-byte aligned).
 * Matrices are processed one after the other.  Workspace: uncomp_matrix_workspace_bytes(N, D).
 */
size_t uncomp_matrix_workspace_bytes(int N, int D);
uncomp_status uncomp_matrix_entropy(uncomp_ctx* ctx, const void* X, uncomp_dtype dtype,
                                    int n_mat, int N, int D, int64_t mat_stride, int64_t ldx,
                                    int k_trunc, unsigned flags, int n_iter,
                                    float* entropy_out, float* eig_out, void* stream);

/*
 * uncomp_head_entropy for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  It takes no context and calls no hipMalloc,
 * hipFree or other allocating routine: the partial second-moment sums that uncomp_head_entropy keeps
 * in the context's workspace live in a fixed array of 32.3 MiB inside the library's code object (each
 * GPU the library runs on holds its copy from the loading of the library to the end of the process).
 * Arguments, results and the kernels are those of uncomp_head_entropy (eigen stage: the fp64
 * tridiagonalisation; no profiling, no overlap mode); the call works on the CURRENT device.
 * Limits: the partial sums of one call must fit the array: at most 512 matrices per call (beyond:
 * UNCOMP_ERR_WORKSPACE, nothing launched); between 1 and 512 matrices the token axis is split into
 * fewer, longer chunks than uncomp_head_entropy would use, which changes the order of the fp32
 * partial sums but not what is computed.  All calls on one GPU share the array: calls that overlap
 * in time on one GPU (different streams, different threads) race; calls on one stream are ordered.
 * The first call on a device looks up the array's address and raises one kernel's LDS limit
 * (no allocation either, but not to be done under stream capture: make one call beforehand).
 * uncomp_last_error(NULL) gives the reason of the calling thread's last failing call.
 */
uncomp_status uncomp_head_entropy_noalloc(const void* X, uncomp_dtype dtype, int n_mat, int N, int D,
                                          int64_t mat_stride, int64_t ldx, int k_trunc, unsigned flags,
                                          float* entropy_out, float* eig_out, void* stream);

/*
 * Budgets from entropies (Sec. 3.3.3 "Design", Eq. 11; Sec. 3.3.2 Eq. 8-10).
 *
 * entropy is [n_layer][n_batch][H] floats.  Per (layer, batch): heads are ranked by entropy,
 * largest first, equal values by lower head index; rank r falls in group g = r / (H/M);
 * head_budget = clamp(n_max - g*step, min(w, N), N)  (n_max is N_{i,1}, step is Delta n_g).
 * Per layer: e_l = mean over batch and heads of exp(entropy), evaluated in double
 * precision; stage counter c_0 = 0, c_{l} = c_{l-1} + [e_{l-1} - e_l > eps] (sign flipped
 * under UNCOMP_LAYER_DELTA_INCREASE); layer_group[l] = c_l;
 * layer_tokens[l] = max(N - c_l*delta_n, w).
 * Outputs (device, int32): head_budget and head_group [n_layer][n_batch][H];
 * layer_group and layer_tokens [n_layer] (either pair may be NULL to skip it).
 * Limits: H <= 1024, n_layer <= 4096.
 */
uncomp_status uncomp_assign_budgets(uncomp_ctx* ctx, const float* entropy,
                                    int n_layer, int n_batch, int H, int M,
                                    int n_max, int step, int N, int w,
                                    float eps, int delta_n, unsigned flags,
                                    int32_t* head_budget, int32_t* head_group,
                                    int32_t* layer_group, int32_t* layer_tokens, void* stream);

/*
 * Observation-window score (Sec. 3.3.3 "Dynamic KV Cache Eviction": the attention the last
 * w tokens pay to each earlier token, summed; followed by a 1-D max-pool over token
 * positions and a sum over the G query heads that share a KV head).
 *
 * Qwin [B][H*G][w][D] dense: the queries at positions P..N-1, P = N - w; query head q reads
 * KV head q / G.  K: head (b,h) starts at element b*k_strides[0] + h*k_strides[1], token t at
 * t*k_strides[2] further on, features contiguous.  For window row i (position P+i):
 * p_ij = softmax over the causal range j <= P+i of q_i . k_j / sqrt(D), in fp32;
 * vote_q[j] = sum_i p_ij for j < P; pooled_q[j] = max of vote_q over |j' - j| <= pool/2,
 * 0 <= j' < P; score_out[b][h][j] = sum over the G query heads of pooled_q[j], j in [0, P).
 * score_out is dense [B][H][P] floats.  Strides are multiples of 8 elements, K and Qwin
 * 16-byte aligned; G*w <= 512.
 *
 * lse_opt (DEVICE, [B][H*G][w] floats, or NULL): the natural-log normaliser of every window
 * row, lse[b][q][i] = ln sum over j <= P+i of exp(q_i . k_j / sqrt(D)), as the attention
 * kernel of the model computes it for these rows anyway.  When given, the library skips
 * its own pass over the keys for the normalisers (half of the key traffic of this call)
 * and uses these; the caller answers for their accuracy (a relative error e in exp(lse)
 * becomes a relative error e in that row's votes).  NULL: the library computes them.
 */
uncomp_status uncomp_window_score(uncomp_ctx* ctx, const void* Qwin, const void* K,
                                  uncomp_dtype dtype, int B, int H, int G, int N, int D,
                                  int w, int pool, const int64_t k_strides[3],
                                  const float* lse_opt, float* score_out, void* stream);

/*
 * Per-head top-k and compaction (Sec. 3.3.3: keep the N_{i,g} highest-scoring tokens;
 * Alg. 2 prefill: compress each head's KV by its group's budget).
 *
 * score [B][H][P] floats, no NaNs (P = N - w), budget [B][H] int32 (device).  Per head:
 * b = clamp(budget, w, min(N, cap)); the b - w prefix positions of largest score are
 * kept, equal scores by lower position, followed by the w window positions.
 * idx_out[b][h][0..len) lists the kept positions in ascending order, len_out[b][h] = b;
 * K_out/V_out[b][h][r][:] = K/V[b][h][idx[r]][:] copied bit for bit.  Rows and indices at
 * r >= len are left untouched.  K and V share kv_strides (element strides of batch, head,
 * token; features contiguous); outputs are dense [B][H][cap][D] / [B][H][cap].
 * Requires w <= cap and score 16-byte aligned.  K/V/K_out/V_out may be NULL together to obtain
 * indices only.
 */
uncomp_status uncomp_select_gather(uncomp_ctx* ctx, const float* score, const int32_t* budget,
                                   const void* K, const void* V, uncomp_dtype dtype,
                                   int B, int H, int N, int D, int w,
                                   const int64_t kv_strides[3], int cap,
                                   void* K_out, void* V_out, int32_t* idx_out, int32_t* len_out,
                                   void* stream);

/*
 * Decode-time eviction (Sec. 3.3.3 "Dynamic KV Cache Eviction", last sentence: as tokens
 * are generated the entry of lowest cumulative attention score leaves; Alg. 2 "Decoding":
 * the new token joins the head's cache, the query attends to the joined cache, the cache
 * is updated).  The state of a head is what uncomp_select_gather produced: K_c / V_c
 * [n_heads][cap][D] rows, idx [n_heads][cap] their original positions, len [n_heads] the
 * rows in use, plus cum [n_heads][cap] floats, the cumulative score of each row.  All of it
 * is DEVICE memory owned by the caller and updated in place.
 *
 * uncomp_decode_init fills cum from the prefill score: cum[h][r] = score[h][idx[h][r]] for
 * r < len[h] and idx < N - w; rows of the observation window (idx >= N - w) and rows at
 * r >= len[h] start at 0.  score is [n_heads][N - w] floats.
 */
uncomp_status uncomp_decode_init(uncomp_ctx* ctx, const float* score, const int32_t* idx,
                                 const int32_t* len, int n_heads, int N, int w, int cap,
                                 float* cum_out, void* stream);

/*
 * One generated token for n_heads KV heads (any mix of layers and sequences).  q
 * [n_heads][G][D], k_new / v_new [n_heads][D] (dense, dtype as the cache), pos [n_heads]
 * int32 the token's position in its sequence, budget [n_heads] int32.  Per head, with n =
 * len[h] rows cached:
 *   1. the new token joins with cumulative score 0 (n + 1 entries);
 *   2. p_g = softmax over the entries of q_g . k / sqrt(D) in fp32;
 *      out[h][g][:] = sum_r p_gr v_r  (floats [n_heads][G][D]; out may be NULL);
 *   3. cum of every entry grows by sum_g p_gr;
 *   4. b = clamp(budget[h], w, cap).  If n + 1 > b, the entry of lowest cum among those at
 *      positions <= pos - w (the w most recent positions are exempt) leaves, equal scores
 *      by lower position, and the new token takes its row; len stays n and evicted[h] is the
 *      position that left.  Otherwise the new token takes row n, len becomes n + 1 and
 *      evicted[h] = -1.  (evicted may be NULL.)
 * Row order inside a head is therefore unspecified after the first eviction; idx tells which
 * position a row holds.  A malformed state in which the head is over budget but no entry is
 * old enough to leave appends while n < cap, else drops the token and reports -2.
 * Requires 1 <= w <= cap, 1 <= G <= 16, D == 128, 16-byte aligned q / k_new / v_new / K_c /
 * V_c.  bf16 caches need uncomp_decode_workspace_bytes(n_heads, G, cap) of workspace (partial
 * results of the two kernels the step is split into) and are limited to caches whose
 * per-head merge tables fit 64 KiB of LDS (cap up to about 43 000 rows at G > 8, 87 000 at
 * G > 4, 349 000 at G <= 4 when the launch uses 256-row parts, half of that with 128-row
 * parts; beyond it UNCOMP_ERR_UNSUPPORTED, before anything is launched); fp32 caches need no
 * workspace but are limited to G*(cap + 1) <= 36864.  The workspace is shared with the prefill
 * calls of the context.
 */
size_t uncomp_decode_workspace_bytes(int n_heads, int G, int cap);
uncomp_status uncomp_decode_step(uncomp_ctx* ctx, const void* q, const void* k_new,
                                 const void* v_new, uncomp_dtype dtype, int n_heads, int G, int D,
                                 const int32_t* pos, const int32_t* budget, int w, int cap,
                                 void* K_c, void* V_c, int32_t* idx, float* cum, int32_t* len,
                                 float* out, int32_t* evicted, void* stream);

/*
 * Stage-1 hidden-state eviction (Sec. 3.3.2 "Hidden State Eviction": the tokens that enter the
 * next layer group are the N_{i+1} that receive the most attention from the last token in the
 * current layer; N_{i+1} is layer_tokens of uncomp_assign_budgets, Eq. 10).
 *
 * q_last [B][H*G][D] dense: the queries of the last position; K as in uncomp_window_score (the
 * current layer's keys over its N positions).  score[b][j] = sum over the H*G query heads of
 * softmax_j(q . k_j / sqrt(D)), j in [0, N), in fp32.  n_keep is a DEVICE pointer to one int32
 * (typically &layer_tokens[l + 1]) used for every batch entry.  Per batch entry:
 * n = clamp(*n_keep, w, min(N, cap)); the last w positions are kept unconditionally (the last
 * token carries the next prediction), plus the n - w earlier positions of largest score, equal
 * scores by lower position.  idx_out[b][0..n) lists them ascending, len_out[b] = n,
 * Hs_out[b][r][:] = Hs[b][idx[r]][:] bit for bit (rows of Dm elements of `dtype`; batch b, row t
 * of Hs at element b*hs_strides[0] + t*hs_strides[1]).  Outputs are dense [B][cap][Dm] / [B][cap];
 * rows at r >= n are left untouched.  score_out, if not NULL, receives score[b][0 .. N-w) as
 * [B][N-w] floats.  Hs / Hs_out may be NULL together to obtain indices only.
 * Requires 1 <= w < N, w <= cap, D == 128, Dm*sizeof(element) and the Hs strides in bytes
 * multiples of 16.  Workspace: uncomp_hidden_workspace_bytes.
 */
size_t uncomp_hidden_workspace_bytes(int B, int H, int G, int N, int w);
uncomp_status uncomp_hidden_evict(uncomp_ctx* ctx, const void* q_last, const void* K,
                                  uncomp_dtype dtype, int B, int H, int G, int N, int D,
                                  const int64_t k_strides[3], const int32_t* n_keep, int w,
                                  const void* Hs, const int64_t hs_strides[2], int Dm, int cap,
                                  void* Hs_out, int32_t* idx_out, int32_t* len_out,
                                  float* score_out, void* stream);

/*
 * Offline preparation (Sec. 3.3.1 "Preparation Stage", Eq. 7: a head's grouping metric is its
 * erank_k averaged over the d sampled prompts; App. "A Comprehensive Walk-Through", Alg. 1: per
 * sample every head gets one of M labels from its entropy, the final label is the majority's).
 *
 * The running statistics are DEVICE memory owned by the caller: erank_sum [n_layer][H] doubles,
 * votes [n_layer][H][M] int32, count one int32.  uncomp_prepare_reset zeroes them.
 * uncomp_prepare_accumulate adds the n_batch samples of entropy [n_layer][n_batch][H] (the layout
 * uncomp_head_entropy is used with): erank_sum += exp(entropy) in double precision, samples in
 * index order; per sample and layer the heads are ranked by entropy (larger first, equal values by
 * lower head index), rank r votes for label r / (H/M); count += n_batch.
 * uncomp_prepare_finish writes labels_mean [n_layer][H] (heads of a layer ranked by erank_sum /
 * count into M groups, group 0 = largest) and labels_vote [n_layer][H] (the label with most votes,
 * equal counts towards the lower label); mean_erank_out, if not NULL, gets the means as floats.
 * uncomp_budgets_from_labels is Eq. 11 from stored labels:
 * head_budget[l][b][h] = clamp(n_max - labels[l][h]*step, min(w, N), N), [n_layer][n_batch][H].
 * Limits as for uncomp_assign_budgets: H <= 1024, n_layer <= 4096, M divides H.
 */
uncomp_status uncomp_prepare_reset(uncomp_ctx* ctx, int n_layer, int H, int M, double* erank_sum,
                                   int32_t* votes, int32_t* count, void* stream);
uncomp_status uncomp_prepare_accumulate(uncomp_ctx* ctx, const float* entropy, int n_layer,
                                        int n_batch, int H, int M, double* erank_sum,
                                        int32_t* votes, int32_t* count, void* stream);
uncomp_status uncomp_prepare_finish(uncomp_ctx* ctx, int n_layer, int H, int M,
                                    const double* erank_sum, const int32_t* votes,
                                    const int32_t* count, int32_t* labels_mean,
                                    int32_t* labels_vote, float* mean_erank_out, void* stream);
uncomp_status uncomp_budgets_from_labels(uncomp_ctx* ctx, const int32_t* labels, int n_layer,
                                         int n_batch, int H, int n_max, int step, int N, int w,
                                         int32_t* head_budget, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* UNCOMP_H */
