/*
 * sp.h -- C ABI of the MI355X (gfx950) token-importance library for
 * cross-family speculative prefill.
 *
 * The library computes, on one GPU, the draft-model token-importance pass of
 * the paper "Cross-Family Speculative Prefill": attention of the lookahead
 * queries over the prompt's keys in every draft layer, max/mean aggregation to
 * one score per prompt token, average pooling, chunk means, top-k chunk
 * selection, merging into spans, projection of those spans through character
 * offsets onto another tokenisation, and assembly of the compressed prompt's
 * token and position ids (Algorithm 1; Appendix A.1).
 *
 * Conventions shared by every call
 *  - Pointers named *_dev point to device memory of the current HIP device and
 *    are owned by the caller; pointers named *_host point to host memory that
 *    is read during the call only. The library never allocates or frees device
 *    memory; scratch space comes from the caller's workspace (`ws_dev`), whose
 *    size the *_workspace functions report. Workspaces must be 256-byte aligned.
 *  - All device work is enqueued on `hip_stream` (a hipStream_t passed as
 *    void*; NULL is the default stream). No call synchronises with the host;
 *    outputs, including the n_*_dev counters, are valid once the stream has
 *    been synchronised. Two calls sharing a workspace must be ordered by the
 *    stream.
 *  - Every call returns an sp_status and never aborts. Host-visible arguments
 *    are validated before anything is launched; on an error nothing is
 *    launched and no output is written. sp_last_error() returns a thread-local
 *    description of the last failure.
 *  - Contents of device buffers (offsets non-decreasing, finite scores, the
 *    host and device copies of the batch offsets agreeing) are the caller's
 *    contract and are not checked.
 */
#ifndef SP_H_
#define SP_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SP_OK = 0,
    SP_ERR_INVALID_ARG = 1,   /* null pointer, non-positive size, inconsistent sizes */
    SP_ERR_UNSUPPORTED = 2,   /* valid request outside the supported set */
    SP_ERR_WORKSPACE = 3,     /* workspace missing, misaligned or too small */
    SP_ERR_DEVICE = 4         /* a HIP call failed */
} sp_status;

/* How per-layer head maxima are combined (Appendix A.1.1; Algorithm 1
 * "AggregateMaxMean"). SP_LAYER_MAX is the paper's statement: maximum over
 * layers and heads, then mean over the lookahead rows. SP_LAYER_MEAN takes the
 * maximum over heads only and averages over lookahead rows and layers. */
typedef enum { SP_LAYER_MEAN = 0, SP_LAYER_MAX = 1 } sp_layer_agg;

/* Shape of the draft model's attention and of its K cache.
 * Q is dense bf16 [n_layers][n_q_heads][n_q][head_dim] (per prompt).
 * K of one layer is bf16 with head_dim contiguous; element (kv head, token j,
 * e) sits at  kv * k_stride_head + j * k_stride_token + e  (strides in
 * elements, multiples of 8; layer base pointers 16-byte aligned). Query head h
 * reads kv head h / (n_q_heads / n_kv_heads).
 * Supported: head_dim 64 or 128; 1 <= n_q <= 16; n_q_heads a multiple of
 * n_kv_heads with ratio G <= 16; n_layers <= 128; n_layers * n_kv_heads <=
 * 65535; scale finite and > 0; and the kv head's query group must fit the
 * on-chip staging: with R = 32 * ceil(G/4) * ceil(n_q/8) padded query rows,
 * R <= 224 at head_dim 64 and R <= 96 at head_dim 128 (so G = 16 with
 * n_q > 8 at head_dim 64, and G > 12 or G > 4 with n_q > 8 at head_dim 128,
 * are SP_ERR_UNSUPPORTED). */
typedef struct {
    int32_t n_layers;
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t n_q;              /* lookahead query rows (the paper's N) */
    float   scale;            /* logit scale, normally 1/sqrt(head_dim) */
    int32_t layer_agg;        /* sp_layer_agg */
    int64_t k_stride_token;
    int64_t k_stride_head;
} sp_score_desc;

/* Bytes of workspace sp_score / sp_score_batch need for `total_tokens` prompt
 * tokens in `n_prompts` prompts (upper bound; 1 prompt for sp_score).
 * The first 32-bit word of the workspace is the status word of the last score
 * call that used it: once the stream has been synchronised it reads 0 when the
 * scores are valid and 1 when the single-launch kernel gave up (see sp_score);
 * a caller that cannot scan the scores for NaN can copy this word back. */
sp_status sp_score_workspace(const sp_score_desc *desc, int64_t total_tokens,
                             int32_t n_prompts, size_t *bytes);

/*
 * Token importance of one prompt (Appendix A.1.1; Algorithm 1, the
 * ForwardWithAttn loop's attention and AggregateMaxMean).
 * For every layer l, query head h and lookahead row n the row
 *   p[l,h,n,j] = softmax_j( scale * <Q[l,h,n,:], K[l,h/G,j,:]> ),  j in [0,L)
 * is formed over exactly the L prompt keys (no mask: lookahead rows follow the
 * prompt), and scores_dev[j] receives
 *   SP_LAYER_MAX :  (1/n_q)          sum_n max_{l,h} p[l,h,n,j]
 *   SP_LAYER_MEAN:  (1/(n_q*Lyr))    sum_l sum_n max_h p[l,h,n,j].
 * q_dev: bf16 Q as described above. k_layers_host: host array of n_layers
 * device pointers. scores_dev: float[L]. L == 0 is a no-op returning SP_OK.
 * The softmax is exact (row maximum and sum over all L keys, fp32); the result
 * is deterministic: the same inputs give bit-identical scores.
 * The single-launch kernel (see sp_score_is_fused) needs all its workgroups
 * resident at once, which an otherwise idle device guarantees; if other work
 * occupies the device, its waits on other workgroups are bounded (about a
 * second), after which the call has failed as a whole: every score of the call
 * is NaN and the workspace's status word (see sp_score_workspace) is 1. It
 * never hangs, and a failed call means "run again", never a wrong value.
 */
sp_status sp_score(const sp_score_desc *desc, const void *q_dev,
                   const void *const *k_layers_host, int64_t L,
                   float *scores_dev, void *ws_dev, size_t ws_bytes,
                   void *hip_stream);

/*
 * sp_score with the lookahead tokens' own keys in the softmax (Algorithm 1, the
 * ForwardWithAttn loop: the forward pass of lookahead step i also attends to
 * the tokens generated in steps 1 .. i-1). Row n (0-based) of every head is
 * normalised over the L prompt keys and the lookahead keys 0 .. n-1, plus key n
 * itself when look_self is 1 (0 or 1; anything else is SP_ERR_INVALID_ARG):
 *   p[l,h,n,j] = exp(s[l,h,n,j]) / ( sum_{j'<L} exp(s[l,h,n,j'])
 *                                    + sum_{m visible} exp(scale*<Q[l,h,n,:], Klook[l,h/G,m,:]>) )
 * Only prompt tokens are scored; aggregation as in sp_score.
 * k_look_dev: device, bf16, dense [n_layers][n_kv_heads][n_q][head_dim],
 * 16-byte aligned, not null, only read. Everything else as in sp_score (same
 * workspace size, same kernels, same determinism and failure behaviour).
 */
sp_status sp_score_look(const sp_score_desc *desc, const void *q_dev,
                        const void *const *k_layers_host, int64_t L,
                        const void *k_look_dev, int32_t look_self,
                        float *scores_dev, void *ws_dev, size_t ws_bytes,
                        void *hip_stream);

/*
 * sp_score over a paged key cache (Section 3.1 describes KV caches kept in
 * fixed-size blocks of 4k tokens). Token j of layer l lives in page
 * block_table_dev[j / page_tokens] of that layer's pool k_pools_host[l]:
 *   K[l, kv, j, e] = pool_l[ page * page_stride + kv * k_stride_head
 *                            + (j % page_tokens) * k_stride_token + e ]
 * with desc's strides now describing one page (e.g. head-major pages:
 * k_stride_token = head_dim, k_stride_head = page_tokens * head_dim,
 * page_stride = n_kv_heads * page_tokens * head_dim). One block table serves all
 * layers, as in paged decoders. block_table_dev: device, int32,
 * ceil(L / page_tokens) entries, only read. page_tokens: a positive multiple of
 * 512; page_stride: elements, a multiple of 8; every page is allocated whole
 * (rows of the last page beyond L may be read, their contents are ignored).
 * Same result as sp_score on the gathered keys, same kernels, same workspace.
 */
sp_status sp_score_paged(const sp_score_desc *desc, const void *q_dev,
                         const void *const *k_pools_host,
                         const int32_t *block_table_dev, int64_t page_tokens,
                         int64_t page_stride, int64_t L, float *scores_dev,
                         void *ws_dev, size_t ws_bytes, void *hip_stream);

/*
 * sp_score over keys stored as 8-bit floating point (Section 3.1: the deployment
 * keeps its KV cache in blocks on the accelerator; a quantised cache halves the
 * bytes this pass streams). k8_layers_host[l] points at layer l's keys as OCP
 * E4M3 codes (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, finite
 * only; one byte per element), addressed with desc's strides counted in
 * elements, i.e. bytes (multiples of 8, layer bases 16-byte aligned).
 * kscale_dev: device, float [n_layers][n_kv_heads], positive and finite, only
 * read: the key vector of (l, kv, j) is kscale[l][kv] * E4M3(code), and the
 * scores are those of sp_score on exactly these dequantised keys (the queries
 * stay bf16; products are exact, sums are fp32). NaN codes are the caller's to
 * avoid. Contiguous keys of one prompt only; same workspace size and the same
 * choice between the two implementations as sp_score (sp_score_fp8_is_fused;
 * the single-launch kernel fetches codes in 16-byte pieces and so needs both
 * strides to be multiples of 16), same status word and failure behaviour.
 */
sp_status sp_score_fp8(const sp_score_desc *desc, const void *q_dev,
                       const void *const *k8_layers_host, const float *kscale_dev,
                       int64_t L, float *scores_dev, void *ws_dev, size_t ws_bytes,
                       void *hip_stream);

/* Which implementation sp_score picks for this shape and length on the current
 * device: 1 = the single-launch kernel that keeps K on chip and reads it from
 * HBM once, 0 = the three-kernel path, -1 = invalid or unsupported desc. The
 * single-launch kernel takes one workgroup per compute unit, each owning T keys:
 * head_dim 64: T = 512, query groups of up to 64 padded rows, 64 to 256
 * workgroups (about 32K to 128K tokens); head_dim 128: T = 256, up to 32 padded
 * rows, 96 to 256 workgroups (about 24K to 64K tokens). Results are the same
 * either way (to rounding); this is for reporting. Host-only. */
int32_t sp_score_is_fused(const sp_score_desc *desc, int64_t L);
/* The same for sp_score_fp8: its single-launch variants need key strides that are
 * multiples of 16 elements; shapes and lengths as above. */
int32_t sp_score_fp8_is_fused(const sp_score_desc *desc, int64_t L);

/*
 * The same for a ragged batch of B prompts whose keys are packed back to back
 * along the token axis: prompt b owns tokens [offsets[b], offsets[b+1]) of each
 * layer's K and of scores_dev; its queries are q_dev + b * (one prompt's Q).
 * offsets_host and offsets_dev hold the same B+1 non-decreasing values with
 * offsets[0] == 0; empty prompts are allowed. Each prompt is softmaxed over
 * its own keys only. 1 <= B <= 4096.
 */
sp_status sp_score_batch(const sp_score_desc *desc, const void *q_dev,
                         const void *const *k_layers_host,
                         const int64_t *offsets_host, const int64_t *offsets_dev,
                         int32_t B, float *scores_dev, void *ws_dev,
                         size_t ws_bytes, void *hip_stream);

/* How sp_score_batch runs this batch on the current device: n > 0 = on the
 * single-launch kernel in n launches (every prompt empty or at least T tokens
 * long and no longer than T tokens per compute unit, T as above; at least 64
 * workgroups in all; prompts share launches, each with all its keys in one),
 * 0 = the three-kernel path, -1 = invalid
 * arguments. Same results either way (to rounding). Host-only. */
int32_t sp_score_batch_is_fused(const sp_score_desc *desc,
                                const int64_t *offsets_host, int32_t B);

/* Number of chunks to keep for a keep rate keep_num/keep_den (Section 3.1: the
 * top-K chunks make up a fraction rho of the draft sequence):
 * clamp(ceil(n_chunks * keep_num / keep_den), 1, n_chunks) in integer
 * arithmetic. Returns -1 on invalid arguments (n_chunks < 1, keep_den < 1,
 * keep_num < 0). Host-only. */
int64_t sp_keep_count(int64_t n_chunks, int64_t keep_num, int64_t keep_den);

/* Bytes of workspace sp_select needs for a prompt of L tokens and this chunk size. */
sp_status sp_select_workspace(int64_t L, int32_t chunk, size_t *bytes);

/*
 * Chunk selection (Algorithm 1: AvgPool1D, PartitionIntoChunks, TopKChunks,
 * MergeAdjacentChunks; Appendix A.1.2; Appendix A.3 for pool 13, chunk 32/128).
 *  - pooled[j] = (1/pool_w) * sum of scores over the pool_w-wide window centred
 *    on j, zeros outside [0,L), divisor always pool_w (pool_w odd, >= 1);
 *  - chunk i covers tokens [i*chunk, min((i+1)*chunk, L)); its score is the
 *    mean of pooled over its true size; C = ceil(L/chunk);
 *  - the k chunks with the largest scores are kept, equal scores resolved in
 *    favour of the lower chunk index (compared as fp32, -0 == +0);
 *  - sel_chunks_dev[k]: kept chunk indices, ascending;
 *  - spans_dev[k][2]: maximal runs of adjacent kept chunks as draft-token
 *    ranges [begin, end), ascending; *n_spans_dev of them are written;
 *  - chunk_scores_dev: optional float[C] copy of the chunk scores (may be NULL).
 * Requires 1 <= k <= C, 1 <= chunk, L >= 1. Scores must not be NaN.
 */
sp_status sp_select(const float *scores_dev, int64_t L, int32_t pool_w,
                    int32_t chunk, int64_t k, int32_t *sel_chunks_dev,
                    int64_t *spans_dev, int32_t *n_spans_dev,
                    float *chunk_scores_dev, void *ws_dev, size_t ws_bytes,
                    void *hip_stream);

/*
 * sp_select for a ragged batch of B prompts in two launches (Algorithm 1, the
 * same four steps, each prompt on its own: pooling windows and chunks never
 * cross a prompt's end). scores_dev is packed as sp_score_batch leaves it:
 * prompt b owns [offsets[b], offsets[b+1]). kept_off holds the prefix sums of the
 * prompts' chunk counts to keep, kept_off[0] = 0: prompt b keeps
 * k_b = kept_off[b+1] - kept_off[b] chunks, 1 <= k_b <= ceil(L_b / chunk), or 0
 * for an empty prompt (the caller fills it with sp_keep_count). offsets and
 * kept_off are each given twice with the same B+1 values, in host and in device
 * memory. Outputs, packed by kept_off:
 *  - sel_chunks_dev[kept_off[B]]: prompt b's k_b kept chunk indices (relative to
 *    the prompt), ascending, from kept_off[b] on;
 *  - spans_dev[kept_off[B]][2]: its spans as token ranges relative to the prompt,
 *    from kept_off[b] on; n_spans_dev[b] of them are written;
 *  - chunk_scores_dev: optional; prompt b's chunk scores start at
 *    offsets[b] / chunk + b (so total / chunk + B + 1 floats in all).
 * Workspace: sp_select_batch_workspace(offsets[B], B, chunk). 1 <= B <= 4096.
 */
sp_status sp_select_batch_workspace(int64_t total_tokens, int32_t B, int32_t chunk,
                                    size_t *bytes);
sp_status sp_select_batch(const float *scores_dev, const int64_t *offsets_host,
                          const int64_t *offsets_dev, int32_t B, int32_t pool_w,
                          int32_t chunk, const int64_t *kept_off_host,
                          const int64_t *kept_off_dev, int32_t *sel_chunks_dev,
                          int64_t *spans_dev, int32_t *n_spans_dev,
                          float *chunk_scores_dev, void *ws_dev, size_t ws_bytes,
                          void *hip_stream);

/*
 * sp_select for callers that cannot allocate device memory or pass a workspace:
 * code recorded into a HIP graph, tight serving loops, harnesses that forbid
 * hipMalloc. Same arguments, kernels and results as sp_select, without ws_dev /
 * ws_bytes: the chunk scores go to an array that is part of the library's
 * device image (SP_SELECT_STATIC_MAX_CHUNKS floats = 1 MiB, held on every
 * device the library is used on until the process ends). The call allocates
 * and frees nothing. More than SP_SELECT_STATIC_MAX_CHUNKS chunks is
 * SP_ERR_UNSUPPORTED (use sp_select). The first call on a device looks the
 * array's address up (a host-only query; make that call outside a graph
 * capture). All calls on one device share the array: calls that may overlap
 * on the device (different streams without ordering) race; calls ordered by a
 * stream or by events do not, and nothing has to be cleared between them.
 */
#define SP_SELECT_STATIC_MAX_CHUNKS (1 << 18)
sp_status sp_select_static(const float *scores_dev, int64_t L, int32_t pool_w,
                           int32_t chunk, int64_t k, int32_t *sel_chunks_dev,
                           int64_t *spans_dev, int32_t *n_spans_dev,
                           float *chunk_scores_dev, void *hip_stream);

/* Bytes of workspace sp_select_budget needs (SP_ERR_UNSUPPORTED beyond 65536 chunks). */
sp_status sp_select_budget_workspace(int64_t L, int32_t chunk, size_t *bytes);

/*
 * Chunk selection for a fixed target-side length (Section 3.1: compressed
 * prompts of 8k .. 32k target tokens, multiples of the KV block size; the
 * paper derives the keep rate from that length and notes that the result only
 * lands near it). Here k is searched on the device: the largest k in 1..C such
 * that the top-k chunks, merged into spans and projected onto the target
 * tokenisation exactly as sp_project does, keep at most `budget` target
 * tokens; k = 1 if a single chunk already keeps more. Pooling, chunk scores,
 * ranking and tie-breaking are those of sp_select, and the outputs are what
 * sp_select would write for that k, except that the buffers must hold the
 * worst case: sel_chunks_dev[C], spans_dev[C][2] (C = ceil(L/chunk) <= 65536).
 *  - draft_off_dev[L+1], target_off_dev[M+1]: character offsets as in sp_project;
 *  - *k_dev: the chosen k (also the number of entries of sel_chunks_dev written);
 *  - *n_kept_dev: optional, the target tokens kept at that k (what sp_project
 *    reports for the written spans);
 *  - chunk_scores_dev: optional float[C].
 * Requires L >= 1, 1 <= M < 2^31, budget >= 0. Integer work after the chunk
 * scores: exact and deterministic.
 */
sp_status sp_select_budget(const float *scores_dev, int64_t L, int32_t pool_w,
                           int32_t chunk, const int64_t *draft_off_dev,
                           const int64_t *target_off_dev, int64_t M,
                           int64_t budget, int32_t *sel_chunks_dev,
                           int64_t *spans_dev, int32_t *n_spans_dev,
                           int64_t *k_dev, int64_t *n_kept_dev,
                           float *chunk_scores_dev, void *ws_dev,
                           size_t ws_bytes, void *hip_stream);

/*
 * Projection of kept draft-token spans onto the target model's tokenisation
 * (Algorithm 1: MapDraftChunksToTextSpans and the target tokenisation of the
 * kept text; Section 3.1), in character-offset form. Both tokenisations are
 * given as non-decreasing character offsets into the same text:
 * draft_off_dev[L+1] and target_off_dev[M+1]. Draft span [a,b) covers
 * characters [draft_off[a], draft_off[b]); target token t is kept iff
 *      target_off[t] < draft_off[b]  and  target_off[t+1] > draft_off[a]
 * for some span. spans_dev is a buffer of max_spans entries whose first
 * *n_spans_dev (at most max_spans) are ascending, disjoint spans, as written by
 * sp_select; the kernels may read the entries after them (so all max_spans
 * must be readable device memory) and do not use what they hold.
 *  - tspans_dev[max_spans][2]: kept target tokens as maximal ranges
 *    [begin, end), ascending, disjoint and non-adjacent (ranges that overlap or
 *    touch are merged); *n_tspans_dev of them are written;
 *  - keep_mask_dev: optional uint8[M], 1 for kept target tokens (may be NULL);
 *  - *n_kept_dev: number of kept target tokens.
 * Requires L >= 1, M >= 1, 1 <= max_spans <= 2^24.
 */
sp_status sp_project(const int64_t *draft_off_dev, int64_t L,
                     const int64_t *target_off_dev, int64_t M,
                     const int64_t *spans_dev, const int32_t *n_spans_dev,
                     int32_t max_spans, int64_t *tspans_dev,
                     int32_t *n_tspans_dev, uint8_t *keep_mask_dev,
                     int64_t *n_kept_dev, void *hip_stream);

/*
 * sp_project for a ragged batch in one launch (Algorithm 1, the same mapping,
 * each prompt on its own text). Packed inputs: prompt b's L_b + 1 draft offsets
 * start at draft_off_dev[offsets[b] + b], its M_b + 1 target offsets at
 * target_off_dev[moffsets[b] + b] (moffsets = prefix sums of the prompts' target
 * token counts), its spans at spans_dev[kept_off[b]] with n_spans_dev[b] of them
 * valid, as sp_select_batch writes them. Packed outputs: prompt b's target ranges
 * (relative to its own target tokens) from tspans_dev[kept_off[b]] on,
 * n_tspans_dev[b] of them; its mask bytes at keep_mask_dev[moffsets[b]] (optional);
 * n_kept_dev[b]. offsets, moffsets and kept_off are each given in host and in
 * device memory with the same B+1 values, first value 0. A prompt may have at
 * most 1024 spans and fewer than 258048 target tokens (SP_ERR_UNSUPPORTED
 * otherwise: call sp_project for it). 1 <= B <= 4096.
 */
sp_status sp_project_batch(const int64_t *draft_off_dev, const int64_t *offsets_host,
                           const int64_t *offsets_dev, const int64_t *target_off_dev,
                           const int64_t *moffsets_host, const int64_t *moffsets_dev,
                           int32_t B, const int64_t *spans_dev,
                           const int32_t *n_spans_dev, const int64_t *kept_off_host,
                           const int64_t *kept_off_dev, int64_t *tspans_dev,
                           int32_t *n_tspans_dev, uint8_t *keep_mask_dev,
                           int64_t *n_kept_dev, void *hip_stream);

/* Bytes of workspace sp_assemble needs for up to max_spans kept ranges. */
sp_status sp_assemble_workspace(int32_t max_spans, size_t *bytes);

/*
 * Compressed target prompt in token-id form (Algorithm 1: ConcatWithDelim, the
 * target tokenisation of the compressed text and the new contiguous position
 * ids; Section 3.2; Appendix A.3 names the delimiters). target_ids_dev[M] is
 * the target tokenisation of the original text; tspans_dev holds
 * *n_tspans_dev (at most max_spans) ascending, disjoint ranges [begin, end) of
 * kept target tokens, as written by sp_project; delim_ids_dev[n_delim] is the
 * delimiter's own tokenisation (n_delim may be 0, then the pointer may be NULL).
 * The output is the kept ranges in order with the delimiter's ids between
 * consecutive ranges (none before the first or after the last):
 *  - *out_len_dev = kept tokens + (ranges - 1) * n_delim  (0 for no range),
 *    the full length even when it exceeds out_capacity;
 *  - the first min(out_len, out_capacity) entries are written of
 *    out_ids_dev (token ids), out_pos_dev (position ids 0, 1, 2, ...: the
 *    compressed prompt is renumbered, original positions are not restored) and
 *    the optional out_src_dev (original target index of each output token, -1
 *    for delimiter tokens; may be NULL).
 * Requires M >= 1, 1 <= max_spans <= 2^24, 0 <= n_delim <= 1024,
 * 1 <= out_capacity < 2^31. Range bounds are not checked beyond clamping to [0, M].
 */
sp_status sp_assemble(const int32_t *target_ids_dev, int64_t M,
                      const int64_t *tspans_dev, const int32_t *n_tspans_dev,
                      int32_t max_spans, const int32_t *delim_ids_dev,
                      int32_t n_delim, int64_t out_capacity,
                      int32_t *out_ids_dev, int32_t *out_pos_dev,
                      int64_t *out_src_dev, int64_t *out_len_dev,
                      void *ws_dev, size_t ws_bytes, void *hip_stream);

/*
 * Measurement aid: streams `bytes` bytes of buf_dev (device, 16-byte aligned,
 * bytes a positive multiple of 16) with plain wide loads and XORs what it read
 * into *sink_dev (device, 64 bits: lanes fold their 16-byte chunks to 64 bits
 * as (x ^ z) << 32 | (y ^ w) of the four 32-bit words; not cleared first).
 * The rate at which this call reads is the device's achievable streaming-read
 * bandwidth: the practical ceiling, next to the datasheet figure, for
 * sp_score, which streams the K cache once (Appendix A.1.1's attention of the
 * lookahead rows over the whole prompt). Enqueued on hip_stream like every
 * other call.
 */
sp_status sp_hbm_read_probe(const void *buf_dev, size_t bytes, uint64_t *sink_dev,
                            void *hip_stream);

/* Test hook for the failure path of the single-launch score kernel; not for
 * production use. Launches that follow give a wait up after `spin_limit` polls
 * (default 1 << 20), and with force_miss != 0 the waves that combine partial
 * results treat them as never arriving, so that the bounded waits give up on an
 * idle device and every kernel still runs to its end. Process-wide. */
void sp_debug_fused_giveup(uint32_t spin_limit, int32_t force_miss);

/* Description of the last error raised on the calling thread ("" if none).
 * The string lives in thread-local storage owned by the library. */
const char *sp_last_error(void);

/* Library version string (static storage). */
const char *sp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SP_H_ */
