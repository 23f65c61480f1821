/*
 * chunkkv.h - C ABI of the MI355X (gfx950) ChunkKV prefill-time KV-cache compression library.
 *
 * The operations follow ChunkKV (arXiv 2502.00299): Algorithm 1 (Section 3.2: observation-window
 * attention scores -> chunk scores -> top-k chunks -> index_select + window concatenation),
 * Algorithm 3 (Appendix A.5: boundary handling, ragged last chunk, window always kept) and
 * Algorithm 2 (Section 3.3: layer-wise index reuse).
 *
 * Conventions
 *   L  sequence length (T_k in the paper)      w  observation window     P = L - w  candidate tokens
 *   c  chunk size                              C = ceil(P / c) chunks    Hq / Hkv query / kv heads
 *   g = Hq / Hkv                               d  head dim               n_keep  candidate tokens kept
 *   n_kept = n_keep + w  (L_max in the paper)  R  reuse depth (N_reuse in the paper)
 *
 * Every pointer named "device" is GPU memory owned by the caller.  No call allocates or frees device
 * memory and none synchronises the device; the one exception is the measurement aid at the end of this
 * file (chunkkv_timing_begin creates HIP events, chunkkv_timing_end waits for them and destroys them).
 * All work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the default stream); there is
 * no process-wide setting: what a call does depends on its arguments alone.  Host arrays inside chunkkv_problem and the per-layer pointer tables are
 * read before the call returns.  Inputs are never written; outputs must not alias inputs.
 * Inputs containing NaN/Inf give undefined results (no fault).
 *
 * Every function returns CHUNKKV_OK (0) or a positive chunkkv_status; nothing is enqueued when an
 * argument check fails.
 */
#ifndef CHUNKKV_H
#define CHUNKKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CHUNKKV_OK = 0,
  CHUNKKV_ERR_NULL = 1,        /* a required pointer is NULL                                     */
  CHUNKKV_ERR_SHAPE = 2,       /* inconsistent sizes: w > L, n_keep > P, Hq % Hkv != 0, caps ... */
  CHUNKKV_ERR_UNSUPPORTED = 3, /* head_dim / dtype / row count not compiled in, K rows span >= 2 GiB */
  CHUNKKV_ERR_WORKSPACE = 4,   /* workspace smaller than chunkkv_workspace_bytes()               */
  CHUNKKV_ERR_LAUNCH = 5       /* the HIP runtime refused a launch                               */
} chunkkv_status;

/* Storage type of Q, K, V (and K', V').  Logits accumulate in fp32 for all three; the 16-bit types take the
 * same kernels (the paper sizes its caches in fp16, Eq. 1). */
typedef enum { CHUNKKV_F32 = 0, CHUNKKV_BF16 = 1, CHUNKKV_F16 = 2 } chunkkv_dtype;

/* One batch of sequences sharing head geometry.  K and V of a layer live in one buffer each; token t
 * of kv-head h of sequence b starts at element  kv_base[b] + h*kv_stride_head + t*kv_stride_tok  and
 * its d elements are contiguous.  Both [B][Hkv][L][d] and packed variable-length [sum L][Hkv][d] fit.
 * Row starts must be 16-byte aligned.  Outputs use out_base / out_stride_* the same way with n_kept_b
 * tokens per head.  Supported: head_dim 64 or 128; g*w <= 512; the K rows of one (sequence, kv-head) must
 * span less than 2 GiB, (L_b + 256) * kv_stride_tok * element size < 2^31 (about 1 M tokens of a packed
 * 8-head bf16 cache, 8 M tokens per head in [B][Hkv][L][d]); batch and heads limited only by int32.   */
typedef struct {
  int32_t batch, n_q_heads, n_kv_heads, head_dim;
  int32_t window, chunk;        /* w >= 1, c >= 1                                                  */
  int32_t dtype;                /* chunkkv_dtype: storage type of Q, K, V and of K', V'            */
  float softmax_scale;          /* 0 selects 1/sqrt(head_dim)                                      */
  const int32_t *seqlen;        /* host[batch]   L_b >= w                                          */
  const int32_t *n_keep;        /* host[batch]   0 <= n_keep_b <= L_b - w                          */
  const int64_t *kv_base;       /* host[batch]   element offsets into K / V                        */
  int64_t kv_stride_head, kv_stride_tok;
  const int64_t *out_base;      /* host[batch]   element offsets into K' / V'                      */
  int64_t out_stride_head, out_stride_tok;
  int32_t sel_cap;              /* >= max_b ceil(n_keep_b / c) + 1 : row pitch of sel_chunk/sel_len */
  int32_t score_cap;            /* >= max_b ceil(P_b / c)          : row pitch of chunk_scores      */
  uint32_t flags;               /* CHUNKKV_FLAG_* bits, 0 = defaults; unknown bits: CHUNKKV_ERR_UNSUPPORTED */
} chunkkv_problem;

/* chunkkv_problem.flags
 * CHUNKKV_FLAG_WHOLE_CHUNKS  selection as Algorithm 3 prints it (Appendix A.5): k = min(floor(n_keep / c), C)
 *     chunks are kept whole and nothing is cut, so a head keeps k*c tokens, or fewer when the ragged last
 *     chunk is among them.  In chunkkv_compact / chunkkv_compress_* the window then follows the kept tokens
 *     directly, rows past kept + w of an output head are left untouched, and the caller reads the kept count
 *     of a head as the sum of its sel_len entries.  Default (bit clear): exactly n_keep tokens are kept, the
 *     lowest-ranked selected chunk is cut to its leading tokens.
 * CHUNKKV_FLAG_TWO_PASS  score with the general two-pass kernels even where the single-pass kernel applies
 *     (same results to rounding; the two implementations are described above chunkkv_timing_begin).       */
#define CHUNKKV_FLAG_WHOLE_CHUNKS 1u
#define CHUNKKV_FLAG_TWO_PASS 2u

/* Selection descriptor (the paper's kept-index set I_l, Algorithm 2), per (sequence, kv-head):
 *   sel_count            number of entries
 *   sel_chunk[0..count)  strictly ascending chunk indices
 *   sel_len[0..count)    leading tokens kept of that chunk, 1 <= len <= size of the chunk
 * The window [P, L) is implicit and always kept.  Entries past sel_count are left untouched.      */

const char *chunkkv_status_string(int status);

/* Bytes of device workspace the calls below need for this problem; n_layers = reuse = 1 for the
 * single-layer calls.  Returns 0 if the problem is invalid.                                        */
size_t chunkkv_workspace_bytes(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse);

/* Algorithm 1, scoring steps (with the softmax the text implies): for every kv-head, the g*w window
 * rows (window row i of a head attends keys 0..P+i) are soft-maxed over their visible keys, summed
 * over rows into per-token importance for tokens < P, and summed per chunk.
 *   q_obs             device [B][Hq][w][d], the last w queries of every head
 *   k                 device, layout given by prob
 *   chunk_scores      device float [B][Hkv][score_cap]; entries [0, C_b) written
 *   token_importance  device float [B][Hkv][score_cap*c] or NULL; entries [0, P_b) written
 * bf16 and fp16 inputs are multiplied on the matrix cores with fp32 accumulation; f32 inputs in fp32.       */
int chunkkv_score(const chunkkv_problem *prob, const void *q_obs, const void *k, float *chunk_scores,
                  float *token_importance, void *workspace, size_t workspace_bytes, void *stream);

/* Algorithm 1, top-k step, with the exact-budget rule: chunks are ranked by (score descending, index
 * ascending); whole chunks are taken in rank order and the last-ranked one is cut to its leading
 * tokens so that exactly n_keep_b tokens are kept.  Scores must be finite; -0 counts as +0.
 *   chunk_scores  device float [B][Hkv][score_cap]
 *   sel_chunk, sel_len  device int32 [B][Hkv][sel_cap];  sel_count device int32 [B][Hkv]           */
int chunkkv_chunk_topk(const chunkkv_problem *prob, const float *chunk_scores, int32_t *sel_chunk,
                       int32_t *sel_len, int32_t *sel_count, void *workspace, size_t workspace_bytes,
                       void *stream);

/* Algorithm 1, compression + concatenation: K'[h] = rows of K[h] named by the selection, in order,
 * followed by the window rows [P, L); same for V.  Pure copies, bit-exact.  The selection must obey
 * the descriptor rules above and keep exactly n_keep_b tokens (not checked on the device).         */
int chunkkv_compact(const chunkkv_problem *prob, const void *k, const void *v, const int32_t *sel_chunk,
                    const int32_t *sel_len, const int32_t *sel_count, void *k_out, void *v_out,
                    void *stream);

/* Algorithm 2: for l = 0..n_layers-1, layers with l % reuse == 0 are scored and selected; every layer
 * is compacted with the selection of layer floor(l/reuse)*reuse.
 *   q_obs, k, v, k_out, v_out   host arrays of n_layers device pointers (q_obs[l] may be NULL when
 *                               l % reuse != 0)
 *   sel_chunk, sel_len          device int32 [G][B][Hkv][sel_cap], G = ceil(n_layers / reuse)
 *   sel_count                   device int32 [G][B][Hkv]                                            */
int chunkkv_compress_stack(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse,
                           const void *const *q_obs, const void *const *k, const void *const *v,
                           void *const *k_out, void *const *v_out, int32_t *sel_chunk, int32_t *sel_len,
                           int32_t *sel_count, void *workspace, size_t workspace_bytes, void *stream);

/* Variants for callers that run behind a fused attention kernel and therefore already hold, for every window
 * row, the log-sum-exp of its softmax (the paper's setup computes prefill attention with FlashAttention-2,
 * Section 4.1): the normalisation is taken from `lse` instead of being recomputed, so K is read once and the
 * statistics pass disappears.  p[i][j] = exp(softmax_scale * q_i . k_j - lse_i); everything after that is
 * as in chunkkv_score / chunkkv_compress_stack.
 *   lse   device float [B][Hq][w], natural logarithm, over the keys row i sees (j <= P + i);
 *         chunkkv_compress_stack_lse takes a host array of n_layers device pointers (entries of layers
 *         with l % reuse != 0 may be NULL).  Values are used as given: an lse that does not match q and k
 *         scales that row's contribution by exp(true lse - given lse).
 * Errors as for the plain calls; CHUNKKV_ERR_NULL for a missing lse.                                          */
int chunkkv_score_lse(const chunkkv_problem *prob, const void *q_obs, const void *k, const float *lse,
                      float *chunk_scores, float *token_importance, void *workspace, size_t workspace_bytes,
                      void *stream);
int chunkkv_compress_stack_lse(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse,
                               const void *const *q_obs, const void *const *k, const void *const *v,
                               const float *const *lse, void *const *k_out, void *const *v_out,
                               int32_t *sel_chunk, int32_t *sel_len, int32_t *sel_count, void *workspace,
                               size_t workspace_bytes, void *stream);

/* Streaming form of Algorithm 2: one call per layer, in layer order, as prefill produces the layer's K and V
 * (the paper compresses each layer's cache before the following attention blocks run, Section 3.1).  Layer
 * `layer` with layer % reuse == 0 is scored and selected into selection group layer / reuse; every layer is
 * compacted with the selection of its group, which an earlier call of the same sequence of calls has written.
 *   q_obs            device [B][Hq][w][d]; may be NULL when layer % reuse != 0
 *   lse              NULL, or the window rows' log-sum-exps as in chunkkv_score_lse (used when not NULL)
 *   k, v, k_out, v_out   this layer's device buffers
 *   sel_chunk, sel_len, sel_count   the arrays of chunkkv_compress_stack ([G][B][Hkv][sel_cap], [G][B][Hkv]);
 *                    group layer / reuse is written (leader layers) or read (the others)
 *   workspace        chunkkv_workspace_bytes(prob, 1, 1) bytes; nothing in it has to survive between calls
 * prob->chunk may differ between reuse groups (Section 4.6 runs different chunk sizes in different layers), but
 * every layer of one group must be passed the chunk size of the group's leader: the selection arrays store
 * chunk indices, the library keeps no record of the grid they refer to, and a follower called with another
 * chunk size gathers other tokens without any error.  chunkkv_compress_stack_hybrid takes the table of chunk
 * sizes once and cannot get this wrong.
 * Results are those of chunkkv_compress_stack over the same layers.  Errors as there.                       */
int chunkkv_compress_layer(const chunkkv_problem *prob, int32_t layer, int32_t reuse, const void *q_obs,
                           const float *lse, const void *k, const void *v, void *k_out, void *v_out,
                           int32_t *sel_chunk, int32_t *sel_len, int32_t *sel_count, void *workspace,
                           size_t workspace_bytes, void *stream);

/* Algorithm 2 with a chunk size per reuse group (the hybrid setting among the chunk-size ablations of
 * Section 4.6; chunk size 1 in a group is token-level selection there).  Group G = l / reuse scores, selects
 * and gathers with chunk_per_group[G]; prob->chunk is ignored; the budget n_keep[b] is the same token count in
 * every group.  Implemented as chunkkv_compress_stack over each run of consecutive groups with one chunk size,
 * so the results of a group are those of chunkkv_compress_stack with that chunk size.
 *   chunk_per_group  HOST int32 [ceil(n_layers / reuse)], every entry >= 1
 *   lse              NULL, or as in chunkkv_compress_stack_lse
 *   sel_chunk, sel_len, sel_count   as in chunkkv_compress_stack; group G's entries count chunks of
 *                    chunk_per_group[G] tokens.  prob->sel_cap and prob->score_cap must hold for the smallest
 *                    chunk size in the table.
 *   workspace        chunkkv_workspace_bytes_hybrid(...) bytes (0 = invalid arguments): the largest need of
 *                    any chunk size in the table
 * All arguments are checked for every run before the first launch.  Errors as for chunkkv_compress_stack;
 * CHUNKKV_ERR_NULL for a missing table, CHUNKKV_ERR_SHAPE for an entry < 1 or a capacity too small for it.    */
size_t chunkkv_workspace_bytes_hybrid(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse,
                                      const int32_t *chunk_per_group);
int chunkkv_compress_stack_hybrid(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse,
                                  const int32_t *chunk_per_group, const void *const *q_obs,
                                  const void *const *k, const void *const *v, const float *const *lse,
                                  void *const *k_out, void *const *v_out, int32_t *sel_chunk, int32_t *sel_len,
                                  int32_t *sel_count, void *workspace, size_t workspace_bytes, void *stream);

/* Adjacent-group Jaccard similarity of the kept token sets, the diagnostic that motivates layer-wise index
 * reuse (Section 3.3 and the similarity tables of Appendix B.2): for g = 0..n_groups-2
 *   jaccard[g][b][h] = |S_g n S_{g+1}| / |S_g u S_{g+1}|,  S_g = non-window tokens kept by group g
 * (1 when both sets are empty).  The window is left out: it is kept by every layer and would only raise
 * every value by the same amount.
 *   sel_chunk, sel_len, sel_count   selections of n_groups groups as written by the calls above (device)
 *   jaccard          device float [n_groups - 1][B][Hkv]
 * Malformed selections (counts outside [0, sel_cap], chunks not ascending) give unspecified values, never
 * an out-of-bounds access.  n_groups < 2 is CHUNKKV_ERR_SHAPE.                                             */
int chunkkv_jaccard(const chunkkv_problem *prob, int32_t n_groups, const int32_t *sel_chunk, const int32_t *sel_len,
                    const int32_t *sel_count, float *jaccard, void *stream);

/* Decoding over the (compressed) cache: the stage whose cache Eq. 1 sizes and whose latency Section 4.4
 * tabulates; Algorithm 1's output K', V' is its input.  One new query token per head attends to every
 * token of the cache of its kv-head (query head i reads kv-head i / g):
 *     out[b][i][:] = sum_t softmax_t(scale * q[b][i] . K[b][i/g][t]) * V[b][i/g][t][:]
 *   compacted   1: k, v are K', V' as written by chunkkv_compact / chunkkv_compress_* (prob->out_base,
 *               out_stride_*), n_keep_b + w tokens per head; 0: the uncompressed caches (prob->kv_base,
 *               kv_stride_*), seqlen_b tokens per head
 *   kv_len      device int32 [B][Hkv] or NULL: tokens to attend to per (sequence, kv-head), clamped to the
 *               count above (whole-chunk selection keeps a data-dependent count); 0 tokens give out = 0
 *   q           device [B][Hq][d] in prob->dtype, 16-byte aligned
 *   out         device float [B][Hq][d]
 *   lse         device float [B][Hq] or NULL: natural log of the softmax denominator (-inf for 0 tokens)
 *   workspace   device, chunkkv_decode_workspace_bytes(prob, compacted) bytes, contents scratch
 * Products and sums are fp32 (16-bit inputs are exact in fp32): an output element differs from the exact value
 * by about 1e-6 of the largest magnitude in its head's output row (an element near zero is a difference of
 * large terms, so the error is relative to the row, not to the element); lse to about 1e-6 absolute.
 * Asynchronous on `stream`; two launches; no allocation.  Errors as for chunkkv_score.                  */
size_t chunkkv_decode_workspace_bytes(const chunkkv_problem *prob, int32_t compacted);
int chunkkv_decode_attention(const chunkkv_problem *prob, int32_t compacted, const int32_t *kv_len, const void *q,
                             const void *k, const void *v, float *out, float *lse, void *workspace,
                             size_t workspace_bytes, void *stream);

/* Quality of one compressed layer against the full one: the two diagnostics Appendix A.1 tabulates per
 * layer.  The paper names them without formulas; this library computes
 *   l1_loss[b]     = sum |X - X~| / sum |X| over all K and V entries of sequence b, X~ being the cache with the
 *                    dropped tokens zeroed: the share of the cache's absolute mass held by dropped tokens
 *                    (0 when everything is kept);
 *   attn_cos[b][i] = cosine between the attention distribution of decoding query i over all L tokens and its
 *                    distribution over the kept tokens (placed at their positions, zero elsewhere);
 *                    average over i for the per-layer figure.
 * Inputs are a layer's full cache and the output chunkkv_compact / chunkkv_compress_stack wrote for it.
 *   kv_len     NULL, or as in chunkkv_decode_attention (whole-chunk mode: sel_count-derived token counts)
 *   q          device [B][Hq][d], the decoding query
 *   k, v       the full cache (kv_* geometry); k_out, v_out the compacted cache (out_* geometry)
 *   l1_loss    device float [B]; attn_cos device float [B][Hq]
 *   workspace  chunkkv_quality_workspace_bytes(prob) bytes (0 = invalid problem)
 * Cost: both caches are read twice (once by decode attention at twice the softmax scale, whose log-sum-exps
 * give the cosine, once by the absolute-mass reduction).  Errors as for chunkkv_decode_attention.            */
size_t chunkkv_quality_workspace_bytes(const chunkkv_problem *prob);
int chunkkv_quality_metrics(const chunkkv_problem *prob, const int32_t *kv_len, const void *q, const void *k,
                            const void *v, const void *k_out, const void *v_out, float *l1_loss, float *attn_cos,
                            void *workspace, size_t workspace_bytes, void *stream);

/* chunkkv_decode_attention for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, results and
 * errors as chunkkv_decode_attention, without the workspace: the partial results of the key ranges live in a
 * device-resident array of CHUNKKV_STATIC_SCRATCH_BYTES that is part of the library image (every GPU the
 * library runs on holds it until the process ends).  The call allocates nothing and frees nothing.
 *   - a problem whose chunkkv_decode_workspace_bytes() exceeds CHUNKKV_STATIC_SCRATCH_BYTES is refused with
 *     CHUNKKV_ERR_WORKSPACE and nothing is enqueued (8 MiB covers 32 query heads over a 128K-token cache and
 *     8 sequences x 28 query heads of up to 64K tokens);
 *   - all calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two streams, two
 *     threads) race on it; calls on one stream are ordered and safe;
 *   - the first call on a device looks up the array's device address (no allocation).                      */
#define CHUNKKV_STATIC_SCRATCH_BYTES (8u << 20)
int chunkkv_decode_attention_static(const chunkkv_problem *prob, int32_t compacted, const int32_t *kv_len,
                                    const void *q, const void *k, const void *v, float *out, float *lse,
                                    void *stream);

/* Scoring has two implementations with the same results (to rounding; both keep logits, exponentials and sums in
 * fp32): a single pass over K (bf16 and fp16 caches of head_dim 128, 65 to 256 window rows per kv-head, chunk
 * sizes 5, 10 and 20; not used when token_importance is requested) and a general two-pass one.
 * CHUNKKV_FLAG_TWO_PASS in chunkkv_problem.flags selects the two-pass kernels for a call.                     */

/* Measurement aid (the per-kernel durations the roofline figures need; Algorithm 2's T_compress and
 * T_select are the scoring+selection and the gather durations).  Between begin and end every kernel
 * the calls above launch is bracketed by a HIP event pair on its stream (up to max_records launches).
 * chunkkv_timing_end waits for those events and returns, per kernel kind, the summed duration in
 * milliseconds and the number of launches:
 *   0 score pass 0 (softmax statistics) or the single-pass kernel   1 statistics merge
 *   2 score pass 1 (importance, chunk sums) or the single-pass row reduction
 *   3 chunk sums for c larger than a key tile   4 chunk selection   5 compaction   6 decode attention
 * total_ms and launches are host arrays of CHUNKKV_TIMING_KINDS entries.  Process-wide and not thread-safe:
 * one measurement at a time, no compression calls from other threads meanwhile.  It changes no result.   */
#define CHUNKKV_TIMING_KINDS 7
int chunkkv_timing_begin(int32_t max_records);
int chunkkv_timing_end(double *total_ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* CHUNKKV_H */
