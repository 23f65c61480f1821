// Internal declarations shared by the translation units of libchunkkv (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "chunkkv.h"

namespace ckv {

constexpr int kMaxLayersPerLaunch = 32;  // pointer tables travel as kernel arguments
constexpr int kMaxBatchPerLaunch = 16;
constexpr int kTileBytes = 16384;        // one K tile staged in LDS (ring slot)
constexpr int kSuperKeys = 256;        // keys per importance / chunk-sum step of pass 1 (several tiles)
constexpr int kThreads = 256;            // 4 wavefronts of 64
constexpr int kMaxRows = 512;            // g * w limit
constexpr int kCompactEntries = 16;      // selection entries per compaction workgroup

// Per-sequence metadata of one launch slice (<= kMaxBatchPerLaunch sequences).
struct SeqTable {
  int32_t seqlen[kMaxBatchPerLaunch];
  int32_t n_keep[kMaxBatchPerLaunch];
  int64_t kv_base[kMaxBatchPerLaunch];
  int64_t out_base[kMaxBatchPerLaunch];
};

// Arguments of the two scoring passes.  "problem" = (leader layer, sequence, kv-head).
// Arrays indexed by problem use the FULL batch (batch_total) so slices address the same buffers.
struct ScoreArgs {
  const void *q[kMaxLayersPerLaunch];
  const void *k[kMaxLayersPerLaunch];
  SeqTable seq;
  int32_t leader0;         // index of this slice's first leader layer
  int32_t batch0;          // index of this slice's first sequence
  int32_t batch_total;
  int32_t n_q_heads, n_kv_heads, window, chunk;
  int64_t kv_stride_head, kv_stride_tok;
  float scale_log2e;       // softmax scale * log2(e)
  int32_t tiles_per_wg;    // pass 0: key tiles, pass 1: super-tiles (kSuperKeys) each workgroup walks
  int32_t max_split;       // pitch of part_stats in splits
  int32_t rows_pad;        // g*w rounded up to 32
  float2 *part_stats;      // [problem][max_split][rows_pad]  (running max, sum) in log2 units
  float *refs;             // [problem][rows_pad]  max + log2(sum)
  float *chunk_scores;     // [leader][batch_total][Hkv][score_cap]
  int32_t score_cap;
  float *token_imp;        // [leader][batch_total][Hkv][imp_pitch] or null
  int64_t imp_pitch;
  int32_t fuse_chunks;     // pass 1: 1 = super-tiles hold whole chunks and chunk sums are written
  // single-pass path (score_single.h): key ranges are single_periods_per_range() whole periods of 160 keys
  int32_t n_periods;       // pitch of e_buf / m_period: max over sequences of ceil(L / 160)
  void *e_buf;             // [problem][n_periods][rows_pad][2 lane halves][80 / c] x 3 bytes: per-(chunk, row) sums of e
  float *m_period;         // [problem][n_periods][rows_pad]  reference those sums are relative to
};

// Caller-supplied row log-sum-exps -> row references of the importance pass.
struct LseArgs {
  const float *lse[kMaxLayersPerLaunch];  // per leader layer: [batch_total][Hq][w], natural log
  float *refs;                            // [problem][rows_pad], log2 units
  int32_t leader0, batch0, batch_total;
  int32_t n_q_heads, n_kv_heads, window, rows_pad;
};

struct TopkArgs {
  SeqTable seq;
  int32_t group0;             // first selection group of this launch
  int32_t batch0, batch_total, n_kv_heads, window, chunk;
  const float *chunk_scores;  // [group][batch_total][Hkv][score_cap]
  int32_t score_cap, sel_cap;
  int32_t *sel_chunk, *sel_len, *sel_count;
  int32_t *sel_off;           // [group][batch_total][Hkv][sel_cap] exclusive token offsets, or null
  int32_t whole_chunks;       // 1: Algorithm 3 as printed: floor(n_keep / c) whole chunks, nothing is cut
};

struct CompactArgs {
  const void *k[kMaxLayersPerLaunch];
  const void *v[kMaxLayersPerLaunch];
  void *k_out[kMaxLayersPerLaunch];
  void *v_out[kMaxLayersPerLaunch];
  SeqTable seq;
  int32_t layer0, reuse;      // selection group of slice layer z is (layer0 + z) / reuse
  int32_t batch0, batch_total, n_kv_heads, window, chunk;
  int32_t elem_bytes;
  int64_t kv_stride_head, kv_stride_tok, out_stride_head, out_stride_tok;
  const int32_t *sel_chunk, *sel_len, *sel_count, *sel_off;  // sel_off may be null
  int32_t sel_cap;
  int32_t whole_chunks;       // 1: the window follows the kept tokens directly (their count varies per head)
};

// Decode attention over one layer's cache (decode.hip).  Per-head partial results use the FULL batch index.
struct DecodeArgs {
  const void *q, *k, *v;
  float *out, *lse;           // [batch_total][Hq][d], [batch_total][Hq] or null
  float2 *part_ml;            // [batch_total * Hq][n_split]  (max in log2 units, sum)
  float *part_o;              // [batch_total * Hq][n_split][d]
  const int32_t *kv_len;      // [batch_total][Hkv] tokens to attend to, or null (= n_tok)
  int32_t n_tok[kMaxBatchPerLaunch];  // tokens the cache of a sequence holds per head
  int64_t base[kMaxBatchPerLaunch];   // element offset of the sequence in k / v
  int64_t stride_head, stride_tok;
  int32_t batch0, n_q_heads, n_kv_heads;
  float scale_log2e;
  int32_t n_split, rows_per_split;
};

// Absolute mass of one layer's cache (quality.hip): sum of |K| + |V| over blocks of rows of every (sequence, kv-head).
struct AbsSumArgs {
  const void *k, *v;
  float *partial;             // [batch_total][Hkv][n_blocks]; blocks past a head's rows hold 0
  const int32_t *kv_len;      // as in DecodeArgs
  int32_t n_tok[kMaxBatchPerLaunch];
  int64_t base[kMaxBatchPerLaunch];
  int64_t stride_head, stride_tok;
  int32_t batch0, n_kv_heads, head_dim, n_blocks;
};

struct QualityFinishArgs {
  const float *partial_full, *partial_kept;   // [B][Hkv][blocks_full], [B][Hkv][blocks_kept]
  const float *lse_full, *lse_kept;           // [B][Hq]: decode log-sum-exps at twice the softmax scale
  float *l1_loss, *attn_cos;                  // [B], [B][Hq]
  int32_t n_q_heads, n_kv_heads, blocks_full, blocks_kept;
};

// query heads of one kv-head that a decode workgroup serves: 1, 2, 4 or 8 (fp32 caches: at most 4, registers)
inline int decode_heads_per_wg(int dtype, int g) {
  const int G = g > 4 ? 8 : (g > 2 ? 4 : g);  // 5..7 heads: one padded batch of 8, not two passes over K and V
  return dtype == CHUNKKV_F32 && G > 4 ? 4 : G;
}

// Reads element i of a small table that travels as a kernel argument.  A chain of selects on the
// (wavefront-uniform) index keeps the table in scalar registers; a dynamic subscript would make the
// compiler copy the whole argument struct to scratch memory first.
template <typename T, int N>
__device__ __forceinline__ T pick(const T (&arr)[N], int i) {
  T r = arr[0];
#pragma unroll
  for (int j = 1; j < N; ++j) r = (i == j) ? arr[j] : r;
  return r;
}

// Single-pass scoring: periods (160 keys) one workgroup walks, for a sequence of n_periods periods.  A function
// of the sequence alone (about 32 ranges per sequence and kv-head, at least 8 periods each), so the key ranges,
// and with them every rounding of a score, do not depend on how many layers or sequences share a launch.
__host__ __device__ inline int single_periods_per_range(int n_periods) {
  const int p = (n_periods + 31) / 32;
  return p < 8 ? 8 : p;
}

// Geometry of the scoring kernels for one (dtype, head_dim, row count).
struct ScoreGeom {
  int row_bytes;   // head_dim * sizeof(element)
  int tile_keys;   // keys per LDS tile
  int nq_blocks;   // 32-row blocks of window rows (padded)
  int nqw;         // blocks held by one wavefront
  int wq;          // wavefronts splitting the rows (the other 4/wq split keys)
};
inline int elem_bytes(int dtype) { return dtype == CHUNKKV_F32 ? 4 : 2; }  // bf16 and fp16: 2
bool score_geometry(int dtype, int head_dim, int rows, ScoreGeom *g);

// Launchers (each checks hipGetLastError and returns a chunkkv_status).
int launch_score_pass(int pass, int dtype, int head_dim, const ScoreGeom &g, const ScoreArgs &a,
                      dim3 grid, hipStream_t s);
int launch_stats_combine(const ScoreArgs &a, int n_leaders_slice, int batch_slice, int tile_keys,
                         hipStream_t s);
int launch_chunk_sums(const ScoreArgs &a, int n_leaders_slice, int batch_slice, hipStream_t s);
int launch_score_single(int dtype, const ScoreArgs &a, dim3 grid, hipStream_t s);
int launch_jaccard(const int32_t *sel_chunk, const int32_t *sel_len, const int32_t *sel_count, int sel_cap, int chunk,
                   int rows_per_group, int n_pairs, float *out, hipStream_t s);
int launch_lse_refs(const LseArgs &a, int n_leaders_slice, int batch_slice, hipStream_t s);
int launch_single_scores(const ScoreArgs &a, int n_leaders_slice, int batch_slice, hipStream_t s);
bool single_pass_ok(int dtype, int head_dim, int rows, int chunk);
int launch_topk(const TopkArgs &a, int n_groups, int batch_slice, hipStream_t s);
int launch_decode(int dtype, int head_dim, const DecodeArgs &a, int batch_slice, hipStream_t s);
int abs_sum_blocks(int n_tok_max);
int launch_abs_sum(int dtype, const AbsSumArgs &a, int batch_slice, hipStream_t s);
int launch_quality_finish(const QualityFinishArgs &a, int batch, hipStream_t s);
int launch_compact(int row_bytes, const CompactArgs &a, int n_layers_slice, int batch_slice,
                   int max_entries, hipStream_t s);

}  // namespace ckv
