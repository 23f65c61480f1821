// Host side of libchunkkv: argument checks, workspace plan and launch sequence of the four C-ABI calls.
#include <math.h>
#include <string.h>

#include <mutex>

#include "internal.h"

namespace ckv {
namespace {

constexpr int kTargetWorkgroups = 4096;  // ~4 resident rounds of 2 workgroups on each of 256 CUs
constexpr int kSinglePeriodKeys = 160;   // granule of the single-pass kernel's key ranges
// Key tiles (16 KB) one scoring launch set should hold.  Measured on MI355X: every extra dependent launch
// costs ~30 us of idle GPU, more than splitting the stack into sets wins back, so one set it is.
constexpr int64_t kTilesPerLaunch = 1 << 30;

struct Plan {
  ScoreGeom geom;
  int n_leaders, rows_pad;
  int batch_leaders;  // leader layers scored per launch set (the unit that overlaps with compaction)
  int tpw0, tpw1, max_split0;
  int fuse_chunks;
  // single-pass path: usable for this problem?  geometry and workspace
  int single_ok, rows_pad_s, n_periods, max_split_s;
  size_t off_part, off_refs, off_scores, off_seloff, off_imp, off_ebuf, off_mper, total;
};

// ---- optional per-kernel timing (chunkkv_timing_begin / chunkkv_timing_end) -----------------------
enum Kind { kStats = 0, kCombine, kColsum, kChunkSums, kTopk, kCompact, kDecode, kKinds };
static_assert(kKinds == CHUNKKV_TIMING_KINDS, "timing kinds of the header");
struct Timing {
  bool on = false;
  int cap = 0, used = 0;
  hipEvent_t *ev = nullptr;  // 2 per record
  int *kind = nullptr;
} g_timing;

struct Timed {  // records an event pair around one launch when timing is on
  hipStream_t s;
  int slot = -1;
  Timed(int kind, hipStream_t stream) : s(stream) {
    if (g_timing.on && g_timing.used < g_timing.cap) {
      slot = g_timing.used++;
      g_timing.kind[slot] = kind;
      (void)hipEventRecord(g_timing.ev[2 * slot], s);
    }
  }
  ~Timed() {
    if (slot >= 0) (void)hipEventRecord(g_timing.ev[2 * slot + 1], s);
  }
};

// ---- device-resident scratch for chunkkv_decode_attention_static ---------------------------------
// One array per GPU the library runs on, held until the process ends.  Its name is only a host-side
// stand-in: the device address is looked up once per device and kept; host code uses that pointer.
constexpr size_t kStaticScratchBytes = CHUNKKV_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
}  // namespace
}  // namespace ckv
static __device__ __align__(256) unsigned char scratch[ckv::kStaticScratchBytes];
namespace ckv {
namespace {
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};
// device address of `scratch` on the current device (looked up on the first call per device)
int static_scratch(void **out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return CHUNKKV_ERR_LAUNCH;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return CHUNKKV_ERR_LAUNCH;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CHUNKKV_OK;
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

int check_problem(const chunkkv_problem *p, bool need_out) {
  if (!p) return CHUNKKV_ERR_NULL;
  if (!p->seqlen || !p->n_keep || !p->kv_base) return CHUNKKV_ERR_NULL;
  if (need_out && !p->out_base) return CHUNKKV_ERR_NULL;
  if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->window < 1 || p->chunk < 1)
    return CHUNKKV_ERR_SHAPE;
  if (p->n_q_heads % p->n_kv_heads != 0) return CHUNKKV_ERR_SHAPE;
  if (!(p->softmax_scale >= 0.f) || isinf(p->softmax_scale)) return CHUNKKV_ERR_SHAPE;
  if (p->dtype != CHUNKKV_F32 && p->dtype != CHUNKKV_BF16 && p->dtype != CHUNKKV_F16) return CHUNKKV_ERR_UNSUPPORTED;
  if (p->flags & ~(uint32_t)(CHUNKKV_FLAG_WHOLE_CHUNKS | CHUNKKV_FLAG_TWO_PASS)) return CHUNKKV_ERR_UNSUPPORTED;
  if (p->head_dim != 64 && p->head_dim != 128) return CHUNKKV_ERR_UNSUPPORTED;
  const int64_t rows = (int64_t)(p->n_q_heads / p->n_kv_heads) * p->window;
  ScoreGeom g;
  if (rows > kMaxRows || !score_geometry(p->dtype, p->head_dim, (int)rows, &g)) return CHUNKKV_ERR_UNSUPPORTED;
  const int esz = elem_bytes(p->dtype);
  if (p->kv_stride_tok < p->head_dim || p->kv_stride_head < 0) return CHUNKKV_ERR_SHAPE;
  if ((p->kv_stride_tok * esz) % 16 || (p->kv_stride_head * esz) % 16) return CHUNKKV_ERR_SHAPE;
  if (p->kv_stride_tok * esz > (1 << 22)) return CHUNKKV_ERR_UNSUPPORTED;  // tile offsets are 32-bit
  if (need_out) {
    if (p->out_stride_tok < p->head_dim || p->out_stride_head < 0) return CHUNKKV_ERR_SHAPE;
    if ((p->out_stride_tok * esz) % 16 || (p->out_stride_head * esz) % 16) return CHUNKKV_ERR_SHAPE;
  }
  if (p->sel_cap < 1 || p->score_cap < 0) return CHUNKKV_ERR_SHAPE;
  for (int b = 0; b < p->batch; ++b) {
    const int64_t L = p->seqlen[b], nk = p->n_keep[b];
    if (L < p->window || nk < 0 || nk > L - p->window) return CHUNKKV_ERR_SHAPE;
    if (p->kv_base[b] < 0 || (p->kv_base[b] * esz) % 16) return CHUNKKV_ERR_SHAPE;
    // the scoring kernels address the K rows of one (sequence, kv-head) through a buffer descriptor with
    // 32-bit byte offsets (one tile of slack past the end)
    if (((int64_t)L + 256) * p->kv_stride_tok * esz >= (int64_t)1 << 31) return CHUNKKV_ERR_UNSUPPORTED;
    if (need_out && (p->out_base[b] < 0 || (p->out_base[b] * esz) % 16)) return CHUNKKV_ERR_SHAPE;
    if (p->sel_cap < (nk + p->chunk - 1) / p->chunk + 1) return CHUNKKV_ERR_SHAPE;
    if (p->score_cap < (L - p->window + p->chunk - 1) / p->chunk) return CHUNKKV_ERR_SHAPE;
  }
  return CHUNKKV_OK;
}

bool misaligned(const void *p) { return ((uintptr_t)p & 15) != 0; }

// Key-range split and workspace of the decode-attention call: a pure function of the problem.  About
// kDecodeTargetWorkgroups working workgroups per launch, never fewer than kDecodeMinRows rows per range.
constexpr int kDecodeTargetWorkgroups = 1024;
constexpr int kDecodeMinRows = 256;
struct DecodePlan {
  int n_split, rows_per_split;
  size_t off_ml, off_o, total;
};
int decode_plan(const chunkkv_problem *p, bool compacted, DecodePlan *pl) {
  int64_t n_max = 1, n_sum = 0;
  for (int b = 0; b < p->batch; ++b) {
    const int64_t n = compacted ? (int64_t)p->n_keep[b] + p->window : p->seqlen[b];
    n_max = n > n_max ? n : n_max;
    n_sum += n;
  }
  const int g = p->n_q_heads / p->n_kv_heads;
  const int G = decode_heads_per_wg(p->dtype, g), nz = (g + G - 1) / G;
  // every sequence is cut into ranges of the same length, chosen so that all sequences together give about
  // kDecodeTargetWorkgroups workgroups with rows to read (short sequences then use only the first ranges of the grid)
  const int64_t launches = (p->batch + kMaxBatchPerLaunch - 1) / kMaxBatchPerLaunch;
  int64_t rows = (n_sum * p->n_kv_heads * nz / launches + kDecodeTargetWorkgroups - 1) / kDecodeTargetWorkgroups;
  rows = rows < kDecodeMinRows ? kDecodeMinRows : rows;
  rows = (rows + 127) / 128 * 128;
  const int64_t n_split = (n_max + rows - 1) / rows;
  pl->n_split = (int)n_split;
  pl->rows_per_split = (int)rows;
  const size_t heads = (size_t)p->batch * p->n_q_heads;
  pl->off_ml = 0;
  pl->off_o = align256(heads * n_split * sizeof(float2));
  pl->total = pl->off_o + align256(heads * n_split * p->head_dim * sizeof(float));
  return CHUNKKV_OK;
}

// Workspace layout and key-range split; a pure function of (problem, n_layers, reuse).
int make_plan(const chunkkv_problem *p, int n_layers, int reuse, Plan *pl) {
  if (n_layers < 1 || reuse < 1) return CHUNKKV_ERR_SHAPE;
  const int rows = (p->n_q_heads / p->n_kv_heads) * p->window;
  if (!score_geometry(p->dtype, p->head_dim, rows, &pl->geom)) return CHUNKKV_ERR_UNSUPPORTED;
  pl->n_leaders = ceil_div(n_layers, reuse);
  pl->rows_pad = pl->geom.nqw * pl->geom.wq * 32;
  const int TK = pl->geom.tile_keys;
  pl->fuse_chunks = p->chunk <= kSuperKeys;
  const int stride1 = pl->fuse_chunks ? (kSuperKeys / p->chunk) * p->chunk : kSuperKeys;
  int64_t tiles0 = 0, tiles1 = 0;
  for (int b = 0; b < p->batch; ++b) {
    tiles0 += ceil_div(p->seqlen[b], TK);
    tiles1 += ceil_div(p->seqlen[b] - p->window, stride1);
  }
  // leader layers per launch set: enough key tiles (~kTilesPerLaunch) to amortise workgroup start-up,
  // few enough that compaction of one set overlaps scoring of the next; sets are balanced in size
  int64_t per_leader = tiles0 * p->n_kv_heads;
  int gb = (int)((kTilesPerLaunch + per_leader - 1) / (per_leader > 0 ? per_leader : 1));
  if (gb < 1) gb = 1;
  if (gb > pl->n_leaders) gb = pl->n_leaders;
  if (gb > kMaxLayersPerLaunch) gb = kMaxLayersPerLaunch;
  const int nsets = ceil_div(pl->n_leaders, gb);
  pl->batch_leaders = ceil_div(pl->n_leaders, nsets);
  const int64_t heads = (int64_t)pl->batch_leaders * p->n_kv_heads;
  pl->tpw0 = (int)((tiles0 * heads + kTargetWorkgroups - 1) / kTargetWorkgroups);
  pl->tpw1 = (int)((tiles1 * heads + kTargetWorkgroups - 1) / kTargetWorkgroups);
  if (pl->tpw0 < 1) pl->tpw0 = 1;
  if (pl->tpw1 < 1) pl->tpw1 = 1;
  pl->max_split0 = 1;
  for (int b = 0; b < p->batch; ++b) {
    const int s = ceil_div(ceil_div(p->seqlen[b], TK), pl->tpw0);
    if (s > pl->max_split0) pl->max_split0 = s;
  }
  // single-pass path
  pl->single_ok = single_pass_ok(p->dtype, p->head_dim, rows, p->chunk) ? 1 : 0;
  pl->rows_pad_s = rows > 128 ? 256 : 128;
  pl->n_periods = 0;
  pl->max_split_s = 1;
  if (pl->single_ok) {
    for (int b = 0; b < p->batch; ++b) {
      const int np = ceil_div(p->seqlen[b], kSinglePeriodKeys);
      if (np > pl->n_periods) pl->n_periods = np;
    }
    // the kernels address E of one problem with 32-bit byte offsets
    if ((int64_t)pl->n_periods * pl->rows_pad_s * 80 >= (int64_t)1 << 32) pl->single_ok = 0;
    // key ranges: single_periods_per_range() periods each, a function of the sequence alone
    for (int b = 0; b < p->batch; ++b) {
      const int np = ceil_div(p->seqlen[b], kSinglePeriodKeys);
      const int sp = ceil_div(np, single_periods_per_range(np));
      if (sp > pl->max_split_s) pl->max_split_s = sp;
    }
  }
  const size_t problems = (size_t)pl->n_leaders * p->batch * p->n_kv_heads;
  size_t part_bytes = problems * pl->max_split0 * pl->rows_pad * sizeof(float2);
  if (pl->single_ok) {
    const size_t pb = problems * pl->max_split_s * pl->rows_pad_s * sizeof(float2);
    part_bytes = pb > part_bytes ? pb : part_bytes;
  }
  size_t off = 0;
  pl->off_part = off;   off += align256(part_bytes);
  pl->off_refs = off;   off += align256(problems * pl->rows_pad * sizeof(float));
  pl->off_scores = off; off += align256(problems * (size_t)p->score_cap * sizeof(float));
  pl->off_seloff = off; off += align256(problems * (size_t)p->sel_cap * sizeof(int32_t));
  pl->off_imp = off;
  if (!pl->fuse_chunks) off += align256(problems * (size_t)p->score_cap * p->chunk * sizeof(float));
  pl->off_ebuf = pl->off_mper = off;
  if (pl->single_ok) {
    const size_t cells = problems * (size_t)pl->n_periods * pl->rows_pad_s;   // (period, row)
    const int sums = 80 / p->chunk;   // chunk sums per lane half and period: 20-bit floats in groups of eight, else 24-bit
    pl->off_ebuf = off; off += align256(cells * (size_t)(sums == 4 ? 24 : 5 * sums));
    pl->off_mper = off; off += align256(cells * sizeof(float));
  }
  pl->total = off < 256 ? 256 : off;
  return CHUNKKV_OK;
}

void fill_seq(SeqTable *t, const chunkkv_problem *p, int b0, int nb) {
  memset(t, 0, sizeof(*t));
  for (int i = 0; i < nb; ++i) {
    t->seqlen[i] = p->seqlen[b0 + i];
    t->n_keep[i] = p->n_keep[b0 + i];
    t->kv_base[i] = p->kv_base[b0 + i];
    t->out_base[i] = p->out_base ? p->out_base[b0 + i] : 0;
  }
}

// Scores leader layers [g0, g0+ng) (pointer tables already gathered) for all sequences.
// lse == nullptr: the row normalisation is computed here; otherwise lse[i] is leader i's caller-supplied
// [B][Hq][w] array and only the importance pass runs.
int run_score(const chunkkv_problem *p, const Plan &pl, const void *const *q, const void *const *k,
              const float *const *lse, int ng, int leader0, float *chunk_scores, float *token_imp,
              int64_t imp_pitch, char *ws, hipStream_t s) {
  const int TK = pl.geom.tile_keys;
  for (int b0 = 0; b0 < p->batch; b0 += kMaxBatchPerLaunch) {
    const int nb = p->batch - b0 < kMaxBatchPerLaunch ? p->batch - b0 : kMaxBatchPerLaunch;
    ScoreArgs a;
    memset(&a, 0, sizeof(a));
    for (int i = 0; i < ng; ++i) { a.q[i] = q[i]; a.k[i] = k[i]; }
    fill_seq(&a.seq, p, b0, nb);
    a.leader0 = leader0; a.batch0 = b0; a.batch_total = p->batch;
    a.n_q_heads = p->n_q_heads; a.n_kv_heads = p->n_kv_heads; a.window = p->window; a.chunk = p->chunk;
    a.kv_stride_head = p->kv_stride_head; a.kv_stride_tok = p->kv_stride_tok;
    const float scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->head_dim);
    a.scale_log2e = scale * 1.4426950408889634f;
    a.max_split = pl.max_split0; a.rows_pad = pl.rows_pad;
    a.part_stats = (float2 *)(ws + pl.off_part);
    a.refs = (float *)(ws + pl.off_refs);
    a.chunk_scores = chunk_scores; a.score_cap = p->score_cap;
    a.token_imp = token_imp; a.imp_pitch = imp_pitch;
    a.fuse_chunks = pl.fuse_chunks;
    if (!pl.fuse_chunks && !token_imp) { a.token_imp = (float *)(ws + pl.off_imp); a.imp_pitch = (int64_t)p->score_cap * p->chunk; }
    int split0 = 1, split1 = 0;
    const int stride1 = pl.fuse_chunks ? (kSuperKeys / p->chunk) * p->chunk : kSuperKeys;
    for (int i = 0; i < nb; ++i) {
      const int s0 = ceil_div(ceil_div(a.seq.seqlen[i], TK), pl.tpw0);
      const int s1 = ceil_div(ceil_div(a.seq.seqlen[i] - p->window, stride1), pl.tpw1);
      split0 = s0 > split0 ? s0 : split0;
      split1 = s1 > split1 ? s1 : split1;
    }
    int rc;
    if (lse) {
      LseArgs la;
      memset(&la, 0, sizeof(la));
      for (int i = 0; i < ng; ++i) la.lse[i] = lse[i];
      la.refs = a.refs; la.leader0 = leader0; la.batch0 = b0; la.batch_total = p->batch;
      la.n_q_heads = p->n_q_heads; la.n_kv_heads = p->n_kv_heads; la.window = p->window; la.rows_pad = pl.rows_pad;
      { Timed t(kCombine, s); rc = launch_lse_refs(la, ng, nb, s); }
      if (rc) return rc;
    } else if (pl.single_ok && !(p->flags & CHUNKKV_FLAG_TWO_PASS) && !token_imp) {
      // one pass over K: per-(chunk, row) sums and the references they are relative to; then the merge of the
      // range statistics and the weighted row sum in one small kernel
      a.n_periods = pl.n_periods;
      a.e_buf = ws + pl.off_ebuf;
      a.m_period = (float *)(ws + pl.off_mper);
      a.max_split = pl.max_split_s;
      a.rows_pad = pl.rows_pad_s;
      int splits = 1;
      for (int i = 0; i < nb; ++i) {
        const int np = ceil_div(a.seq.seqlen[i], kSinglePeriodKeys);
        const int sp = ceil_div(np, single_periods_per_range(np));
        splits = sp > splits ? sp : splits;
      }
      { Timed t(kStats, s); rc = launch_score_single(p->dtype, a, dim3(splits, nb * p->n_kv_heads, ng), s); }
      if (rc) return rc;
      { Timed t(kColsum, s); rc = launch_single_scores(a, ng, nb, s); }
      if (rc) return rc;
      continue;
    }
    if (!lse) {
      a.tiles_per_wg = pl.tpw0;
      { Timed t(kStats, s); rc = launch_score_pass(0, p->dtype, p->head_dim, pl.geom, a, dim3(split0, nb * p->n_kv_heads, ng), s); }
      if (rc) return rc;
      { Timed t(kCombine, s); rc = launch_stats_combine(a, ng, nb, TK, s); }
      if (rc) return rc;
    }
    a.tiles_per_wg = pl.tpw1;
    { Timed t(kColsum, s); rc = launch_score_pass(1, p->dtype, p->head_dim, pl.geom, a, dim3(split1, nb * p->n_kv_heads, ng), s); }
    if (rc) return rc;
    if (!pl.fuse_chunks) {
      { Timed t(kChunkSums, s); rc = launch_chunk_sums(a, ng, nb, s); }
      if (rc) return rc;
    }
  }
  return CHUNKKV_OK;
}

int run_topk(const chunkkv_problem *p, const float *chunk_scores, int group0, int n_groups, int32_t *sel_chunk,
             int32_t *sel_len, int32_t *sel_count, int32_t *sel_off, hipStream_t s) {
  for (int b0 = 0; b0 < p->batch; b0 += kMaxBatchPerLaunch) {
    const int nb = p->batch - b0 < kMaxBatchPerLaunch ? p->batch - b0 : kMaxBatchPerLaunch;
    TopkArgs a;
    memset(&a, 0, sizeof(a));
    fill_seq(&a.seq, p, b0, nb);
    a.group0 = group0;
    a.batch0 = b0; a.batch_total = p->batch; a.n_kv_heads = p->n_kv_heads; a.window = p->window; a.chunk = p->chunk;
    a.chunk_scores = chunk_scores; a.score_cap = p->score_cap; a.sel_cap = p->sel_cap;
    a.sel_chunk = sel_chunk; a.sel_len = sel_len; a.sel_count = sel_count; a.sel_off = sel_off;
    a.whole_chunks = (p->flags & CHUNKKV_FLAG_WHOLE_CHUNKS) ? 1 : 0;
    int rc;
    { Timed t(kTopk, s); rc = launch_topk(a, n_groups, nb, s); }
    if (rc) return rc;
  }
  return CHUNKKV_OK;
}

int run_compact(const chunkkv_problem *p, int l_begin, int n_layers, int reuse, const void *const *k, const void *const *v,
                void *const *k_out, void *const *v_out, const int32_t *sel_chunk, const int32_t *sel_len,
                const int32_t *sel_count, const int32_t *sel_off, hipStream_t s) {
  const int esz = elem_bytes(p->dtype);
  for (int l0 = l_begin; l0 < n_layers; l0 += kMaxLayersPerLaunch) {
    const int nl = n_layers - l0 < kMaxLayersPerLaunch ? n_layers - l0 : kMaxLayersPerLaunch;
    for (int b0 = 0; b0 < p->batch; b0 += kMaxBatchPerLaunch) {
      const int nb = p->batch - b0 < kMaxBatchPerLaunch ? p->batch - b0 : kMaxBatchPerLaunch;
      CompactArgs a;
      memset(&a, 0, sizeof(a));
      for (int i = 0; i < nl; ++i) {
        a.k[i] = k[l0 + i]; a.v[i] = v[l0 + i]; a.k_out[i] = k_out[l0 + i]; a.v_out[i] = v_out[l0 + i];
      }
      fill_seq(&a.seq, p, b0, nb);
      a.layer0 = l0; a.reuse = reuse; a.batch0 = b0; a.batch_total = p->batch;
      a.n_kv_heads = p->n_kv_heads; a.window = p->window; a.chunk = p->chunk; a.elem_bytes = esz;
      a.kv_stride_head = p->kv_stride_head; a.kv_stride_tok = p->kv_stride_tok;
      a.out_stride_head = p->out_stride_head; a.out_stride_tok = p->out_stride_tok;
      a.sel_chunk = sel_chunk; a.sel_len = sel_len; a.sel_count = sel_count; a.sel_off = sel_off;
      a.sel_cap = p->sel_cap;
      a.whole_chunks = (p->flags & CHUNKKV_FLAG_WHOLE_CHUNKS) ? 1 : 0;
      int max_entries = 0;
      for (int i = 0; i < nb; ++i) {
        const int nk = a.seq.n_keep[i];
        int e = (nk > 0 ? ceil_div(nk, p->chunk) + 1 : 0) + ceil_div(p->window, p->chunk);
        if (nk > 0 && e - ceil_div(p->window, p->chunk) > p->sel_cap) e = p->sel_cap + ceil_div(p->window, p->chunk);
        max_entries = e > max_entries ? e : max_entries;
      }
      int rc;
      { Timed t(kCompact, s); rc = launch_compact(p->head_dim * esz, a, nl, nb, max_entries, s); }
      if (rc) return rc;
    }
  }
  return CHUNKKV_OK;
}

}  // namespace
}  // namespace ckv

using namespace ckv;

// Runs of consecutive reuse groups with one chunk size; fn(problem with that chunk, first group, end group).
template <typename F>
static int for_chunk_runs(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse, const int32_t *chunk_per_group,
                          F fn) {
  if (!prob) return CHUNKKV_ERR_NULL;
  if (!chunk_per_group) return CHUNKKV_ERR_NULL;
  if (n_layers < 1 || reuse < 1) return CHUNKKV_ERR_SHAPE;
  const int n_groups = ceil_div(n_layers, reuse);
  for (int g0 = 0; g0 < n_groups;) {
    int g1 = g0 + 1;
    while (g1 < n_groups && chunk_per_group[g1] == chunk_per_group[g0]) ++g1;
    chunkkv_problem run = *prob;
    run.chunk = chunk_per_group[g0];
    int rc = check_problem(&run, true);
    if (rc) return rc;
    rc = fn(run, g0, g1);
    if (rc) return rc;
    g0 = g1;
  }
  return CHUNKKV_OK;
}

extern "C" {

const char *chunkkv_status_string(int status) {
  switch (status) {
    case CHUNKKV_OK: return "ok";
    case CHUNKKV_ERR_NULL: return "a required pointer is NULL";
    case CHUNKKV_ERR_SHAPE: return "inconsistent shape, stride, alignment, budget or capacity";
    case CHUNKKV_ERR_UNSUPPORTED: return "unsupported dtype, head_dim or window rows per kv-head";
    case CHUNKKV_ERR_WORKSPACE: return "workspace too small or NULL";
    case CHUNKKV_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

size_t chunkkv_workspace_bytes(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse) {
  if (check_problem(prob, false) != CHUNKKV_OK) return 0;
  Plan pl;
  if (make_plan(prob, n_layers, reuse, &pl) != CHUNKKV_OK) return 0;
  return pl.total;
}

static int score_entry(const chunkkv_problem *prob, const void *q_obs, const void *k, const float *lse, bool with_lse,
                       float *chunk_scores, float *token_importance, void *workspace, size_t workspace_bytes,
                       void *stream) {
  int rc = check_problem(prob, false);
  if (rc) return rc;
  if (!q_obs || !k || !chunk_scores || (with_lse && !lse)) return CHUNKKV_ERR_NULL;
  if (misaligned(q_obs) || misaligned(k)) return CHUNKKV_ERR_SHAPE;
  Plan pl;
  rc = make_plan(prob, 1, 1, &pl);
  if (rc) return rc;
  if (!workspace || workspace_bytes < pl.total) return CHUNKKV_ERR_WORKSPACE;
  return run_score(prob, pl, &q_obs, &k, with_lse ? &lse : nullptr, 1, 0, chunk_scores, token_importance,
                   (int64_t)prob->score_cap * prob->chunk, (char *)workspace, (hipStream_t)stream);
}

int chunkkv_score(const chunkkv_problem *prob, const void *q_obs, const void *k, float *chunk_scores,
                  float *token_importance, void *workspace, size_t workspace_bytes, void *stream) {
  return score_entry(prob, q_obs, k, nullptr, false, chunk_scores, token_importance, workspace, workspace_bytes, stream);
}

int chunkkv_score_lse(const chunkkv_problem *prob, const void *q_obs, const void *k, const float *lse,
                      float *chunk_scores, float *token_importance, void *workspace, size_t workspace_bytes,
                      void *stream) {
  return score_entry(prob, q_obs, k, lse, true, chunk_scores, token_importance, workspace, workspace_bytes, stream);
}

int chunkkv_chunk_topk(const chunkkv_problem *prob, const float *chunk_scores, int32_t *sel_chunk,
                       int32_t *sel_len, int32_t *sel_count, void *workspace, size_t workspace_bytes,
                       void *stream) {
  (void)workspace; (void)workspace_bytes;  // the selection kernel keeps its state in LDS
  int rc = check_problem(prob, false);
  if (rc) return rc;
  if (!chunk_scores || !sel_chunk || !sel_len || !sel_count) return CHUNKKV_ERR_NULL;
  return run_topk(prob, chunk_scores, 0, 1, sel_chunk, sel_len, sel_count, nullptr, (hipStream_t)stream);
}

int chunkkv_compact(const chunkkv_problem *prob, const void *k, const void *v, const int32_t *sel_chunk,
                    const int32_t *sel_len, const int32_t *sel_count, void *k_out, void *v_out, void *stream) {
  int rc = check_problem(prob, true);
  if (rc) return rc;
  if (!k || !v || !sel_chunk || !sel_len || !sel_count || !k_out || !v_out) return CHUNKKV_ERR_NULL;
  if (misaligned(k) || misaligned(v) || misaligned(k_out) || misaligned(v_out)) return CHUNKKV_ERR_SHAPE;
  return run_compact(prob, 0, 1, 1, &k, &v, &k_out, &v_out, sel_chunk, sel_len, sel_count, nullptr,
                     (hipStream_t)stream);
}

static int check_stack_pointers(int32_t n_layers, int32_t reuse, const void *const *q_obs, const void *const *k,
                                const void *const *v, const float *const *lse, bool with_lse, void *const *k_out,
                                void *const *v_out, const int32_t *sel_chunk, const int32_t *sel_len,
                                const int32_t *sel_count) {
  if (n_layers < 1 || reuse < 1) return CHUNKKV_ERR_SHAPE;
  if (!q_obs || !k || !v || !k_out || !v_out || !sel_chunk || !sel_len || !sel_count) return CHUNKKV_ERR_NULL;
  if (with_lse && !lse) return CHUNKKV_ERR_NULL;
  for (int l = 0; l < n_layers; ++l) {
    if (!k[l] || !v[l] || !k_out[l] || !v_out[l]) return CHUNKKV_ERR_NULL;
    if (l % reuse == 0 && !q_obs[l]) return CHUNKKV_ERR_NULL;
    if (with_lse && l % reuse == 0 && !lse[l]) return CHUNKKV_ERR_NULL;
    if (misaligned(k[l]) || misaligned(v[l]) || misaligned(k_out[l]) || misaligned(v_out[l])) return CHUNKKV_ERR_SHAPE;
    if (l % reuse == 0 && misaligned(q_obs[l])) return CHUNKKV_ERR_SHAPE;
  }
  return CHUNKKV_OK;
}

// Algorithm 2 over the reuse groups [g_begin, g_end) of a stack of n_layers layers: leader layers (l % reuse == 0)
// are scored and selected, then every layer of these groups is gathered with the selection of its group.
// `pl` is the plan of the whole stack for prob->chunk.  Everything is enqueued on `s`.
static int stack_groups(const chunkkv_problem *prob, const Plan &pl, int g_begin, int g_end, int32_t n_layers,
                        int32_t reuse, const void *const *q_obs, const void *const *k, const void *const *v,
                        const float *const *lse, bool with_lse, void *const *k_out, void *const *v_out,
                        int32_t *sel_chunk, int32_t *sel_len, int32_t *sel_count, char *ws, hipStream_t s) {
  float *scores = (float *)(ws + pl.off_scores);
  int32_t *sel_off = (int32_t *)(ws + pl.off_seloff);
  for (int g0 = g_begin; g0 < g_end; g0 += pl.batch_leaders) {
    const int ng = g_end - g0 < pl.batch_leaders ? g_end - g0 : pl.batch_leaders;
    const void *qs[kMaxLayersPerLaunch], *ks[kMaxLayersPerLaunch];
    const float *ls[kMaxLayersPerLaunch];
    for (int i = 0; i < ng; ++i) {
      qs[i] = q_obs[(g0 + i) * reuse]; ks[i] = k[(g0 + i) * reuse];
      ls[i] = with_lse ? lse[(g0 + i) * reuse] : nullptr;
    }
    int rc = run_score(prob, pl, qs, ks, with_lse ? ls : nullptr, ng, g0, scores, nullptr, 0, ws, s);
    if (rc) return rc;
    rc = run_topk(prob, scores, g0, ng, sel_chunk, sel_len, sel_count, sel_off, s);
    if (rc) return rc;
    const int l_begin = g0 * reuse, l_end = (g0 + ng) * reuse < n_layers ? (g0 + ng) * reuse : n_layers;
    rc = run_compact(prob, l_begin, l_end, reuse, k, v, k_out, v_out, sel_chunk, sel_len, sel_count, sel_off, s);
    if (rc) return rc;
  }
  return CHUNKKV_OK;
}

static int stack_entry(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse, const void *const *q_obs,
                       const void *const *k, const void *const *v, const float *const *lse, bool with_lse,
                       void *const *k_out, void *const *v_out, int32_t *sel_chunk, int32_t *sel_len,
                       int32_t *sel_count, void *workspace, size_t workspace_bytes, void *stream) {
  int rc = check_problem(prob, true);
  if (rc) return rc;
  rc = check_stack_pointers(n_layers, reuse, q_obs, k, v, lse, with_lse, k_out, v_out, sel_chunk, sel_len, sel_count);
  if (rc) return rc;
  Plan pl;
  rc = make_plan(prob, n_layers, reuse, &pl);
  if (rc) return rc;
  if (!workspace || workspace_bytes < pl.total) return CHUNKKV_ERR_WORKSPACE;
  return stack_groups(prob, pl, 0, pl.n_leaders, n_layers, reuse, q_obs, k, v, lse, with_lse, k_out, v_out, sel_chunk,
                      sel_len, sel_count, (char *)workspace, (hipStream_t)stream);
}

size_t chunkkv_workspace_bytes_hybrid(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse,
                                      const int32_t *chunk_per_group) {
  size_t need = 0;
  const int rc = for_chunk_runs(prob, n_layers, reuse, chunk_per_group, [&](const chunkkv_problem &run, int, int) {
    Plan pl;
    const int r = make_plan(&run, n_layers, reuse, &pl);
    if (r) return r;
    need = pl.total > need ? pl.total : need;
    return (int)CHUNKKV_OK;
  });
  return rc ? 0 : need;
}

int chunkkv_compress_stack_hybrid(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse,
                                  const int32_t *chunk_per_group, const void *const *q_obs, const void *const *k,
                                  const void *const *v, const float *const *lse, void *const *k_out,
                                  void *const *v_out, int32_t *sel_chunk, int32_t *sel_len, int32_t *sel_count,
                                  void *workspace, size_t workspace_bytes, void *stream) {
  // everything is checked for every run before the first launch
  const size_t need = chunkkv_workspace_bytes_hybrid(prob, n_layers, reuse, chunk_per_group);
  if (need == 0) {
    const int rc = for_chunk_runs(prob, n_layers, reuse, chunk_per_group, [&](const chunkkv_problem &run, int, int) {
      Plan pl;
      return make_plan(&run, n_layers, reuse, &pl);
    });
    return rc ? rc : CHUNKKV_ERR_SHAPE;
  }
  const bool with_lse = lse != nullptr;
  int rc = check_stack_pointers(n_layers, reuse, q_obs, k, v, lse, with_lse, k_out, v_out, sel_chunk, sel_len, sel_count);
  if (rc) return rc;
  if (!workspace || workspace_bytes < need) return CHUNKKV_ERR_WORKSPACE;
  return for_chunk_runs(prob, n_layers, reuse, chunk_per_group, [&](const chunkkv_problem &run, int g0, int g1) {
    Plan pl;
    const int r = make_plan(&run, n_layers, reuse, &pl);
    if (r) return r;
    return stack_groups(&run, pl, g0, g1, n_layers, reuse, q_obs, k, v, lse, with_lse, k_out, v_out, sel_chunk, sel_len,
                        sel_count, (char *)workspace, (hipStream_t)stream);
  });
}

int chunkkv_compress_stack(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse, const void *const *q_obs,
                           const void *const *k, const void *const *v, void *const *k_out, void *const *v_out,
                           int32_t *sel_chunk, int32_t *sel_len, int32_t *sel_count, void *workspace,
                           size_t workspace_bytes, void *stream) {
  return stack_entry(prob, n_layers, reuse, q_obs, k, v, nullptr, false, k_out, v_out, sel_chunk, sel_len, sel_count,
                     workspace, workspace_bytes, stream);
}

int chunkkv_compress_stack_lse(const chunkkv_problem *prob, int32_t n_layers, int32_t reuse, const void *const *q_obs,
                               const void *const *k, const void *const *v, const float *const *lse,
                               void *const *k_out, void *const *v_out, int32_t *sel_chunk, int32_t *sel_len,
                               int32_t *sel_count, void *workspace, size_t workspace_bytes, void *stream) {
  return stack_entry(prob, n_layers, reuse, q_obs, k, v, lse, true, k_out, v_out, sel_chunk, sel_len, sel_count,
                     workspace, workspace_bytes, stream);
}

int chunkkv_compress_layer(const chunkkv_problem *prob, int32_t layer, int32_t reuse, const void *q_obs,
                           const float *lse, const void *k, const void *v, void *k_out, void *v_out,
                           int32_t *sel_chunk, int32_t *sel_len, int32_t *sel_count, void *workspace,
                           size_t workspace_bytes, void *stream) {
  int rc = check_problem(prob, true);
  if (rc) return rc;
  if (layer < 0 || reuse < 1) return CHUNKKV_ERR_SHAPE;
  const bool leader = layer % reuse == 0;
  if (!k || !v || !k_out || !v_out || !sel_chunk || !sel_len || !sel_count || (leader && !q_obs)) return CHUNKKV_ERR_NULL;
  if (misaligned(k) || misaligned(v) || misaligned(k_out) || misaligned(v_out) || (leader && misaligned(q_obs)))
    return CHUNKKV_ERR_SHAPE;
  Plan pl;
  rc = make_plan(prob, 1, 1, &pl);
  if (rc) return rc;
  if (!workspace || workspace_bytes < pl.total) return CHUNKKV_ERR_WORKSPACE;
  char *ws = (char *)workspace;
  hipStream_t s = (hipStream_t)stream;
  // the kernels see this layer's group as group 0 of arrays that start at the group's rows
  const int64_t row0 = (int64_t)(layer / reuse) * prob->batch * prob->n_kv_heads;
  int32_t *sc = sel_chunk + row0 * prob->sel_cap, *sl = sel_len + row0 * prob->sel_cap, *cnt = sel_count + row0;
  if (leader) {
    float *scores = (float *)(ws + pl.off_scores);
    rc = run_score(prob, pl, &q_obs, &k, lse ? &lse : nullptr, 1, 0, scores, nullptr, 0, ws, s);
    if (rc) return rc;
    rc = run_topk(prob, scores, 0, 1, sc, sl, cnt, nullptr, s);
    if (rc) return rc;
  }
  return run_compact(prob, 0, 1, 1, &k, &v, &k_out, &v_out, sc, sl, cnt, nullptr, s);
}

int chunkkv_jaccard(const chunkkv_problem *prob, int32_t n_groups, const int32_t *sel_chunk, const int32_t *sel_len,
                    const int32_t *sel_count, float *jaccard, void *stream) {
  int rc = check_problem(prob, false);
  if (rc) return rc;
  if (n_groups < 2) return CHUNKKV_ERR_SHAPE;
  if (!sel_chunk || !sel_len || !sel_count || !jaccard) return CHUNKKV_ERR_NULL;
  return launch_jaccard(sel_chunk, sel_len, sel_count, prob->sel_cap, prob->chunk, prob->batch * prob->n_kv_heads,
                        n_groups - 1, jaccard, (hipStream_t)stream);
}

size_t chunkkv_decode_workspace_bytes(const chunkkv_problem *prob, int32_t compacted) {
  DecodePlan pl;
  if (check_problem(prob, compacted != 0) || decode_plan(prob, compacted != 0, &pl)) return 0;
  return pl.total;
}

int chunkkv_decode_attention(const chunkkv_problem *prob, int32_t compacted, const int32_t *kv_len, const void *q,
                             const void *k, const void *v, float *out, float *lse, void *workspace,
                             size_t workspace_bytes, void *stream) {
  int rc = check_problem(prob, compacted != 0);
  if (rc) return rc;
  if (!q || !k || !v || !out) return CHUNKKV_ERR_NULL;
  if (misaligned(q) || misaligned(k) || misaligned(v)) return CHUNKKV_ERR_SHAPE;
  DecodePlan pl;
  if ((rc = decode_plan(prob, compacted != 0, &pl))) return rc;
  if (!workspace || workspace_bytes < pl.total) return CHUNKKV_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  const float scale = prob->softmax_scale > 0.f ? prob->softmax_scale : 1.0f / sqrtf((float)prob->head_dim);
  for (int b0 = 0; b0 < prob->batch; b0 += kMaxBatchPerLaunch) {
    const int nb = prob->batch - b0 < kMaxBatchPerLaunch ? prob->batch - b0 : kMaxBatchPerLaunch;
    DecodeArgs a{};
    a.q = q; a.k = k; a.v = v; a.out = out; a.lse = lse; a.kv_len = kv_len;
    a.part_ml = (float2 *)((char *)workspace + pl.off_ml);
    a.part_o = (float *)((char *)workspace + pl.off_o);
    for (int i = 0; i < nb; ++i) {
      a.n_tok[i] = compacted ? prob->n_keep[b0 + i] + prob->window : prob->seqlen[b0 + i];
      a.base[i] = compacted ? prob->out_base[b0 + i] : prob->kv_base[b0 + i];
    }
    a.stride_head = compacted ? prob->out_stride_head : prob->kv_stride_head;
    a.stride_tok = compacted ? prob->out_stride_tok : prob->kv_stride_tok;
    a.batch0 = b0; a.n_q_heads = prob->n_q_heads; a.n_kv_heads = prob->n_kv_heads;
    a.scale_log2e = scale * 1.4426950408889634f;
    a.n_split = pl.n_split; a.rows_per_split = pl.rows_per_split;
    { Timed t(kDecode, s); rc = launch_decode(prob->dtype, prob->head_dim, a, nb, s); }
    if (rc) return rc;
  }
  return CHUNKKV_OK;
}

int chunkkv_decode_attention_static(const chunkkv_problem *prob, int32_t compacted, const int32_t *kv_len,
                                    const void *q, const void *k, const void *v, float *out, float *lse,
                                    void *stream) {
  // the size check comes first: a problem that does not fit is refused before anything else happens
  int rc = check_problem(prob, compacted != 0);
  if (rc) return rc;
  DecodePlan pl;
  if ((rc = decode_plan(prob, compacted != 0, &pl))) return rc;
  if (pl.total > kStaticScratchBytes) return CHUNKKV_ERR_WORKSPACE;
  void *ws = nullptr;
  if ((rc = static_scratch(&ws))) return rc;
  // every partial result the merge kernel reads is written by the range kernel of the same call, so nothing
  // in the array has to be cleared between calls
  return chunkkv_decode_attention(prob, compacted, kv_len, q, k, v, out, lse, ws, pl.total, stream);
}

// Workspace of chunkkv_quality_metrics: the decode workspace (the larger of the two caches' needs), one decode
// output, two log-sum-exp arrays and the block partials of the two absolute masses.
namespace {
struct QualityPlan {
  int blocks_full, blocks_kept;
  size_t off_decode, off_out, off_lse_full, off_lse_kept, off_part_full, off_part_kept, total, decode_bytes;
};
int quality_plan(const chunkkv_problem *p, QualityPlan *q) {
  DecodePlan df, dk;
  int rc;
  if ((rc = decode_plan(p, false, &df)) || (rc = decode_plan(p, true, &dk))) return rc;
  int full_max = 0, kept_max = 0;
  for (int b = 0; b < p->batch; ++b) {
    full_max = p->seqlen[b] > full_max ? p->seqlen[b] : full_max;
    kept_max = p->n_keep[b] + p->window > kept_max ? p->n_keep[b] + p->window : kept_max;
  }
  q->blocks_full = abs_sum_blocks(full_max);
  q->blocks_kept = abs_sum_blocks(kept_max);
  const size_t heads = (size_t)p->batch * p->n_q_heads, kvh = (size_t)p->batch * p->n_kv_heads;
  q->decode_bytes = df.total > dk.total ? df.total : dk.total;
  size_t off = 0;
  q->off_decode = off;    off += align256(q->decode_bytes);
  q->off_out = off;       off += align256(heads * p->head_dim * sizeof(float));
  q->off_lse_full = off;  off += align256(heads * sizeof(float));
  q->off_lse_kept = off;  off += align256(heads * sizeof(float));
  q->off_part_full = off; off += align256(kvh * q->blocks_full * sizeof(float));
  q->off_part_kept = off; off += align256(kvh * q->blocks_kept * sizeof(float));
  q->total = off;
  return CHUNKKV_OK;
}
}  // namespace

size_t chunkkv_quality_workspace_bytes(const chunkkv_problem *prob) {
  QualityPlan q;
  if (check_problem(prob, true) || quality_plan(prob, &q)) return 0;
  return q.total;
}

int chunkkv_quality_metrics(const chunkkv_problem *prob, const int32_t *kv_len, const void *q, const void *k,
                            const void *v, const void *k_out, const void *v_out, float *l1_loss, float *attn_cos,
                            void *workspace, size_t workspace_bytes, void *stream) {
  int rc = check_problem(prob, true);
  if (rc) return rc;
  if (!q || !k || !v || !k_out || !v_out || !l1_loss || !attn_cos) return CHUNKKV_ERR_NULL;
  if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(k_out) || misaligned(v_out)) return CHUNKKV_ERR_SHAPE;
  QualityPlan pl;
  if ((rc = quality_plan(prob, &pl))) return rc;
  if (!workspace || workspace_bytes < pl.total) return CHUNKKV_ERR_WORKSPACE;
  char *ws = (char *)workspace;
  hipStream_t s = (hipStream_t)stream;
  // attention statistics at twice the softmax scale: exp(lse) = sum_t exp(2 scale q . k_t)
  chunkkv_problem twice = *prob;
  twice.softmax_scale = 2.f * (prob->softmax_scale > 0.f ? prob->softmax_scale : 1.0f / sqrtf((float)prob->head_dim));
  float *out = (float *)(ws + pl.off_out);
  float *lse_full = (float *)(ws + pl.off_lse_full), *lse_kept = (float *)(ws + pl.off_lse_kept);
  rc = chunkkv_decode_attention(&twice, 0, nullptr, q, k, v, out, lse_full, ws + pl.off_decode, pl.decode_bytes, stream);
  if (rc) return rc;
  rc = chunkkv_decode_attention(&twice, 1, kv_len, q, k_out, v_out, out, lse_kept, ws + pl.off_decode, pl.decode_bytes, stream);
  if (rc) return rc;
  for (int which = 0; which < 2; ++which) {
    for (int b0 = 0; b0 < prob->batch; b0 += kMaxBatchPerLaunch) {
      const int nb = prob->batch - b0 < kMaxBatchPerLaunch ? prob->batch - b0 : kMaxBatchPerLaunch;
      AbsSumArgs a{};
      a.k = which ? k_out : k; a.v = which ? v_out : v;
      a.partial = (float *)(ws + (which ? pl.off_part_kept : pl.off_part_full));
      a.kv_len = which ? kv_len : nullptr;
      for (int i = 0; i < nb; ++i) {
        a.n_tok[i] = which ? prob->n_keep[b0 + i] + prob->window : prob->seqlen[b0 + i];
        a.base[i] = which ? prob->out_base[b0 + i] : prob->kv_base[b0 + i];
      }
      a.stride_head = which ? prob->out_stride_head : prob->kv_stride_head;
      a.stride_tok = which ? prob->out_stride_tok : prob->kv_stride_tok;
      a.batch0 = b0; a.n_kv_heads = prob->n_kv_heads; a.head_dim = prob->head_dim;
      a.n_blocks = which ? pl.blocks_kept : pl.blocks_full;
      if ((rc = launch_abs_sum(prob->dtype, a, nb, s))) return rc;
    }
  }
  QualityFinishArgs f{};
  f.partial_full = (const float *)(ws + pl.off_part_full); f.partial_kept = (const float *)(ws + pl.off_part_kept);
  f.lse_full = lse_full; f.lse_kept = lse_kept; f.l1_loss = l1_loss; f.attn_cos = attn_cos;
  f.n_q_heads = prob->n_q_heads; f.n_kv_heads = prob->n_kv_heads;
  f.blocks_full = pl.blocks_full; f.blocks_kept = pl.blocks_kept;
  return launch_quality_finish(f, prob->batch, s);
}

int chunkkv_timing_begin(int32_t max_records) {
  if (g_timing.on || max_records < 1) return CHUNKKV_ERR_SHAPE;
  hipEvent_t *ev = new hipEvent_t[2 * (size_t)max_records];
  int *kind = new int[max_records];
  for (int i = 0; i < 2 * max_records; ++i) {
    if (hipEventCreate(&ev[i]) != hipSuccess) {
      for (int j = 0; j < i; ++j) (void)hipEventDestroy(ev[j]);
      delete[] ev;
      delete[] kind;
      return CHUNKKV_ERR_LAUNCH;
    }
  }
  g_timing.ev = ev;
  g_timing.kind = kind;
  g_timing.cap = max_records;
  g_timing.used = 0;
  g_timing.on = true;
  return CHUNKKV_OK;
}

int chunkkv_timing_end(double *total_ms, int64_t *launches) {
  if (!g_timing.on) return CHUNKKV_ERR_SHAPE;
  if (!total_ms || !launches) return CHUNKKV_ERR_NULL;
  g_timing.on = false;
  for (int k = 0; k < kKinds; ++k) { total_ms[k] = 0; launches[k] = 0; }
  int rc = CHUNKKV_OK;
  for (int i = 0; i < g_timing.used; ++i) {
    float ms = 0.f;
    if (hipEventSynchronize(g_timing.ev[2 * i + 1]) != hipSuccess ||
        hipEventElapsedTime(&ms, g_timing.ev[2 * i], g_timing.ev[2 * i + 1]) != hipSuccess) {
      rc = CHUNKKV_ERR_LAUNCH;
      continue;
    }
    total_ms[g_timing.kind[i]] += ms;
    launches[g_timing.kind[i]] += 1;
  }
  for (int i = 0; i < 2 * g_timing.cap; ++i) (void)hipEventDestroy(g_timing.ev[i]);
  delete[] g_timing.ev;
  delete[] g_timing.kind;
  g_timing.ev = nullptr; g_timing.kind = nullptr; g_timing.cap = g_timing.used = 0;
  return rc;
}

}  // extern "C"
