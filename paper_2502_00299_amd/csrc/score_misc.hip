// Small kernels around the two scoring passes: merging the per-range softmax statistics, and the
// chunk sums for chunk sizes too large to fit one key tile.
#include "internal.h"

namespace ckv {

int launch_score_bf16(int pass, int head_dim, const ScoreGeom &g, const ScoreArgs &a, dim3 grid, hipStream_t s);
int launch_score_f16(int pass, int head_dim, const ScoreGeom &g, const ScoreArgs &a, dim3 grid, hipStream_t s);
int launch_score_f32(int pass, int head_dim, const ScoreGeom &g, const ScoreArgs &a, dim3 grid, hipStream_t s);
int launch_score_single_bf16(const ScoreArgs &a, dim3 grid, hipStream_t s);
int launch_score_single_f16(const ScoreArgs &a, dim3 grid, hipStream_t s);

bool score_geometry(int dtype, int head_dim, int rows, ScoreGeom *g) {
  if (dtype != CHUNKKV_F32 && dtype != CHUNKKV_BF16 && dtype != CHUNKKV_F16) return false;
  if (head_dim != 64 && head_dim != 128) return false;
  if (rows < 1 || rows > kMaxRows) return false;
  g->row_bytes = head_dim * elem_bytes(dtype);
  g->tile_keys = kTileBytes / g->row_bytes;
  g->nq_blocks = (rows + 31) / 32;
  if (g->nq_blocks == 1) { g->nqw = 1; g->wq = 1; }
  else if (g->nq_blocks == 2) { g->nqw = 1; g->wq = 2; }
  else if (g->nq_blocks <= 4) { g->nqw = 1; g->wq = 4; }
  else if (g->nq_blocks <= 8) { g->nqw = 2; g->wq = 4; }
  else { g->nqw = 4; g->wq = 4; }
  if (g->nqw == 4 && dtype == CHUNKKV_F32 && head_dim == 128) return false;  // operand registers exceed the file
  return true;
}

int launch_score_pass(int pass, int dtype, int head_dim, const ScoreGeom &g, const ScoreArgs &a, dim3 grid,
                      hipStream_t s) {
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return CHUNKKV_OK;
  if (dtype == CHUNKKV_BF16) return launch_score_bf16(pass, head_dim, g, a, grid, s);
  if (dtype == CHUNKKV_F16) return launch_score_f16(pass, head_dim, g, a, grid, s);
  return launch_score_f32(pass, head_dim, g, a, grid, s);
}

// Does the single-pass kernel take this problem?  16-bit caches of head_dim 128, 65 to 256 window rows per
// kv-head, chunk sizes that cut a lane half's 80 keys into a multiple of four chunks.
bool single_pass_ok(int dtype, int head_dim, int rows, int chunk) {
  return (dtype == CHUNKKV_BF16 || dtype == CHUNKKV_F16) && head_dim == 128 && rows > 64 && rows <= 256 &&
         (chunk == 5 || chunk == 10 || chunk == 20);
}

int launch_score_single(int dtype, const ScoreArgs &a, dim3 grid, hipStream_t s) {
  if (grid.x == 0 || grid.y == 0 || grid.z == 0) return CHUNKKV_OK;
  if (dtype == CHUNKKV_BF16) return launch_score_single_bf16(a, grid, s);
  if (dtype == CHUNKKV_F16) return launch_score_single_f16(a, grid, s);
  return CHUNKKV_ERR_UNSUPPORTED;
}

// ref_r = max_r + log2(sum_r) over all key ranges of a problem.  Four lanes share a row: each merges a
// quarter of the ranges in one pass ((m, l) pairs merge associatively), then the four partial pairs are
// merged with two shuffles, always in the same order.  grid: x = (sequence, kv-head), y = leader; 256 threads.
__global__ __launch_bounds__(256) void stats_combine_kernel(ScoreArgs a, int tile_keys) {
  const int bl = blockIdx.x / a.n_kv_heads, h = blockIdx.x % a.n_kv_heads, z = blockIdx.y;
  const int64_t problem = ((int64_t)(a.leader0 + z) * a.batch_total + (a.batch0 + bl)) * a.n_kv_heads + h;
  const int L = pick(a.seq.seqlen, bl);
  const int ntiles = (L + tile_keys - 1) / tile_keys;
  const int nsplit = (ntiles + a.tiles_per_wg - 1) / a.tiles_per_wg;
  const int part = threadIdx.x & 3;
  for (int row0 = 0; row0 < a.rows_pad; row0 += 64) {
    const int row = row0 + (threadIdx.x >> 2);  // rows_pad is a multiple of 32; rows past it are skipped below
    const bool live = row < a.rows_pad;
    const float2 *ps = a.part_stats + problem * a.max_split * a.rows_pad + (live ? row : 0);
    float m = -1.0e30f, l = 0.f;
    for (int s = part; s < nsplit; s += 4) {
      const float2 x = ps[(int64_t)s * a.rows_pad];
      const float mm = fmaxf(m, x.x);
      l = l * exp2f(m - mm) + x.y * exp2f(x.x - mm);
      m = mm;
    }
#pragma unroll
    for (int o = 1; o < 4; o <<= 1) {
      const float mo = __shfl_xor(m, o), lo = __shfl_xor(l, o);
      const float mm = fmaxf(m, mo);
      // both partners compute the same sum in the same order: lower lane's term first
      const bool low = (part & o) == 0;
      const float a0 = (low ? l : lo) * exp2f((low ? m : mo) - mm), a1 = (low ? lo : l) * exp2f((low ? mo : m) - mm);
      l = a0 + a1;
      m = mm;
    }
    if (live && part == 0) a.refs[problem * a.rows_pad + row] = m + log2f(l);
  }
}

int launch_stats_combine(const ScoreArgs &a, int n_leaders_slice, int batch_slice, int tile_keys, hipStream_t s) {
  if (n_leaders_slice <= 0 || batch_slice <= 0) return CHUNKKV_OK;
  dim3 grid(batch_slice * a.n_kv_heads, n_leaders_slice);
  hipLaunchKernelGGL(stats_combine_kernel, grid, dim3(256), 0, s, a, tile_keys);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

// ref_r = lse_r * log2(e): the caller's natural-log normalisation of a window row in the importance pass's
// units.  grid: x = (sequence, kv-head), y = leader; one thread per (padded) row.
__global__ void lse_refs_kernel(LseArgs a) {
  const int bl = blockIdx.x / a.n_kv_heads, h = blockIdx.x % a.n_kv_heads, z = blockIdx.y;
  const int g = a.n_q_heads / a.n_kv_heads, w = a.window, nrows = g * w;
  const int64_t problem = ((int64_t)(a.leader0 + z) * a.batch_total + (a.batch0 + bl)) * a.n_kv_heads + h;
  const float *lse = pick(a.lse, z) + ((int64_t)(a.batch0 + bl) * a.n_q_heads + (int64_t)h * g) * w;
  for (int row = threadIdx.x; row < a.rows_pad; row += blockDim.x)
    a.refs[problem * a.rows_pad + row] = row < nrows ? lse[row] * 1.4426950408889634f : 0.f;
}

int launch_lse_refs(const LseArgs &a, int n_leaders_slice, int batch_slice, hipStream_t s) {
  if (n_leaders_slice <= 0 || batch_slice <= 0) return CHUNKKV_OK;
  dim3 grid(batch_slice * a.n_kv_heads, n_leaders_slice);
  hipLaunchKernelGGL(lse_refs_kernel, grid, dim3(a.rows_pad < 256 ? a.rows_pad : 256), 0, s, a);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

// Chunk sums from per-token importance, one wavefront per chunk, fixed summation order.
// grid: x = chunk group of 4, y = (sequence, kv-head), z = leader.
__global__ void chunk_sums_kernel(ScoreArgs a) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int bl = blockIdx.y / a.n_kv_heads, h = blockIdx.y % a.n_kv_heads, z = blockIdx.z;
  const int64_t problem = ((int64_t)(a.leader0 + z) * a.batch_total + (a.batch0 + bl)) * a.n_kv_heads + h;
  const int P = pick(a.seq.seqlen, bl) - a.window, c = a.chunk;
  const int C = (P + c - 1) / c;
  const int ci = blockIdx.x * 4 + wave;
  if (ci >= C) return;
  const float *imp = a.token_imp + problem * a.imp_pitch;
  const int64_t j0 = (int64_t)ci * c, j1 = j0 + c < P ? j0 + c : P;
  float sum = 0.f;
  for (int64_t j = j0 + lane; j < j1; j += 64) sum += imp[j];
  for (int o = 32; o > 0; o >>= 1) sum += __shfl_xor(sum, o);
  if (lane == 0) a.chunk_scores[problem * a.score_cap + ci] = sum;
}

int launch_chunk_sums(const ScoreArgs &a, int n_leaders_slice, int batch_slice, hipStream_t s) {
  int maxC = 0;
  for (int b = 0; b < batch_slice; ++b) {
    const int P = a.seq.seqlen[b] - a.window;
    const int C = (P + a.chunk - 1) / a.chunk;
    maxC = C > maxC ? C : maxC;
  }
  if (maxC == 0 || n_leaders_slice <= 0) return CHUNKKV_OK;
  dim3 grid((maxC + 3) / 4, batch_slice * a.n_kv_heads, n_leaders_slice);
  hipLaunchKernelGGL(chunk_sums_kernel, grid, dim3(256), 0, s, a);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

// Single-pass path, second kernel: the row references and the chunk scores.
//   ref_r = m_r + log2(sum_r), merged from the (reference, sum) pairs the key ranges left for row r
//           (pairs merge associatively; always in the same order: range by range);
//   score[chunk] = sum over rows of E[chunk][row] * exp2(m[chunk][row] - ref[row]).
// A workgroup of 256 threads merges the statistics of its problem (one row per thread) and then takes
// kPeriodsPerGroup consecutive periods.  Per period the scoring kernel left, for each lane half h and each
// group of eight consecutive chunks of that half, rows_pad pieces of 16 + 4 bytes (eight sums as 20-bit floats:
// 8 exponent and 12 mantissa bits; chunk size 20 has four chunks per half: pieces of 12 bytes, four 24-bit
// floats), and rows_pad references (one per row).  A wavefront takes one (period, half, group) at a time: its
// lanes walk the rows (consecutive lanes read consecutive pieces), weigh, and the sums are reduced over the
// lanes in a fixed order.  The chunk of (half h, position s) is 2 s + h of the period's 2 S chunks.  Rows past
// the real ones are skipped: nothing was written for them.
// grid: x = period group, y = (sequence, kv-head), z = leader.
constexpr int kPeriodsPerGroup = 32;
constexpr int kSinglePeriod = 160, kSingleHalf = 80;   // as in the single-pass scoring kernel

__global__ __launch_bounds__(256) void single_scores_kernel(ScoreArgs a) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  typedef unsigned int u32x3 __attribute__((ext_vector_type(3)));
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int bl = blockIdx.y / a.n_kv_heads, h = blockIdx.y % a.n_kv_heads, z = blockIdx.z;
  const int64_t problem = ((int64_t)(a.leader0 + z) * a.batch_total + (a.batch0 + bl)) * a.n_kv_heads + h;
  const int L = pick(a.seq.seqlen, bl), P = L - a.window, c = a.chunk;
  const int C = (P + c - 1) / c, S = kSingleHalf / c;
  const int np = (P + kSinglePeriod - 1) / kSinglePeriod;   // periods that hold prefix keys
  const int p0 = blockIdx.x * kPeriodsPerGroup;
  if (p0 >= np) return;
  const int p1 = p0 + kPeriodsPerGroup < np ? p0 + kPeriodsPerGroup : np;
  const int nrows = (a.n_q_heads / a.n_kv_heads) * a.window;
  __shared__ float s_ref[256];

  // ---- references
  {
    const int np_total = (L + kSinglePeriod - 1) / kSinglePeriod, ppr = single_periods_per_range(np_total);
    const int nsplit = (np_total + ppr - 1) / ppr;
    float m = -1.0e30f, l = 0.f;
    if (tid < nrows) {
      const float2 *ps = a.part_stats + problem * a.max_split * a.rows_pad + tid;
      for (int s = 0; s < nsplit; ++s) {
        const float2 x = ps[(int64_t)s * a.rows_pad];
        const float mm = fmaxf(m, x.x);
        l = l * exp2f(m - mm) + x.y * exp2f(x.x - mm);
        m = mm;
      }
    }
    s_ref[tid] = tid < nrows ? m + log2f(l) : 3.0e38f;
  }
  __syncthreads();

  // ---- chunk scores
  const int64_t prow = (int64_t)a.rows_pad;
  const float *m_problem = a.m_period + problem * a.n_periods * prow;
  if (S == 4) {
    // [lane half][rows_pad] x 12 bytes: four sums as the upper three bytes of their fp32
    const char *e_problem = (const char *)a.e_buf + problem * a.n_periods * prow * 24;
    for (int task = wave; task < (p1 - p0) * 2; task += 4) {
      const int period = p0 + task / 2, hh = task % 2;
      const char *src = e_problem + ((int64_t)period * 2 + hh) * prow * 12;
      const float *mp = m_problem + (int64_t)period * prow;
      f32x4 v = {0.f, 0.f, 0.f, 0.f};
      for (int row = lane; row < nrows; row += 64) {
        const float wgt = exp2f(mp[row] - s_ref[row]);
        const u32x3 d = __builtin_nontemporal_load((const u32x3 *)(src + row * 12));
        const f32x4 x = {__uint_as_float(d.x << 8), __uint_as_float(__builtin_amdgcn_alignbit(d.y, d.x, 24) << 8),
                         __uint_as_float(__builtin_amdgcn_alignbit(d.z, d.y, 16) << 8), __uint_as_float(d.z & 0xFFFFFF00u)};
        v += x * wgt;
      }
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        v.x += __shfl_xor(v.x, o); v.y += __shfl_xor(v.y, o); v.z += __shfl_xor(v.z, o); v.w += __shfl_xor(v.w, o);
      }
      if (lane < 4) {
        const int chunk = period * 2 * S + 2 * lane + hh;
        const float val = lane == 0 ? v.x : (lane == 1 ? v.y : (lane == 2 ? v.z : v.w));
        if (chunk < C) a.chunk_scores[problem * a.score_cap + chunk] = val;
      }
    }
  } else {
    // groups of eight sums as 20-bit floats: [lane half][group][rows_pad] x 16 bytes, then x 4 bytes
    const int G8 = S / 8, combos = 2 * G8;
    const char *e_problem = (const char *)a.e_buf + problem * a.n_periods * prow * (combos * 20);
    for (int task = wave; task < (p1 - p0) * combos; task += 4) {
      const int period = p0 + task / combos, combo = task % combos;   // combo = half * G8 + group
      const int hh = combo / G8, g8 = combo % G8;
      const char *pbase = e_problem + (int64_t)period * prow * (combos * 20);
      const char *src_lo = pbase + (int64_t)combo * prow * 16, *src_hi = pbase + (int64_t)combos * prow * 16 + (int64_t)combo * prow * 4;
      const float *mp = m_problem + (int64_t)period * prow;
      float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      for (int row = lane; row < nrows; row += 64) {
        const float wgt = exp2f(mp[row] - s_ref[row]);
        const u32x4 w = __builtin_nontemporal_load((const u32x4 *)(src_lo + row * 16));
        const uint32_t w4 = __builtin_nontemporal_load((const uint32_t *)(src_hi + row * 4));
        uint32_t q[8];
        q[0] = w.x & 0xFFFFFu;
        q[1] = (w.x >> 20) | ((w.y & 0xFFu) << 12);
        q[2] = (w.y >> 8) & 0xFFFFFu;
        q[3] = (w.y >> 28) | ((w.z & 0xFFFFu) << 4);
        q[4] = (w.z >> 16) | ((w.w & 0xFu) << 16);
        q[5] = (w.w >> 4) & 0xFFFFFu;
        q[6] = (w.w >> 24) | ((w4 & 0xFFFu) << 8);
        q[7] = w4 >> 12;
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] += __uint_as_float(q[i] << 11) * wgt;
      }
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] += __shfl_xor(v[i], o);
      }
      if (lane < 8) {
        float val = v[0];
#pragma unroll
        for (int i = 1; i < 8; ++i) val = lane == i ? v[i] : val;
        const int chunk = period * 2 * S + 2 * (8 * g8 + lane) + hh;
        if (chunk < C) a.chunk_scores[problem * a.score_cap + chunk] = val;
      }
    }
  }
}

int launch_single_scores(const ScoreArgs &a, int n_leaders_slice, int batch_slice, hipStream_t s) {
  int max_periods = 0;
  for (int b = 0; b < batch_slice; ++b) {
    const int P = a.seq.seqlen[b] - a.window;
    const int np = (P + kSinglePeriod - 1) / kSinglePeriod;
    max_periods = np > max_periods ? np : max_periods;
  }
  if (max_periods == 0 || n_leaders_slice <= 0) return CHUNKKV_OK;
  if (a.rows_pad > 256 || kSingleHalf % a.chunk != 0 || (kSingleHalf / a.chunk) % 4 != 0) return CHUNKKV_ERR_UNSUPPORTED;
  dim3 grid((max_periods + kPeriodsPerGroup - 1) / kPeriodsPerGroup, batch_slice * a.n_kv_heads, n_leaders_slice);
  hipLaunchKernelGGL(single_scores_kernel, grid, dim3(256), 0, s, a);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

}  // namespace ckv
