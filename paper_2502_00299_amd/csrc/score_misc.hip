// Small kernels around the two scoring passes: merging the per-range softmax statistics, and the
// chunk sums for chunk sizes too large to fit one key tile.
#include "internal.h"

namespace ckv {

int launch_score_bf16(int pass, int head_dim, const ScoreGeom &g, const ScoreArgs &a, dim3 grid, hipStream_t s);
int launch_score_f32(int pass, int head_dim, const ScoreGeom &g, const ScoreArgs &a, dim3 grid, hipStream_t s);

bool score_geometry(int dtype, int head_dim, int rows, ScoreGeom *g) {
  if (dtype != CHUNKKV_F32 && dtype != CHUNKKV_BF16) return false;
  if (head_dim != 64 && head_dim != 128) return false;
  if (rows < 1 || rows > kMaxRows) return false;
  g->row_bytes = head_dim * (dtype == CHUNKKV_BF16 ? 2 : 4);
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
  return dtype == CHUNKKV_BF16 ? launch_score_bf16(pass, head_dim, g, a, grid, s)
                               : launch_score_f32(pass, head_dim, g, a, grid, s);
}

// ref_r = max_r + log2(sum_r) over all key ranges of a problem.  grid: x = (sequence, kv-head), y = leader.
__global__ void stats_combine_kernel(ScoreArgs a, int tile_keys) {
  const int bl = blockIdx.x / a.n_kv_heads, h = blockIdx.x % a.n_kv_heads, z = blockIdx.y;
  const int64_t problem = ((int64_t)(a.leader0 + z) * a.batch_total + (a.batch0 + bl)) * a.n_kv_heads + h;
  const int L = pick(a.seq.seqlen, bl);
  const int ntiles = (L + tile_keys - 1) / tile_keys;
  const int nsplit = (ntiles + a.tiles_per_wg - 1) / a.tiles_per_wg;
  for (int row = threadIdx.x; row < a.rows_pad; row += blockDim.x) {
    const float2 *ps = a.part_stats + problem * a.max_split * a.rows_pad + row;
    float m = -1.0e30f;
    for (int s = 0; s < nsplit; ++s) m = fmaxf(m, ps[(int64_t)s * a.rows_pad].x);
    float l = 0.f;
    for (int s = 0; s < nsplit; ++s) {
      const float2 x = ps[(int64_t)s * a.rows_pad];
      l += x.y * exp2f(x.x - m);
    }
    a.refs[problem * a.rows_pad + row] = m + log2f(l);
  }
}

int launch_stats_combine(const ScoreArgs &a, int n_leaders_slice, int batch_slice, int tile_keys, hipStream_t s) {
  if (n_leaders_slice <= 0 || batch_slice <= 0) return CHUNKKV_OK;
  dim3 grid(batch_slice * a.n_kv_heads, n_leaders_slice);
  hipLaunchKernelGGL(stats_combine_kernel, grid, dim3(a.rows_pad < 256 ? a.rows_pad : 256), 0, s, a, tile_keys);
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

// Single-pass path, last step: score[chunk] = sum over rows of E[chunk][row] * exp2(m_period[row] - ref[row]).
// One workgroup per (period, sequence, kv-head, leader), one thread per (padded) window row: a thread reads
// its 16 slot values (64 contiguous bytes), weights them, and the 16 sums are reduced across the workgroup
// in a fixed order.  grid: x = period, y = (sequence, kv-head), z = leader.
__global__ void fused_scores_kernel(ScoreArgs a) {
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nwaves = blockDim.x >> 6;
  const int bl = blockIdx.y / a.n_kv_heads, h = blockIdx.y % a.n_kv_heads, z = blockIdx.z;
  const int64_t problem = ((int64_t)(a.leader0 + z) * a.batch_total + (a.batch0 + bl)) * a.n_kv_heads + h;
  const int P = pick(a.seq.seqlen, bl) - a.window, c = a.chunk;
  const int C = (P + c - 1) / c, nslots = a.period_keys / c, period = blockIdx.x;
  if ((int64_t)period * a.period_keys >= P) return;
  const int nrows = (a.n_q_heads / a.n_kv_heads) * a.window;
  __shared__ float s_red[8][16];
  float v[16];
  if (tid < nrows) {
    const int64_t pr = ((int64_t)problem * a.n_periods + period) * a.rows_pad + tid;
    const float wgt = exp2f(a.m_period[pr] - a.refs[problem * a.rows_pad + tid]);
    const f32x4 *src = (const f32x4 *)(a.e_buf + pr * 16);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const f32x4 x = src[q];
      v[4 * q] = x.x * wgt; v[4 * q + 1] = x.y * wgt; v[4 * q + 2] = x.z * wgt; v[4 * q + 3] = x.w * wgt;
    }
  } else {
#pragma unroll
    for (int s = 0; s < 16; ++s) v[s] = 0.f;
  }
#pragma unroll
  for (int s = 0; s < 16; ++s) {
    for (int o = 32; o > 0; o >>= 1) v[s] += __shfl_xor(v[s], o);
  }
  if (lane == 0) {
#pragma unroll
    for (int s = 0; s < 16; ++s) s_red[wave][s] = v[s];
  }
  __syncthreads();
  if (tid < nslots) {
    const int chunk = period * nslots + tid;
    if (chunk < C) {
      float sum = 0.f;
      for (int i = 0; i < nwaves; ++i) sum += s_red[i][tid];
      a.chunk_scores[problem * a.score_cap + chunk] = sum;
    }
  }
}

int launch_fused_scores(const ScoreArgs &a, int n_leaders_slice, int batch_slice, hipStream_t s) {
  int max_periods = 0;
  for (int b = 0; b < batch_slice; ++b) {
    const int P = a.seq.seqlen[b] - a.window;
    const int np = (P + a.period_keys - 1) / a.period_keys;
    max_periods = np > max_periods ? np : max_periods;
  }
  if (max_periods == 0 || n_leaders_slice <= 0) return CHUNKKV_OK;
  dim3 grid(max_periods, batch_slice * a.n_kv_heads, n_leaders_slice);
  hipLaunchKernelGGL(fused_scores_kernel, grid, dim3(a.rows_pad), 0, s, a);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

}  // namespace ckv
