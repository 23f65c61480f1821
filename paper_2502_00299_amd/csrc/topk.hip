// Chunk selection (Algorithm 1, top-k step, with the exact-budget rule).
//
// One workgroup per (selection group, sequence, kv-head).  Chunks are ranked by (score descending,
// index ascending).  The m highest-ranked chunks are found with a most-significant-digit radix select
// over the order-preserving integer image of the fp32 scores (4 passes of 8 bits, histograms in LDS);
// ties at the threshold value are resolved towards the lower index by a prefix count in index order.
// m = ceil(n_keep / c); if the ragged last chunk is among those m and leaves the budget short, one
// more chunk is taken.  The lowest-ranked selected chunk is cut to the tokens still missing.
// Entries are emitted in ascending chunk order with a block-wide prefix scan; their exclusive token
// offsets are written next to them for the compaction kernel.
#include "internal.h"

namespace ckv {

constexpr int kTopkThreads = 1024;

__device__ __forceinline__ uint32_t order_key(float x) {
  uint32_t u = __float_as_uint(x);
  if (u == 0x80000000u) u = 0;  // -0 ranks as +0
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Block-wide exclusive scan of one int per thread (1024 threads); returns the exclusive prefix and
// stores the block total in *total.  s_tmp needs 16 ints.  Starts with a barrier (which also orders it after a
// previous call's reads of s_tmp) and does not end with one: the caller must not touch s_tmp before its next barrier.
__device__ __forceinline__ int block_exscan(int x, int *s_tmp, int *total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int inc = x;
  for (int o = 1; o < 64; o <<= 1) {
    const int y = __shfl_up(inc, o);
    if (lane >= o) inc += y;
  }
  __syncthreads();
  if (lane == 63) s_tmp[wave] = inc;
  __syncthreads();
  int wave_base = 0, tot = 0;
  for (int i = 0; i < kTopkThreads / 64; ++i) {
    const int v = s_tmp[i];
    if (i < wave) wave_base += v;
    tot += v;
  }
  *total = tot;
  return wave_base + inc - x;
}

__global__ __launch_bounds__(kTopkThreads) void topk_kernel(TopkArgs a) {
  const int tid = threadIdx.x;
  const int bl = blockIdx.x / a.n_kv_heads, h = blockIdx.x % a.n_kv_heads, group = a.group0 + blockIdx.y;
  const int64_t row = ((int64_t)group * a.batch_total + (a.batch0 + bl)) * a.n_kv_heads + h;
  const float *scores = a.chunk_scores + row * a.score_cap;
  int32_t *sel_chunk = a.sel_chunk + row * a.sel_cap;
  int32_t *sel_len = a.sel_len + row * a.sel_cap;
  int32_t *sel_off = a.sel_off ? a.sel_off + row * a.sel_cap : nullptr;
  const int c = a.chunk, P = pick(a.seq.seqlen, bl) - a.window, n_keep = pick(a.seq.n_keep, bl);
  const int C = (P + c - 1) / c;
  if (n_keep <= 0 || C <= 0) {
    if (tid == 0) a.sel_count[row] = 0;
    return;
  }
  const int tail_size = P - (C - 1) * c;  // == c when there is no ragged tail
  // exact budget: ceil(n_keep / c) chunks, the lowest-ranked one cut; whole-chunk mode: floor(n_keep / c)
  // chunks (at most C), none cut
  const int m0 = a.whole_chunks ? (n_keep / c < C ? n_keep / c : C) : (n_keep + c - 1) / c;
  if (m0 <= 0) {
    if (tid == 0) a.sel_count[row] = 0;
    return;
  }

  __shared__ int s_hist[256];
  __shared__ int s_tmp[16];
  __shared__ uint32_t s_prefix;
  __shared__ int s_remaining;
  __shared__ int s_pos_trunc;

  uint32_t thr = 0;   // key of the lowest-ranked selected chunk
  int need = 0;       // how many chunks with key == thr are selected (lowest indices first)
  int m = m0, total = 0;
  bool tail_sel = false;
  for (int attempt = 0; attempt < 2; ++attempt) {
    // ---- radix select: the m-th largest key
    if (tid == 0) { s_prefix = 0; s_remaining = m; }
    for (int shift = 24; shift >= 0; shift -= 8) {
      if (tid < 256) s_hist[tid] = 0;
      __syncthreads();
      const uint32_t prefix = s_prefix;
      const uint32_t mask = shift == 24 ? 0u : (0xFFFFFFFFu << (shift + 8));
      for (int i = tid; i < C; i += kTopkThreads) {
        const uint32_t key = order_key(scores[i]);
        if ((key & mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 255], 1);
      }
      __syncthreads();
      if (tid < 64) {
        // lane l owns digits 255-4l .. 252-4l (descending); find where the running count reaches `remaining`
        const int rem = s_remaining;
        int v[4], sum = 0;
        for (int j = 0; j < 4; ++j) { v[j] = s_hist[255 - 4 * tid - j]; sum += v[j]; }
        int inc = sum;
        for (int o = 1; o < 64; o <<= 1) {
          const int y = __shfl_up(inc, o);
          if (tid >= o) inc += y;
        }
        int before = inc - sum;  // keys with a larger digit than this lane's first
        if (before < rem && inc >= rem) {
          for (int j = 0; j < 4; ++j) {
            if (before + v[j] >= rem) {
              s_prefix = prefix | ((uint32_t)(255 - 4 * tid - j) << shift);
              s_remaining = rem - before;
              break;
            }
            before += v[j];
          }
        }
      }
      __syncthreads();
    }
    thr = s_prefix;
    need = s_remaining;  // rank of the threshold chunk among the chunks with key == thr, 1-based
    // ---- does the ragged tail chunk belong to the m selected?  It has the highest index, so among
    // equal keys it is taken last: selected iff key > thr, or key == thr and every equal key is taken.
    if (tid < 256) s_hist[tid] = 0;
    __syncthreads();
    int eq = 0;
    for (int i = tid; i < C; i += kTopkThreads) eq += order_key(scores[i]) == thr;
    if (eq) atomicAdd(&s_hist[0], eq);
    __syncthreads();
    const int cnt_eq = s_hist[0];
    const uint32_t tail_key = order_key(scores[C - 1]);
    tail_sel = tail_key > thr || (tail_key == thr && need == cnt_eq);
    total = m * c - (tail_sel ? c - tail_size : 0);
    __syncthreads();
    if (total >= n_keep || a.whole_chunks) break;
    m = m0 + 1;  // tail selected and budget short by < c tokens: exactly one more chunk is needed
  }
  // The lowest-ranked selected chunk is the need-th (index order) chunk with key == thr.  It is the
  // tail iff the tail's key == thr and the tail is selected.
  const bool trunc_is_tail = tail_sel && order_key(scores[C - 1]) == thr;
  const int size_trunc = trunc_is_tail ? tail_size : c;
  const int len_trunc = a.whole_chunks ? size_trunc : n_keep - (total - size_trunc);

  // ---- emit in ascending chunk order
  if (tid == 0) s_pos_trunc = 0x7FFFFFFF;
  // A thread takes kPerThread consecutive chunks per round, so a round costs two block-wide scans for
  // kPerThread * 1024 chunks.
  constexpr int kPerThread = 4;
  int base_sel = 0, base_eq = 0;
  for (int i0 = 0; i0 < C; i0 += kTopkThreads * kPerThread) {
    const int first = i0 + tid * kPerThread;
    uint32_t key[kPerThread];
    int is_eq[kPerThread], n_eq = 0;
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
      const int i = first + j;
      key[j] = i < C ? order_key(scores[i]) : 0u;
      is_eq[j] = i < C && key[j] == thr;
      n_eq += is_eq[j];
    }
    int tot_eq, tot_sel;
    int eq_rank = base_eq + block_exscan(n_eq, s_tmp, &tot_eq);
    int flag[kPerThread], n_sel = 0;
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
      const int i = first + j;
      flag[j] = i < C && (key[j] > thr || (is_eq[j] && eq_rank < need));
      // remember the rank this chunk has among the equal keys, then advance it
      is_eq[j] = is_eq[j] ? eq_rank + 1 : 0;  // 1-based rank, 0 = not equal
      eq_rank += is_eq[j] != 0;
      n_sel += flag[j];
    }
    int pos = base_sel + block_exscan(n_sel, s_tmp, &tot_sel);
#pragma unroll
    for (int j = 0; j < kPerThread; ++j) {
      const int i = first + j;
      if (flag[j] && pos < a.sel_cap) {
        const bool is_trunc = is_eq[j] == need;  // the need-th equal key in index order
        sel_chunk[pos] = i;
        sel_len[pos] = is_trunc ? len_trunc : (i == C - 1 ? tail_size : c);
        if (is_trunc) s_pos_trunc = pos;
      }
      pos += flag[j];
    }
    base_eq += tot_eq;
    base_sel += tot_sel;
    __syncthreads();
  }
  if (sel_off) {
    const int pos_trunc = s_pos_trunc;
    for (int p = tid; p < m && p < a.sel_cap; p += kTopkThreads)
      sel_off[p] = p * c - (p > pos_trunc ? size_trunc - len_trunc : 0);
  }
  if (tid == 0) a.sel_count[row] = m;
}

int launch_topk(const TopkArgs &a, int n_groups, int batch_slice, hipStream_t s) {
  if (n_groups <= 0 || batch_slice <= 0) return CHUNKKV_OK;
  dim3 grid(batch_slice * a.n_kv_heads, n_groups);
  hipLaunchKernelGGL(topk_kernel, grid, dim3(kTopkThreads), 0, s, a);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

// Adjacent-group Jaccard similarity of two selections of one (sequence, kv-head).  Both are ascending lists
// of (chunk, leading tokens kept); a chunk present in both shares min(len) tokens.  One workgroup per
// (pair of groups, sequence, kv-head): every thread takes entries of the first list and finds their chunk
// in the second by binary search; sums are reduced in a fixed order.
__global__ __launch_bounds__(256) void jaccard_kernel(const int32_t *sel_chunk, const int32_t *sel_len,
                                                      const int32_t *sel_count, int sel_cap, int rows_per_group,
                                                      float *out) {
  const int64_t ra = (int64_t)blockIdx.y * rows_per_group + blockIdx.x, rb = ra + rows_per_group;
  int na = sel_count[ra], nb = sel_count[rb];
  na = na < 0 ? 0 : (na > sel_cap ? sel_cap : na);
  nb = nb < 0 ? 0 : (nb > sel_cap ? sel_cap : nb);
  const int32_t *ca = sel_chunk + ra * sel_cap, *la = sel_len + ra * sel_cap;
  const int32_t *cb = sel_chunk + rb * sel_cap, *lb = sel_len + rb * sel_cap;
  int inter = 0, size_a = 0, size_b = 0;
  for (int i = threadIdx.x; i < na; i += 256) {
    const int ch = ca[i], ln = la[i];
    size_a += ln;
    int lo = 0, hi = nb;  // first entry of b with chunk >= ch
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (cb[mid] < ch) lo = mid + 1; else hi = mid;
    }
    if (lo < nb && cb[lo] == ch) inter += ln < lb[lo] ? ln : lb[lo];
  }
  for (int i = threadIdx.x; i < nb; i += 256) size_b += lb[i];
  __shared__ int s_red[3][4];
  for (int o = 32; o > 0; o >>= 1) {
    inter += __shfl_xor(inter, o); size_a += __shfl_xor(size_a, o); size_b += __shfl_xor(size_b, o);
  }
  if ((threadIdx.x & 63) == 0) {
    s_red[0][threadIdx.x >> 6] = inter; s_red[1][threadIdx.x >> 6] = size_a; s_red[2][threadIdx.x >> 6] = size_b;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    const int it = s_red[0][0] + s_red[0][1] + s_red[0][2] + s_red[0][3];
    const int un = s_red[1][0] + s_red[1][1] + s_red[1][2] + s_red[1][3] +
                   s_red[2][0] + s_red[2][1] + s_red[2][2] + s_red[2][3] - it;
    out[ra] = un > 0 ? (float)it / (float)un : 1.0f;
  }
}

int launch_jaccard(const int32_t *sel_chunk, const int32_t *sel_len, const int32_t *sel_count, int sel_cap, int chunk,
                   int rows_per_group, int n_pairs, float *out, hipStream_t s) {
  (void)chunk;
  if (rows_per_group <= 0 || n_pairs <= 0) return CHUNKKV_OK;
  hipLaunchKernelGGL(jaccard_kernel, dim3(rows_per_group, n_pairs), dim3(256), 0, s, sel_chunk, sel_len, sel_count,
                     sel_cap, rows_per_group, out);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

}  // namespace ckv
