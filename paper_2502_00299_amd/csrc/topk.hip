// Chunk selection (Algorithm 1, top-k step, with the exact-budget rule).
//
// One workgroup per (selection group, sequence, kv-head).  Chunks are ranked by (score descending,
// index ascending).  The m highest-ranked chunks are found with a most-significant-digit radix select
// over the order-preserving integer image of the fp32 scores (4 passes of 8 bits, histograms in LDS);
// ties at the threshold value are resolved towards the lower index by a prefix count in index order.
// m = ceil(n_keep / c); if the ragged last chunk is among those m and leaves the budget short, one
// more chunk is taken.  The lowest-ranked selected chunk is cut to the tokens still missing.
// Entries are emitted in ascending chunk order with a block-wide prefix scan; their exclusive token
// offsets are written next to them for the compaction kernel.  Up to 16384 chunks per head the scores are
// read from global memory once and live in registers as keys.
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

constexpr int kRegKeys = 16;   // REG: a thread keeps its (at most 16) consecutive chunks' keys in registers

// Thread t owns the K = ceil(C / 1024) consecutive chunks from t * K on, so thread order is chunk order and one
// pair of block-wide scans emits the whole selection.  REG (C <= 16384, every configuration of the paper at
// 128K tokens with c >= 8): the scores are read from global memory once; otherwise each step re-reads them.
template <bool REG>
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

  const int K = (C + kTopkThreads - 1) / kTopkThreads;
  const int first = tid * K, last = first + K < C ? first + K : C;   // own chunks: [first, last), may be empty
  uint32_t kreg[REG ? kRegKeys : 1];
  if constexpr (REG) {
#pragma unroll
    for (int j = 0; j < kRegKeys; ++j) kreg[j] = first + j < last ? order_key(scores[first + j]) : 0u;
  }
  // f(chunk index, key) for every own chunk, in index order
  auto each = [&](auto f) __attribute__((always_inline)) {
    if constexpr (REG) {
#pragma unroll
      for (int j = 0; j < kRegKeys; ++j)
        if (first + j < last) f(first + j, kreg[j]);
    } else {
      for (int i = first; i < last; ++i) f(i, order_key(scores[i]));
    }
  };

  // Bits the keys of this head have in common (scores of one head share sign and most of the exponent): the
  // radix select starts at the first bit that differs, so its first digit already spreads the keys over the
  // histogram (few same-bin LDS atomics) and there are usually three passes, not four.
  uint32_t kmn = 0xFFFFFFFFu, kmx = 0u;
  each([&](int, uint32_t key) { kmn = key < kmn ? key : kmn; kmx = key > kmx ? key : kmx; });
  for (int o = 32; o > 0; o >>= 1) {
    const uint32_t x = __shfl_xor(kmn, o), y = __shfl_xor(kmx, o);
    kmn = x < kmn ? x : kmn; kmx = y > kmx ? y : kmx;
  }
  __shared__ uint32_t s_mn[kTopkThreads / 64], s_mx[kTopkThreads / 64];
  if ((tid & 63) == 0) { s_mn[tid >> 6] = kmn; s_mx[tid >> 6] = kmx; }
  __syncthreads();
  for (int i = 0; i < kTopkThreads / 64; ++i) { kmn = s_mn[i] < kmn ? s_mn[i] : kmn; kmx = s_mx[i] > kmx ? s_mx[i] : kmx; }
  const int hi = kmn == kmx ? 0 : 32 - __builtin_clz(kmn ^ kmx);   // bits [0, hi) vary
  const uint32_t common = hi >= 32 ? 0u : (kmx >> hi) << hi;

  uint32_t thr = 0;   // key of the lowest-ranked selected chunk
  int need = 0;       // how many chunks with key == thr are selected (lowest indices first)
  int m = m0, total = 0, eq_own = 0;
  bool tail_sel = false;
  const uint32_t tail_key = order_key(scores[C - 1]);
  for (int attempt = 0; attempt < 2; ++attempt) {
    // ---- radix select: the m-th largest key, 8 bits per pass from bit `top` down
    if (tid == 0) { s_prefix = common; s_remaining = m; }
    for (int top = hi; top > 0;) {
      const int shift = top > 8 ? top - 8 : 0;
      if (tid < 256) s_hist[tid] = 0;
      __syncthreads();
      const uint32_t prefix = s_prefix;
      const uint32_t mask = top >= 32 ? 0u : (0xFFFFFFFFu << top);   // bits settled so far; prefix is zero below
      each([&](int, uint32_t key) {
        if ((key & mask) == prefix) atomicAdd(&s_hist[(key >> shift) & 255], 1);
      });
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
              // with fewer than 8 varying bits left the digit's upper bits repeat bits of the prefix
              s_prefix = prefix | ((uint32_t)(255 - 4 * tid - j) << shift);
              s_remaining = rem - before;
              break;
            }
            before += v[j];
          }
        }
      }
      __syncthreads();
      top = shift;
    }
    thr = s_prefix;
    need = s_remaining;  // rank of the threshold chunk among the chunks with key == thr, 1-based
    // ---- does the ragged tail chunk belong to the m selected?  It has the highest index, so among
    // equal keys it is taken last: selected iff key > thr, or key == thr and every equal key is taken.
    if (tid < 256) s_hist[tid] = 0;
    __syncthreads();
    eq_own = 0;
    each([&](int, uint32_t key) { eq_own += key == thr; });
    int eq = eq_own;
    for (int o = 32; o > 0; o >>= 1) eq += __shfl_xor(eq, o);
    if ((tid & 63) == 0 && eq) atomicAdd(&s_hist[0], eq);
    __syncthreads();
    const int cnt_eq = s_hist[0];
    tail_sel = tail_key > thr || (tail_key == thr && need == cnt_eq);
    total = m * c - (tail_sel ? c - tail_size : 0);
    __syncthreads();
    if (total >= n_keep || a.whole_chunks) break;
    m = m0 + 1;  // tail selected and budget short by < c tokens: exactly one more chunk is needed
  }
  // The lowest-ranked selected chunk is the need-th (index order) chunk with key == thr.  It is the
  // tail iff the tail's key == thr and the tail is selected.
  const bool trunc_is_tail = tail_sel && tail_key == thr;
  const int size_trunc = trunc_is_tail ? tail_size : c;
  const int len_trunc = a.whole_chunks ? size_trunc : n_keep - (total - size_trunc);

  // ---- emit in ascending chunk order: rank among the equal keys, then position among the selected
  if (tid == 0) s_pos_trunc = 0x7FFFFFFF;
  int tot_eq, tot_sel;
  const int eq_rank0 = block_exscan(eq_own, s_tmp, &tot_eq);   // equal keys before this thread's chunks
  int n_sel = 0, eq_rank = eq_rank0;
  each([&](int, uint32_t key) {
    const bool is_eq = key == thr;
    n_sel += key > thr || (is_eq && eq_rank < need);
    eq_rank += is_eq;
  });
  int pos = block_exscan(n_sel, s_tmp, &tot_sel);
  eq_rank = eq_rank0;
  each([&](int i, uint32_t key) {
    const bool is_eq = key == thr;
    const bool sel = key > thr || (is_eq && eq_rank < need);
    if (sel && pos < a.sel_cap) {
      const bool is_trunc = is_eq && eq_rank + 1 == need;  // the need-th equal key in index order
      sel_chunk[pos] = i;
      sel_len[pos] = is_trunc ? len_trunc : (i == C - 1 ? tail_size : c);
      if (is_trunc) s_pos_trunc = pos;
    }
    pos += sel;
    eq_rank += is_eq;
  });
  __syncthreads();
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
  int c_max = 0;
  for (int i = 0; i < batch_slice; ++i) {
    const int C = (a.seq.seqlen[i] - a.window + a.chunk - 1) / a.chunk;
    c_max = C > c_max ? C : c_max;
  }
  if (c_max <= kTopkThreads * kRegKeys) hipLaunchKernelGGL(topk_kernel<true>, grid, dim3(kTopkThreads), 0, s, a);
  else hipLaunchKernelGGL(topk_kernel<false>, grid, dim3(kTopkThreads), 0, s, a);
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
