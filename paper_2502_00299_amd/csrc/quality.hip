// Quality of a compressed layer against the full one (Appendix A.1): the share of the cache's absolute mass
// that the dropped tokens held, and the cosine between the decoding query's attention distribution over the
// full cache and over the kept tokens.
//
// The absolute mass of a cache is a plain streaming reduction (HBM-bound, 16 bytes per lane and load).  The
// gather copies rows verbatim, so the kept tokens' mass is the mass of the compacted cache and
// loss = 1 - mass(K', V') / mass(K, V).  For the cosine, with p the softmax over all tokens and p~ the softmax
// over the kept ones placed at their positions, p . p~ / (|p| |p~|) = sqrt(A_kept / A_all) where
// A = sum_t exp(2 scale q . k_t): the two sums are the log-sum-exps the decode-attention kernel returns when it
// runs at twice the softmax scale, so the host runs that kernel over both caches and a small kernel finishes.
#include "internal.h"

namespace ckv {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr int kAbsRowsPerWg = 1024;   // rows of K and of V one workgroup sums

template <int DT>
__device__ __forceinline__ float abs_sum16(const u32x4 &r) {
  const uint32_t d[4] = {r.x, r.y, r.z, r.w};
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if constexpr (DT == CHUNKKV_F32) {
      s += __builtin_fabsf(__uint_as_float(d[i]));
    } else if constexpr (DT == CHUNKKV_BF16) {
      s += __builtin_fabsf(__uint_as_float(d[i] << 16)) + __builtin_fabsf(__uint_as_float(d[i] & 0xFFFF0000u));
    } else {
      const f16x2 h = __builtin_bit_cast(f16x2, d[i]);
      s += __builtin_fabsf((float)h[0]) + __builtin_fabsf((float)h[1]);
    }
  }
  return s;
}

// grid: x = row block, y = (sequence, kv-head); partial[(b * Hkv + h) * n_blocks + x] = sum over the block's
// rows of |K| + |V|.  Fixed summation order: a thread adds its pieces in row order, the workgroup folds its
// threads in a fixed tree.
template <int DT>
__global__ __launch_bounds__(kThreads) void abs_sum_kernel(AbsSumArgs a) {
  const int bl = blockIdx.y / a.n_kv_heads, h = blockIdx.y % a.n_kv_heads;
  const int b = a.batch0 + bl;
  const int cap = pick(a.n_tok, bl);
  int n = cap;
  if (a.kv_len != nullptr) {
    n = a.kv_len[(int64_t)b * a.n_kv_heads + h];
    n = n < 0 ? 0 : (n > cap ? cap : n);
  }
  const int esz = DT == CHUNKKV_F32 ? 4 : 2;
  const int lpr = a.head_dim * esz / 16;             // 16-byte pieces per row
  const int r0 = blockIdx.x * kAbsRowsPerWg;
  const int r1 = r0 + kAbsRowsPerWg < n ? r0 + kAbsRowsPerWg : n;
  const int64_t head_off = (pick(a.base, bl) + (int64_t)h * a.stride_head) * esz;
  const int64_t tok = a.stride_tok * esz;
  float acc = 0.f;
  const int pieces = (r1 > r0 ? r1 - r0 : 0) * lpr;
  for (int i = threadIdx.x; i < pieces; i += kThreads) {
    const int64_t off = head_off + (int64_t)(r0 + i / lpr) * tok + (i % lpr) * 16;
    acc += abs_sum16<DT>(*(const u32x4 *)((const char *)a.k + off));
    acc += abs_sum16<DT>(*(const u32x4 *)((const char *)a.v + off));
  }
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o);
  __shared__ float s_w[kThreads / 64];
  if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0)
    a.partial[((int64_t)b * a.n_kv_heads + h) * a.n_blocks + blockIdx.x] = (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
}

// grid: x = sequence.  l1_loss[b] = 1 - mass of the compacted cache / mass of the full cache (block partials
// added in fp64, in index order); attn_cos[b][i] = exp((lse2_kept - lse2_all) / 2).
__global__ __launch_bounds__(kThreads) void quality_finish_kernel(QualityFinishArgs a) {
  const int b = blockIdx.x, t = threadIdx.x;
  __shared__ double s_sum[2][kThreads];
  for (int which = 0; which < 2; ++which) {
    const float *p = (which ? a.partial_kept : a.partial_full) + (int64_t)b * a.n_kv_heads * (which ? a.blocks_kept : a.blocks_full);
    const int n = a.n_kv_heads * (which ? a.blocks_kept : a.blocks_full);
    double acc = 0.0;
    for (int i = t; i < n; i += kThreads) acc += (double)p[i];
    s_sum[which][t] = acc;
  }
  __syncthreads();
  for (int o = kThreads / 2; o > 0; o >>= 1) {
    if (t < o) { s_sum[0][t] += s_sum[0][t + o]; s_sum[1][t] += s_sum[1][t + o]; }
    __syncthreads();
  }
  if (t == 0) {
    const double full = s_sum[0][0], kept = s_sum[1][0];
    double loss = full > 0.0 ? 1.0 - kept / full : 0.0;
    a.l1_loss[b] = (float)(loss < 0.0 ? 0.0 : loss);
  }
  for (int i = t; i < a.n_q_heads; i += kThreads) {
    const float all = a.lse_full[(int64_t)b * a.n_q_heads + i], kept = a.lse_kept[(int64_t)b * a.n_q_heads + i];
    // no kept token (or no token at all): similarity 0
    a.attn_cos[(int64_t)b * a.n_q_heads + i] = (kept == -__builtin_inff()) ? 0.f : __expf(0.5f * (kept - all));
  }
}

int abs_sum_blocks(int n_tok_max) { return n_tok_max > 0 ? (n_tok_max + kAbsRowsPerWg - 1) / kAbsRowsPerWg : 1; }

int launch_abs_sum(int dtype, const AbsSumArgs &a, int batch_slice, hipStream_t s) {
  const dim3 grid(a.n_blocks, batch_slice * a.n_kv_heads);
  if (dtype == CHUNKKV_BF16) hipLaunchKernelGGL(abs_sum_kernel<CHUNKKV_BF16>, grid, dim3(kThreads), 0, s, a);
  else if (dtype == CHUNKKV_F16) hipLaunchKernelGGL(abs_sum_kernel<CHUNKKV_F16>, grid, dim3(kThreads), 0, s, a);
  else if (dtype == CHUNKKV_F32) hipLaunchKernelGGL(abs_sum_kernel<CHUNKKV_F32>, grid, dim3(kThreads), 0, s, a);
  else return CHUNKKV_ERR_UNSUPPORTED;
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

int launch_quality_finish(const QualityFinishArgs &a, int batch, hipStream_t s) {
  hipLaunchKernelGGL(quality_finish_kernel, dim3(batch), dim3(kThreads), 0, s, a);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

}  // namespace ckv
