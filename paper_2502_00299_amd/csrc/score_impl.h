// Observation-window scoring (Algorithm 1, first two steps, with the row softmax the text implies).
//
// For one (leader layer, sequence, kv-head) the g*w window rows are multiplied with every key on the
// matrix cores (bf16: v_mfma_f32_32x32x16_bf16, f32: v_mfma_f32_32x32x2_f32; fp32 accumulation).
// The exact softmax needs each row's maximum and sum over ALL visible keys before any column can be
// normalised, so the work is two passes over K:
//   pass 0  (keys x rows orientation: a lane owns one window row)  streams K, keeps a running
//           (max, sum) per row in registers, and writes one partial pair per row and key range;
//   -----   a tiny kernel merges the partial pairs into ref_r = max_r + log2(sum_r);
//   pass 1  (rows x keys orientation: a lane owns one key)  streams K again, forms
//           p = exp2(s*scale*log2e - ref_r), sums it over the rows in registers, across the two lane
//           halves by one shuffle, across wavefronts in LDS, and reduces the per-token importance to
//           chunk sums with a fixed-order segmented sum in LDS (no atomics: results are deterministic).
// K tiles of 32 KB are copied global -> registers -> LDS with 16-byte accesses, double buffered; the
// 16-byte segments of a row are XOR-swizzled with the key index so that the MFMA operand reads
// (one 16-byte segment per lane, 32 different keys per instruction) are free of bank conflicts.
// The window queries stay in registers for the whole kernel.
#pragma once
#include "internal.h"

namespace ckv {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr float kNegBig = -1.0e30f;
constexpr int kScoreMiscBytes = 4096 + 1024;
constexpr int kScoreLdsBytes = 2 * kTileBytes + kScoreMiscBytes;

template <int DT>
__device__ __forceinline__ void mma(f32x16 &acc, const u32x4 &a, const u32x4 &b) {
  if constexpr (DT == CHUNKKV_BF16) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                  acc, 0, 0, 0);
  } else {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// DT: chunkkv_dtype, HD: head dim, NQW: 32-row blocks per wavefront, WQ: wavefronts splitting the rows
template <int DT, int HD, int NQW, int WQ, int PASS>
__global__ __launch_bounds__(kThreads, (NQW >= 4 ? 1 : 2)) void score_kernel(ScoreArgs a) {
  constexpr int ESZ = DT == CHUNKKV_BF16 ? 2 : 4;
  constexpr int ROWB = HD * ESZ;
  constexpr int NSEG = ROWB / 16;
  constexpr int NKS = ROWB / 32;
  constexpr int TK = kTileBytes / ROWB;
  constexpr int KBT = TK / 32;
  constexpr int WK = 4 / WQ;
  constexpr int LOADS = kTileBytes / 16 / kThreads;  // 16-byte loads per thread per tile (8)

  extern __shared__ __align__(16) char smem[];
  float *s_misc = (float *)(smem + 2 * kTileBytes);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, half = lane >> 5;
  const int wq = wave % WQ, wk = wave / WQ;
  const int bl = blockIdx.y / a.n_kv_heads, h = blockIdx.y % a.n_kv_heads, z = blockIdx.z;
  const int split = blockIdx.x;
  const int g = a.n_q_heads / a.n_kv_heads, w = a.window, c = a.chunk;
  const int L = pick(a.seq.seqlen, bl), P = L - w, nrows = g * w;
  const int64_t problem = ((int64_t)(a.leader0 + z) * a.batch_total + (a.batch0 + bl)) * a.n_kv_heads + h;

  const int stride = (PASS == 1 && a.fuse_chunks) ? (TK / c) * c : TK;  // keys a tile advances by
  const int span = PASS == 0 ? L : P;                                   // keys this pass must cover
  const int ntiles = (span + stride - 1) / stride;
  const int t0 = split * a.tiles_per_wg;
  const int t1 = t0 + a.tiles_per_wg < ntiles ? t0 + a.tiles_per_wg : ntiles;
  if (t0 >= ntiles) return;

  const char *qbase = (const char *)pick(a.q, z) + ((int64_t)(a.batch0 + bl) * a.n_q_heads + (int64_t)h * g) * w * ROWB;
  const char *kbase = (const char *)pick(a.k, z) + (pick(a.seq.kv_base, bl) + (int64_t)h * a.kv_stride_head) * ESZ;
  const int64_t ktok = a.kv_stride_tok * ESZ;
  const float c1 = a.scale_log2e;

  // window queries: operand fragments, resident for the whole kernel
  u32x4 qf[NQW][NKS];
#pragma unroll
  for (int qi = 0; qi < NQW; ++qi) {
    const int row = (wq * NQW + qi) * 32 + n;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      qf[qi][ks] = u32x4{0, 0, 0, 0};
      if (row < nrows) qf[qi][ks] = *(const u32x4 *)(qbase + (int64_t)row * ROWB + (2 * ks + half) * 16);
    }
  }

  // pass 0 state: running (max, sum) of the lane's row; pass 1 state: ref of the 16 rows a lane sees
  float m_run[NQW], l_run[NQW];
  int lim[NQW];
  float ref[NQW][16];
#pragma unroll
  for (int qi = 0; qi < NQW; ++qi) {
    m_run[qi] = kNegBig;
    l_run[qi] = 0.f;
    const int row = (wq * NQW + qi) * 32 + n;
    lim[qi] = P + (row < nrows ? row % w : 0);  // last key window row i may see
    if constexpr (PASS == 1) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = (wq * NQW + qi) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
        ref[qi][v] = r < nrows ? a.refs[problem * a.rows_pad + r] : 1.0e30f;
      }
    }
  }

  // One K tile in flight: LOADS 16-byte segments per thread, fetched before the current tile is
  // consumed and committed to the other LDS buffer afterwards.
  u32x4 stage[LOADS];
#define CKV_TILE_FETCH(tile)                                                                      \
  {                                                                                               \
    const int fk0 = (tile) * stride;                                                              \
    _Pragma("unroll") for (int j = 0; j < LOADS; ++j) {                                           \
      const int id = j * kThreads + tid, key = id / NSEG, seg = id % NSEG;                        \
      int gk = fk0 + key;                                                                         \
      gk = gk < L ? gk : L - 1; /* rows past the sequence are never read; results are masked */   \
      stage[j] = *(const u32x4 *)(kbase + (int64_t)gk * ktok + seg * 16);                         \
    }                                                                                             \
  }
#define CKV_TILE_COMMIT(buf)                                                                      \
  {                                                                                               \
    _Pragma("unroll") for (int j = 0; j < LOADS; ++j) {                                           \
      const int id = j * kThreads + tid, key = id / NSEG, seg = id % NSEG;                        \
      *(u32x4 *)((buf) + (key * NSEG + (seg ^ (key & 7))) * 16) = stage[j];                       \
    }                                                                                             \
  }

  CKV_TILE_FETCH(t0);
  CKV_TILE_COMMIT(smem);
  __syncthreads();

  for (int t = t0; t < t1; ++t) {
    const char *buf = smem + ((t - t0) & 1) * kTileBytes;
    const int key0 = t * stride;
    if (t + 1 < t1) CKV_TILE_FETCH(t + 1);

    for (int kb = wk; kb < KBT; kb += WK) {
      f32x16 acc[NQW];
#pragma unroll
      for (int qi = 0; qi < NQW; ++qi)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[qi][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
        const u32x4 kf = *(const u32x4 *)(buf + ((kb * 32 + n) * NSEG + ((2 * ks + half) ^ (n & 7))) * 16);
#pragma unroll
        for (int qi = 0; qi < NQW; ++qi) {
          if constexpr (PASS == 0) mma<DT>(acc[qi], kf, qf[qi][ks]);   // D[key][row]
          else mma<DT>(acc[qi], qf[qi][ks], kf);                       // D[row][key]
        }
      }

      if constexpr (PASS == 0) {
        // lane: row n of block qi; registers: keys kb*32 + 8*(v/4) + 4*half + v%4
        const bool masked = key0 + TK > P;
#pragma unroll
        for (int qi = 0; qi < NQW; ++qi) {
          if (masked) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              const int key = key0 + kb * 32 + 8 * (v / 4) + 4 * half + (v % 4);
              acc[qi][v] = key <= lim[qi] ? acc[qi][v] : -3.0e38f;
            }
          }
          float bm = acc[qi][0];
#pragma unroll
          for (int v = 1; v < 16; ++v) bm = fmaxf(bm, acc[qi][v]);
          const float m_new = fmaxf(m_run[qi], bm * c1);
          float sum = 0.f;
#pragma unroll
          for (int v = 0; v < 16; ++v) sum += fast_exp2(__builtin_fmaf(acc[qi][v], c1, -m_new));
          l_run[qi] = __builtin_fmaf(l_run[qi], fast_exp2(m_run[qi] - m_new), sum);
          m_run[qi] = m_new;
        }
      } else {
        // lane: key kb*32 + n; registers: rows 8*(v/4) + 4*half + v%4 of block qi
        float colsum = 0.f;
#pragma unroll
        for (int qi = 0; qi < NQW; ++qi)
#pragma unroll
          for (int v = 0; v < 16; ++v) colsum += fast_exp2(__builtin_fmaf(acc[qi][v], c1, -ref[qi][v]));
        colsum += __shfl_xor(colsum, 32);
        if (half == 0) s_misc[wq * TK + kb * 32 + n] = colsum;
      }
    }

    if constexpr (PASS == 1) {
      __syncthreads();
      float *s_imp = s_misc + 1024;  // TK <= 256 floats
      if (tid < TK) {
        float imp = 0.f;
#pragma unroll
        for (int q = 0; q < WQ; ++q) imp += s_misc[q * TK + tid];
        const int key = key0 + tid;
        const bool owned = tid < stride && key < P;
        imp = owned ? imp : 0.f;
        s_imp[tid] = imp;
        if (owned && a.token_imp) a.token_imp[problem * a.imp_pitch + key] = imp;
      }
      if (a.fuse_chunks) {
        __syncthreads();
        const int nch = stride / c;
        if (tid < nch) {
          const int cidx = key0 / c + tid;
          if ((int64_t)cidx * c < P) {
            float sum = 0.f;
            for (int i = 0; i < c; ++i) sum += s_imp[tid * c + i];
            a.chunk_scores[problem * a.score_cap + cidx] = sum;
          }
        }
      }
    }

    if (t + 1 < t1) CKV_TILE_COMMIT(smem + (((t - t0) & 1) ^ 1) * kTileBytes);
    __syncthreads();
  }

  if constexpr (PASS == 0) {
    float2 *s_st = (float2 *)s_misc;  // [4 wavefronts][32 rows]
#pragma unroll
    for (int qi = 0; qi < NQW; ++qi) {
      // merge the two lane halves (same row, different keys)
      const float m_o = __shfl_xor(m_run[qi], 32), l_o = __shfl_xor(l_run[qi], 32);
      float m = fmaxf(m_run[qi], m_o);
      float l = l_run[qi] * fast_exp2(m_run[qi] - m) + l_o * fast_exp2(m_o - m);
      if constexpr (WK > 1) {
        // NQW == 1 here: merge the wavefronts that split the keys
        if (half == 0) s_st[wave * 32 + n] = make_float2(m, l);
        __syncthreads();
        if (wk == 0) {
          for (int o = 1; o < WK; ++o) {
            const float2 x = s_st[(o * WQ + wq) * 32 + n];
            const float mm = fmaxf(m, x.x);
            l = l * fast_exp2(m - mm) + x.y * fast_exp2(x.x - mm);
            m = mm;
          }
        }
      }
      if (wk == 0 && half == 0) {
        const int row = (wq * NQW + qi) * 32 + n;
        a.part_stats[(problem * a.max_split + split) * a.rows_pad + row] = make_float2(m, l);
      }
    }
  }
}

#undef CKV_TILE_FETCH
#undef CKV_TILE_COMMIT

template <int DT, int HD, int NQW, int WQ>
int launch_score_cfg(int pass, const ScoreArgs &a, dim3 grid, hipStream_t s) {
  static bool attr_done[2] = {false, false};
  auto k0 = score_kernel<DT, HD, NQW, WQ, 0>;
  auto k1 = score_kernel<DT, HD, NQW, WQ, 1>;
  auto kern = pass == 0 ? k0 : k1;
  if (!attr_done[pass]) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            kScoreLdsBytes) != hipSuccess)
      return CHUNKKV_ERR_LAUNCH;
    attr_done[pass] = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(kThreads), kScoreLdsBytes, s, a);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

template <int DT, int HD>
int launch_score_hd(int pass, const ScoreGeom &g, const ScoreArgs &a, dim3 grid, hipStream_t s) {
  if (g.nqw == 1 && g.wq == 1) return launch_score_cfg<DT, HD, 1, 1>(pass, a, grid, s);
  if (g.nqw == 1 && g.wq == 2) return launch_score_cfg<DT, HD, 1, 2>(pass, a, grid, s);
  if (g.nqw == 1 && g.wq == 4) return launch_score_cfg<DT, HD, 1, 4>(pass, a, grid, s);
  if (g.nqw == 2 && g.wq == 4) return launch_score_cfg<DT, HD, 2, 4>(pass, a, grid, s);
  if constexpr (!(DT == CHUNKKV_F32 && HD == 128)) {
    if (g.nqw == 4 && g.wq == 4) return launch_score_cfg<DT, HD, 4, 4>(pass, a, grid, s);
  }
  return CHUNKKV_ERR_UNSUPPORTED;
}

}  // namespace ckv
