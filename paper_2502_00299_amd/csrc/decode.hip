// Decoding over the (compressed) cache: one new query token per head attends to every token of K', V'
// (the stage whose cache Eq. 1 sizes and whose latency Section 4.4 tabulates; Algorithm 1's output is its
// input).  out_i = sum_t softmax_t(scale * q_i . k_t) v_t, query head i reading kv-head i / g.
//
// Bound by HBM bandwidth: every K and V row is read once, g dot products and g axpys per row are far below
// the vector ALU's rate, so this is a streaming kernel on the vector ALU, not a matrix-core kernel.  A row
// (d elements) is spread over LPR = d * element size / 16 lanes, 16 bytes each, so one load instruction of
// a wavefront reads 64 / LPR consecutive rows as one contiguous piece.  The lanes of a row reduce their
// partial dot products with DPP adds (no LDS).  Each group of LPR lanes runs its own online softmax over the
// rows it meets; the groups of a wavefront, the wavefronts of a workgroup and the key ranges of a head are
// merged afterwards by the usual (max, sum, weighted output) rule, always in the same order.
// With 16 lanes per row and 4 or 8 heads per workgroup the 4 x G partial dot products of a step are not
// all-reduced but reduce-scattered: the lanes hold them in an order permuted by their own index (the rows
// they load and the heads they keep in registers are XOR-swizzled), so each of the four halving steps is
// one DPP add per kept value and lane (4u + jb) of a row group ends with the complete scores of row u for
// heads jb*G/4 .. jb*G/4 + G/4 - 1.  That lane alone does the softmax arithmetic of those scores; the
// weights reach the 16 lanes again as DPP row broadcasts feeding the value accumulation.
// Grid: x = key range, y = (sequence, kv-head), z = batch of G query heads of the kv-head.
#include <type_traits>
#include <utility>

#include "internal.h"

namespace ckv {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr int kDecodeUnroll = 4;        // row loads of K (and of V) in flight per lane
constexpr float kDecodeNegBig = -1.0e30f;

template <int CTRL>
__device__ __forceinline__ float dpp_add(float x) {
  return x + __builtin_amdgcn_update_dpp(0.f, x, CTRL, 0xf, 0xf, false);
}
// Sum over the LPR lanes that share a row; every lane of the group ends with the same bits.
template <int LPR>
__device__ __forceinline__ float row_sum(float x) {
  x = dpp_add<0xB1>(x);                          // quad_perm [1,0,3,2]
  x = dpp_add<0x4E>(x);                          // quad_perm [2,3,0,1]
  if constexpr (LPR >= 8) x = dpp_add<0x141>(x);   // row_half_mirror: the other quad of 8 lanes
  if constexpr (LPR >= 16) x = dpp_add<0x140>(x);  // row_mirror: the other half of 16 lanes
  if constexpr (LPR >= 32) x += __shfl_xor(x, 16);
  return x;
}

template <int CTRL>
__device__ __forceinline__ float dpp_get(float x) {
  return __builtin_amdgcn_update_dpp(0.f, x, CTRL, 0xf, 0xf, false);
}
// value of lane N of every row of 16 lanes
template <int N>
__device__ __forceinline__ float row_bcast(float x) {
  return dpp_get<0x150 + N>(x);  // row_newbcast:N
}
template <int... I, typename F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, I...>, F f) {
  (f(std::integral_constant<int, I>{}), ...);
}

// 16 bytes of a row as fp32 values (8 for the 16-bit types, 4 for fp32)
template <int DT>
__device__ __forceinline__ void widen16(const u32x4 &r, float (&f)[16 / (DT == CHUNKKV_F32 ? 4 : 2)]) {
  if constexpr (DT == CHUNKKV_F32) {
    f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y); f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
  } else if constexpr (DT == CHUNKKV_BF16) {
    const uint32_t d[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { f[2 * i] = __uint_as_float(d[i] << 16); f[2 * i + 1] = __uint_as_float(d[i] & 0xFFFF0000u); }
  } else {
    const uint32_t d[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const f16x2 h = __builtin_bit_cast(f16x2, d[i]);
      f[2 * i] = (float)h[0]; f[2 * i + 1] = (float)h[1];
    }
  }
}

// partial dot product of a lane's 16 bytes of a K row with its 16 bytes of a query row
template <int DT>
__device__ __forceinline__ float dot16(const u32x4 &k, const u32x4 &q) {
  if constexpr (DT == CHUNKKV_F32) {
    float s = __uint_as_float(k.x) * __uint_as_float(q.x);
    s = __builtin_fmaf(__uint_as_float(k.y), __uint_as_float(q.y), s);
    s = __builtin_fmaf(__uint_as_float(k.z), __uint_as_float(q.z), s);
    return __builtin_fmaf(__uint_as_float(k.w), __uint_as_float(q.w), s);
  } else if constexpr (DT == CHUNKKV_BF16) {
    // the pairs are taken from whole-vector casts: a bit cast of a single vector element reads element 0
    const bf16x8 kk = __builtin_bit_cast(bf16x8, k), qq = __builtin_bit_cast(bf16x8, q);
    float s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(kk, kk, 0, 1), __builtin_shufflevector(qq, qq, 0, 1), 0.f, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(kk, kk, 2, 3), __builtin_shufflevector(qq, qq, 2, 3), s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(kk, kk, 4, 5), __builtin_shufflevector(qq, qq, 4, 5), s, false);
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(kk, kk, 6, 7), __builtin_shufflevector(qq, qq, 6, 7), s, false);
  } else {
    const f16x8 kk = __builtin_bit_cast(f16x8, k), qq = __builtin_bit_cast(f16x8, q);
    float s = __builtin_amdgcn_fdot2(__builtin_shufflevector(kk, kk, 0, 1), __builtin_shufflevector(qq, qq, 0, 1), 0.f, false);
    s = __builtin_amdgcn_fdot2(__builtin_shufflevector(kk, kk, 2, 3), __builtin_shufflevector(qq, qq, 2, 3), s, false);
    s = __builtin_amdgcn_fdot2(__builtin_shufflevector(kk, kk, 4, 5), __builtin_shufflevector(qq, qq, 4, 5), s, false);
    return __builtin_amdgcn_fdot2(__builtin_shufflevector(kk, kk, 6, 7), __builtin_shufflevector(qq, qq, 6, 7), s, false);
  }
}

// DT: chunkkv_dtype, HD: head dim, G: query heads of the kv-head handled by one workgroup
template <int DT, int HD, int G>
__global__ __launch_bounds__(kThreads) void decode_kernel(DecodeArgs a) {
  constexpr int ESZ = DT == CHUNKKV_F32 ? 4 : 2;
  constexpr int ROWB = HD * ESZ;
  constexpr int LPR = ROWB / 16;   // lanes per row
  constexpr int RPW = 64 / LPR;    // rows per wavefront load
  constexpr int EPL = 16 / ESZ;    // elements per lane
  constexpr int U = kDecodeUnroll;
  constexpr int NW = kThreads / 64;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int grp = lane / LPR, seg = lane % LPR;
  const int bl = blockIdx.y / a.n_kv_heads, h = blockIdx.y % a.n_kv_heads;
  const int split = blockIdx.x;
  const int g = a.n_q_heads / a.n_kv_heads;
  const int j0 = blockIdx.z * G;  // first query head (within the kv-head's group) of this workgroup
  const int b = a.batch0 + bl;

  // tokens of this (sequence, kv-head): the capacity of the cache, or the caller's count clamped to it
  const int cap = pick(a.n_tok, bl);
  int n = cap;
  if (a.kv_len != nullptr) {
    n = a.kv_len[(int64_t)b * a.n_kv_heads + h];
    n = n < 0 ? 0 : (n > cap ? cap : n);
  }
  const int r0 = split * a.rows_per_split;
  const int r1 = r0 + a.rows_per_split < n ? r0 + a.rows_per_split : n;

  const int64_t head_off = (pick(a.base, bl) + (int64_t)h * a.stride_head) * ESZ;
  const char *kbase = (const char *)a.k + head_off + seg * 16;
  const char *vbase = (const char *)a.v + head_off + seg * 16;
  const int64_t tok = a.stride_tok * ESZ;

  // reduce-scatter variant (see the file header): lane (4 * ub + jb) of a row group owns row ub, heads jb * NR ..
  constexpr bool kScatter = LPR == 16 && U == 4 && (G == 4 || G == 8);
  constexpr int LG = G == 8 ? 3 : 2;   // log2(G) where the variant applies
  constexpr int NR = kScatter ? G / 4 : 1;
  const int ub = kScatter ? (lane & 15) >> 2 : 0, jb = kScatter ? lane & 3 : 0;
  const int jsw = jb << (LG - 2);      // register j holds head j ^ jsw

  u32x4 qreg[G];
#pragma unroll
  for (int j = 0; j < G; ++j) {
    const int jh = j ^ jsw;
    qreg[j] = u32x4{0, 0, 0, 0};
    if (j0 + jh < g)
      qreg[j] = *(const u32x4 *)((const char *)a.q + ((int64_t)b * a.n_q_heads + (int64_t)h * g + j0 + jh) * ROWB + seg * 16);
  }
  float m_own[NR], l_own[NR];          // scatter variant: statistics of the heads this lane owns
#pragma unroll
  for (int x = 0; x < NR; ++x) { m_own[x] = kDecodeNegBig; l_own[x] = 0.f; }
  float m[G], l[G], o[G][EPL];
#pragma unroll
  for (int j = 0; j < G; ++j) {
    m[j] = kDecodeNegBig;
    l[j] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) o[j][e] = 0.f;
  }
  const float c1 = a.scale_log2e;

  // rows r0 .. r1-1; a step of the workgroup covers NW * U * RPW consecutive rows
  for (int base = r0 + wave * (U * RPW); base < r1; base += NW * U * RPW) {
    u32x4 kr[U], vr[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int rowv = base + u * RPW + grp;           // V: register u holds row u
      const int rowk = base + (u ^ ub) * RPW + grp;    // K: register u holds row u ^ ub (ub = 0 without the swizzle)
      // every row is read once: streaming (non-temporal) loads
      kr[u] = __builtin_nontemporal_load((const u32x4 *)(kbase + (int64_t)(rowk < r1 ? rowk : r1 - 1) * tok));  // r1 >= 1 inside the loop
      vr[u] = __builtin_nontemporal_load((const u32x4 *)(vbase + (int64_t)(rowv < r1 ? rowv : r1 - 1) * tok));
    }
    if constexpr (kScatter) {
      float x[U][G];
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int jj = 0; jj < G; ++jj) x[u][jj] = dot16<DT>(kr[u], qreg[jj]);
      // four halving steps; the partner lane differs in bit 3 / bits 0-2 / bit 1 / bit 0 of the lane index
      constexpr int J3 = 3 << (LG - 2);
      float y[2][G], z[G], t[G / 2], r[NR];
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int jj = 0; jj < G; ++jj) y[u][jj] = x[u][jj] + dpp_get<0x128>(x[u ^ 2][jj]);   // row_ror:8
#pragma unroll
      for (int jj = 0; jj < G; ++jj) z[jj] = y[0][jj] + dpp_get<0x141>(y[1][jj ^ J3]);        // row_half_mirror
#pragma unroll
      for (int jj = 0; jj < G / 2; ++jj) t[jj] = z[jj] + dpp_get<0x4E>(z[jj ^ (G / 2)]);      // quad_perm [2,3,0,1]
#pragma unroll
      for (int jj = 0; jj < NR; ++jj) r[jj] = t[jj] + dpp_get<0xB1>(t[jj ^ (G / 4)]);         // quad_perm [1,0,3,2]
      // r[x]: row ub of the step, head jb * NR + x.  Softmax statistics per head: maximum over the four rows,
      // which sit in the lanes 4, 8 and 12 further on.
      const bool valid_own = base + ub * RPW + grp < r1;
      float p[NR];
#pragma unroll
      for (int xx = 0; xx < NR; ++xx) {
        const float sc = valid_own ? r[xx] * c1 : -3.0e38f;
        float smax = fmaxf(sc, dpp_get<0x128>(sc));
        smax = fmaxf(smax, dpp_get<0x124>(smax));   // row_ror:4; the value is already the same 8 lanes apart
        if (__builtin_amdgcn_ballot_w64(smax > m_own[xx]) != 0) {
          const float m_new = fmaxf(m_own[xx], smax);
          const float f = __builtin_amdgcn_exp2f(m_own[xx] - m_new);
          l_own[xx] *= f;
          m_own[xx] = m_new;
          // the outputs of head jbp * NR + xx live in all 16 lanes: its factor comes from lane jbp
          static_for(std::make_integer_sequence<int, 4>{}, [&](auto jbp_c) __attribute__((always_inline)) {
            constexpr int JBP = decltype(jbp_c)::value;
            const float fb = row_bcast<JBP>(f);
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[JBP * NR + xx][e] *= fb;
          });
        }
        p[xx] = __builtin_amdgcn_exp2f(sc - m_own[xx]);
        l_own[xx] += p[xx];
      }
      static_for(std::make_integer_sequence<int, U>{}, [&](auto u_c) __attribute__((always_inline)) {
        constexpr int UU = decltype(u_c)::value;
        float vf[EPL];
        widen16<DT>(vr[UU], vf);
        static_for(std::make_integer_sequence<int, G>{}, [&](auto j_c) __attribute__((always_inline)) {
          constexpr int JJ = decltype(j_c)::value;
          const float pb = row_bcast<4 * UU + JJ / NR>(p[JJ % NR]);   // weight of (row UU, head JJ)
#pragma unroll
          for (int e = 0; e < EPL; ++e) o[JJ][e] = __builtin_fmaf(pb, vf[e], o[JJ][e]);
        });
      });
    } else {
      float s[U][G];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool valid = base + u * RPW + grp < r1;
#pragma unroll
        for (int jj = 0; jj < G; ++jj) {
          const float d = row_sum<LPR>(dot16<DT>(kr[u], qreg[jj]));
          s[u][jj] = valid ? d * c1 : -3.0e38f;
        }
      }
#pragma unroll
      for (int jj = 0; jj < G; ++jj) {
        float smax = s[0][jj];
#pragma unroll
        for (int u = 1; u < U; ++u) smax = fmaxf(smax, s[u][jj]);
        if (__builtin_amdgcn_ballot_w64(smax > m[jj]) != 0) {
          const float m_new = fmaxf(m[jj], smax);
          const float f = __builtin_amdgcn_exp2f(m[jj] - m_new);
          l[jj] *= f;
#pragma unroll
          for (int e = 0; e < EPL; ++e) o[jj][e] *= f;
          m[jj] = m_new;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) s[u][jj] = __builtin_amdgcn_exp2f(s[u][jj] - m[jj]);  // now the weight p
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        float vf[EPL];
        widen16<DT>(vr[u], vf);
#pragma unroll
        for (int jj = 0; jj < G; ++jj) {
          l[jj] += s[u][jj];
#pragma unroll
          for (int e = 0; e < EPL; ++e) o[jj][e] = __builtin_fmaf(s[u][jj], vf[e], o[jj][e]);
        }
      }
    }
  }
  if constexpr (kScatter) {
    // back to the replicated form the merges below expect: every lane learns (m, l) of every head
    float lsum[NR];
#pragma unroll
    for (int xx = 0; xx < NR; ++xx) {
      lsum[xx] = l_own[xx] + dpp_get<0x128>(l_own[xx]);
      lsum[xx] += dpp_get<0x124>(lsum[xx]);
    }
    static_for(std::make_integer_sequence<int, G>{}, [&](auto j_c) __attribute__((always_inline)) {
      constexpr int JJ = decltype(j_c)::value;
      m[JJ] = row_bcast<JJ / NR>(m_own[JJ % NR]);
      l[JJ] = row_bcast<JJ / NR>(lsum[JJ % NR]);
    });
  }

  // merge the row groups of the wavefront (lanes that hold the same 16 bytes of the row)
#pragma unroll
  for (int x = LPR; x < 64; x *= 2) {
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const float m_o = __shfl_xor(m[j], x), l_o = __shfl_xor(l[j], x);
      const float M = fmaxf(m[j], m_o);
      const float fa = __builtin_amdgcn_exp2f(m[j] - M), fb = __builtin_amdgcn_exp2f(m_o - M);
      l[j] = l[j] * fa + l_o * fb;
#pragma unroll
      for (int e = 0; e < EPL; ++e) o[j][e] = o[j][e] * fa + __shfl_xor(o[j][e], x) * fb;
      m[j] = M;
    }
  }
  // merge the wavefronts through LDS: thread (j, seg) folds the four states in wavefront order
  __shared__ float s_m[NW][G][LPR], s_l[NW][G][LPR], s_o[NW][G][LPR][EPL];
  if (grp == 0) {
#pragma unroll
    for (int j = 0; j < G; ++j) {
      s_m[wave][j][seg] = m[j];
      s_l[wave][j][seg] = l[j];
#pragma unroll
      for (int e = 0; e < EPL; ++e) s_o[wave][j][seg][e] = o[j][e];
    }
  }
  __syncthreads();
  const int t = threadIdx.x;
  if (t < G * LPR) {
    const int j = t / LPR, sg = t % LPR;
    if (j0 + j < g) {
      float M = s_m[0][j][sg];
#pragma unroll
      for (int w = 1; w < NW; ++w) M = fmaxf(M, s_m[w][j][sg]);
      float Lsum = 0.f, acc[EPL];
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] = 0.f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        const float f = __builtin_amdgcn_exp2f(s_m[w][j][sg] - M);
        Lsum += s_l[w][j][sg] * f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] += s_o[w][j][sg][e] * f;
      }
      const int64_t head = (int64_t)b * a.n_q_heads + (int64_t)h * g + j0 + j;
      const int64_t slot = head * a.n_split + split;
      if (sg == 0) a.part_ml[slot] = make_float2(M, Lsum);
      float *po = a.part_o + slot * HD + sg * EPL;
#pragma unroll
      for (int e = 0; e < EPL; ++e) po[e] = acc[e];
    }
  }
}

// out = sum_s o_s 2^(m_s - M) / sum_s l_s 2^(m_s - M) over the key ranges of one query head.
// grid: x = query head of the batch slice; 256 threads: a thread owns four consecutive output elements
// and every kCombineGroups-th key range; the groups are folded through LDS in group order, so the
// summation order is fixed.
constexpr int kCombineThreads = 256;
template <int HD>
__global__ __launch_bounds__(kCombineThreads) void decode_combine_kernel(DecodeArgs a) {
  constexpr int TPR = HD / 4;                     // threads per partial row
  constexpr int NG = kCombineThreads / TPR;       // key-range groups
  const int64_t head = (int64_t)a.batch0 * a.n_q_heads + blockIdx.x;
  const float2 *ml = a.part_ml + head * a.n_split;
  const int t = threadIdx.x, col = t % TPR, grp = t / TPR;
  __shared__ float s_red[kCombineThreads / 64];
  __shared__ float s_acc[NG][HD + 1];
  // maximum over the key ranges
  float M = kDecodeNegBig;
  for (int s = t; s < a.n_split; s += kCombineThreads) M = fmaxf(M, ml[s].x);
  for (int o = 32; o > 0; o >>= 1) M = fmaxf(M, __shfl_xor(M, o));
  if ((t & 63) == 0) s_red[t >> 6] = M;
  __syncthreads();
  M = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
  // weighted sums of this thread's key ranges
  const float *po = a.part_o + head * a.n_split * HD + col * 4;
  float acc[4] = {0.f, 0.f, 0.f, 0.f}, lsum = 0.f;
#pragma unroll 4
  for (int s = grp; s < a.n_split; s += NG) {
    const float2 p = ml[s];
    const float f = __builtin_amdgcn_exp2f(p.x - M);
    const float4 o4 = *(const float4 *)(po + (int64_t)s * HD);
    lsum += p.y * f;
    acc[0] += o4.x * f; acc[1] += o4.y * f; acc[2] += o4.z * f; acc[3] += o4.w * f;
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) s_acc[grp][col * 4 + e] = acc[e];
  if (col == 0) s_acc[grp][HD] = lsum;
  __syncthreads();
  if (t < HD) {
    float v = 0.f, Lsum = 0.f;
#pragma unroll
    for (int g2 = 0; g2 < NG; ++g2) { v += s_acc[g2][t]; Lsum += s_acc[g2][HD]; }
    a.out[head * HD + t] = Lsum > 0.f ? v / Lsum : 0.f;
    if (a.lse != nullptr && t == 0)
      a.lse[head] = Lsum > 0.f ? (M + __builtin_log2f(Lsum)) * 0.6931471805599453f : -__builtin_inff();
  }
}

template <int DT, int HD>
int launch_decode_hd(const DecodeArgs &a, int batch_slice, int g, hipStream_t s) {
  const int G = decode_heads_per_wg(DT, g);
  const dim3 grid(a.n_split, batch_slice * a.n_kv_heads, (g + G - 1) / G);
  if (grid.x == 0 || grid.y == 0) return CHUNKKV_OK;
  if (G == 1) hipLaunchKernelGGL((decode_kernel<DT, HD, 1>), grid, dim3(kThreads), 0, s, a);
  else if (G == 2) hipLaunchKernelGGL((decode_kernel<DT, HD, 2>), grid, dim3(kThreads), 0, s, a);
  else if (G == 4) hipLaunchKernelGGL((decode_kernel<DT, HD, 4>), grid, dim3(kThreads), 0, s, a);
  else if constexpr (DT != CHUNKKV_F32) hipLaunchKernelGGL((decode_kernel<DT, HD, 8>), grid, dim3(kThreads), 0, s, a);
  else return CHUNKKV_ERR_UNSUPPORTED;
  if (hipGetLastError() != hipSuccess) return CHUNKKV_ERR_LAUNCH;
  hipLaunchKernelGGL((decode_combine_kernel<HD>), dim3(batch_slice * a.n_q_heads), dim3(kCombineThreads), 0, s, a);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

int launch_decode(int dtype, int head_dim, const DecodeArgs &a, int batch_slice, hipStream_t s) {
  const int g = a.n_q_heads / a.n_kv_heads;
  if (head_dim == 128) {
    if (dtype == CHUNKKV_BF16) return launch_decode_hd<CHUNKKV_BF16, 128>(a, batch_slice, g, s);
    if (dtype == CHUNKKV_F16) return launch_decode_hd<CHUNKKV_F16, 128>(a, batch_slice, g, s);
    if (dtype == CHUNKKV_F32) return launch_decode_hd<CHUNKKV_F32, 128>(a, batch_slice, g, s);
  } else if (head_dim == 64) {
    if (dtype == CHUNKKV_BF16) return launch_decode_hd<CHUNKKV_BF16, 64>(a, batch_slice, g, s);
    if (dtype == CHUNKKV_F16) return launch_decode_hd<CHUNKKV_F16, 64>(a, batch_slice, g, s);
    if (dtype == CHUNKKV_F32) return launch_decode_hd<CHUNKKV_F32, 64>(a, batch_slice, g, s);
  }
  return CHUNKKV_ERR_UNSUPPORTED;
}

}  // namespace ckv
