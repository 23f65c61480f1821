// Single-pass observation-window scoring (Algorithm 1, first two steps) for bf16 caches.
//
// K is streamed ONCE.  The kernel is an attention forward pass whose "value" matrix is the 0/1 indicator
// of chunk membership: for every window row r and every key block it keeps a running maximum m_r
// (online softmax), forms e = exp2(logit*scale*log2e - m_r) and multiplies the block's e values (cast to
// fp16, scaled by 2^12) with the indicator block on the matrix cores, so the accumulator holds, per row,
// the sum of e over each chunk of the current PERIOD of lcm(32, c) keys (at most 16 chunk slots).
// The accumulators are rescaled by exp2(old maximum - new maximum) every block (branch-free; the factor
// is 1 unless the maximum grew).  At the end of a period the per-(chunk, row) sums E and the maximum
// they are relative to are written out; the row's total sum follows from the E sums (plus the window
// keys, which belong to no chunk).  Afterwards a merge kernel turns the per-range (max, sum) pairs into
// ref_r = max_r + log2(sum_r) and a small reduction kernel forms
//     score[chunk] = sum_r E[chunk][r] * exp2(m_period[r] - ref_r).
// Nothing is approximated except the fp16 rounding of e (relative 2^-11, the same values feed numerator
// and denominator); chunk scores stay well inside the 1e-3 tolerance.
//
// Streaming, ring, swizzle and software pipelining are those of the two-pass kernels (score_impl.h): a
// step issues the 16 bf16 MFMAs of block b, the LDS reads of block b+1's fragments, and block b-1's
// exp / pack / indicator-MFMA epilogue as one scheduled region.  Every wavefront owns its 32*NQW rows
// for all keys of the workgroup's range, so there is no cross-wavefront reduction and no barrier besides
// the ring's.
#pragma once
#include "score_impl.h"

namespace ckv {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kFusedTableBytes = 6144;  // indicator fragments: phases * 2 * 2 * (nslots + 1) * 16 B
constexpr int kFusedLdsBytes = kRing * kTileBytes + kFusedTableBytes;
constexpr float kHalfShift = 12.f;      // e is scaled by 2^12 before the fp16 cast (<= 4096, denormals below 2^-26)

template <int HD, int NQW>
__global__ __launch_bounds__(kThreads, (NQW >= 4 ? 1 : 2)) void score_fused_kernel(ScoreArgs a) {
  constexpr int ROWB = HD * 2;
  constexpr int NSEG = ROWB / 16;
  constexpr int NKS = ROWB / 32;
  constexpr int TK = kTileBytes / ROWB;
  constexpr int KBT = TK / 32;
  constexpr int DT = CHUNKKV_BF16;
  constexpr int ESZ_BF16 = 2;

  extern __shared__ __align__(16) char smem[];
  char *s_tab = smem + kRing * kTileBytes;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, half = lane >> 5;
  const int wq = wave;  // four wavefronts split the rows
  const int bl = blockIdx.y / a.n_kv_heads, h = blockIdx.y % a.n_kv_heads, z = blockIdx.z;
  const int split = blockIdx.x;
  const int g = a.n_q_heads / a.n_kv_heads, w = a.window, c = a.chunk;
  const int L = pick(a.seq.seqlen, bl), P = L - w, nrows = g * w;
  const int64_t problem = ((int64_t)(a.leader0 + z) * a.batch_total + (a.batch0 + bl)) * a.n_kv_heads + h;

  const int pk = a.period_keys, phases = pk / 32, nslots = pk / c, U = a.unit_keys;
  const int nunits = (L + U - 1) / U;
  const int u0 = split * a.tiles_per_wg;
  const int u1 = u0 + a.tiles_per_wg < nunits ? u0 + a.tiles_per_wg : nunits;
  if (u0 >= nunits) return;
  const int range0 = u0 * U;                                   // first key of this workgroup (multiple of pk)
  const int range_keys = (u1 * U < L ? u1 * U : L) - range0;
  const int nt = (range_keys + TK - 1) / TK;
  const int nblk = (range_keys + 31) / 32;  // key blocks that hold at least one key of the sequence

  const char *qbase = (const char *)pick(a.q, z) + ((int64_t)(a.batch0 + bl) * a.n_q_heads + (int64_t)h * g) * w * ROWB;
  const char *kbase = (const char *)pick(a.k, z) + (pick(a.seq.kv_base, bl) + (int64_t)h * a.kv_stride_head) * ESZ_BF16;
  const int64_t ktok = a.kv_stride_tok * ESZ_BF16;
  const float c1 = a.scale_log2e;

  // ---- K tiles: HBM -> LDS ring (see score_impl.h)
  auto issue_tile = [&](int i) __attribute__((always_inline)) {
    const int fk0 = range0 + i * TK;
    char *slot = smem + (i % kRing) * kTileBytes;
    if (fk0 + TK <= L) {
      const char *tbase = kbase + (int64_t)fk0 * ktok;
#pragma unroll
      for (int j = 0; j < kLoadsPerWave; ++j) {
        const int key = (wave * kLoadsPerWave + j) * (1024 / ROWB) + lane / NSEG, segp = lane % NSEG;
        const uint32_t lane_off = (uint32_t)(key * (int)ktok + ((segp ^ (key & 7)) * 16));
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(tbase + lane_off),
                                         (__attribute__((address_space(3))) void *)(slot + (wave * kLoadsPerWave + j) * 1024),
                                         16, 0, 0);
      }
    } else {
#pragma unroll
      for (int j = 0; j < kLoadsPerWave; ++j) {
        const int grp = wave * kLoadsPerWave + j;
        const int key = grp * (1024 / ROWB) + lane / NSEG, segp = lane % NSEG;
        int gk = fk0 + key;
        gk = gk < L ? gk : L - 1;
        const char *src = kbase + (int64_t)gk * ktok + ((segp ^ (key & 7)) * 16);
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)src,
                                         (__attribute__((address_space(3))) void *)(slot + grp * 1024), 16, 0, 0);
      }
    }
  };
  // tile i has landed once at most `newer` tile loads issued after it are outstanding
  auto wait_tile = [&](int newer) __attribute__((always_inline)) {
    if (newer >= 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * kLoadsPerWave));
    else if (newer == 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kLoadsPerWave));
    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  };
#pragma unroll
  for (int s = 0; s < kRing - 1; ++s)
    if (s < nt) issue_tile(s);

  // ---- indicator fragments.  Entry (phase, j, kgroup, slot) holds, for the 8 k-positions e of MFMA j
  // and lane half kgroup, 1.0 where the key of accumulator register 8j+e (block-relative key
  // 8*((8j+e)/4) + 4*kgroup + (8j+e)%4) belongs to chunk slot `slot` of the period; slot == nslots is zero.
  {
    const int entries = phases * 4 * (nslots + 1);
    for (int en = tid; en < entries; en += kThreads) {
      const int slot = en % (nslots + 1), kg = (en / (nslots + 1)) & 1, j = (en / (2 * (nslots + 1))) & 1;
      const int phase = en / (4 * (nslots + 1));
      f16x8 v;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int r = 8 * j + e;
        const int key = phase * 32 + 8 * (r / 4) + 4 * kg + (r % 4);
        v[e] = (slot < nslots && key / c == slot) ? (_Float16)1.0f : (_Float16)0.0f;
      }
      *(f16x8 *)(s_tab + en * 16) = v;
    }
  }
  // lane's table offset when its slot row n serves an even (rows 0..15) or an odd (rows 16..31) row block
  const int lane_tab_even = (half * (nslots + 1) + (n < nslots ? n : nslots)) * 16;
  const int lane_tab_odd = (half * (nslots + 1) + ((n >= 16 && n - 16 < nslots) ? n - 16 : nslots)) * 16;
  const int tab_stride = 2 * (nslots + 1) * 16;  // bytes between consecutive (phase, j)

  // ---- window queries, running statistics
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
  float m_run[NQW], l_run[NQW];  // l_run: this lane half's share of the row sum, relative to m_run
  // Indicator accumulators.  A 32x32 tile has 32 slot rows but a period has at most 16 chunk slots, so two
  // row blocks share one tile: block qi uses slot rows 16*(qi%2).., i.e. registers 8*(qi%2) + 0..7
  // (register 8*(qi%2) + v <-> chunk slot 8*(v/4) + 4*half + v%4 for v < 8).
  constexpr int NA = (NQW + 1) / 2;
  f32x16 acc2[NA];
#pragma unroll
  for (int qi = 0; qi < NQW; ++qi) {
    m_run[qi] = kNegBig;
    l_run[qi] = 0.f;
  }
#pragma unroll
  for (int i = 0; i < NA; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc2[i][v] = 0.f;

  auto frag_ptr = [&](int b, int ks) __attribute__((always_inline)) {
    const char *buf = smem + ((b / KBT) % kRing) * kTileBytes;
    const int kb = b % KBT;
    return (const u32x4 *)(buf + ((kb * 32 + n) * NSEG + ((2 * ks + half) ^ (n & 7))) * 16);
  };
  auto block_key0 = [&](int b) __attribute__((always_inline)) { return range0 + b * 32; };
  auto block_masked = [&](int b) __attribute__((always_inline)) { return block_key0(b) + 32 > P; };

  // The pipeline advances in micro-steps t = b * NQW + qi (key block b, row block qi of this
  // wavefront).  A micro-step finishes the previous one's logits in three parts:
  // part 1: new running maximum of the row; rescale what is relative to the old one
  auto update_max = [&](f32x16 &acc, int b, auto qi_c, auto masked_c) __attribute__((always_inline)) {
    constexpr int QI = decltype(qi_c)::value;
    constexpr bool MASKED = decltype(masked_c)::value;
    if constexpr (MASKED) {
      // only the last blocks of a sequence come here: the row's last visible key is recomputed
      const int k0 = block_key0(b) + 4 * half;
      const int row = (wq * NQW + QI) * 32 + n;
      const int lim = P + (row < nrows ? row % w : 0);
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = k0 + 8 * (v / 4) + (v % 4) <= lim ? acc[v] : -3.0e38f;
    }
    float bm = acc[0];
#pragma unroll
    for (int v = 1; v < 16; ++v) bm = fmaxf(bm, acc[v]);
    // both lane halves of a row share one reference: exchange across the halves without LDS
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(bm), __float_as_uint(bm), false, false);
    bm = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    const float m_new = fmaxf(m_run[QI], bm * c1);
    // rescale what was accumulated relative to the old maximum (factor 1 when it did not grow);
    // branch-free so that this, the MFMAs and the exponentials form one scheduled region
    const float f = fast_exp2(m_run[QI] - m_new);
#pragma unroll
    for (int v = 0; v < 8; ++v) acc2[QI / 2][8 * (QI % 2) + v] *= f;
    l_run[QI] *= f;
    m_run[QI] = m_new;
  };
  // part 2 (inside the region): e = exp2(...), fp16 pack, two indicator MFMAs
  auto accumulate = [&](f32x16 &acc, int b, auto qi_c, auto masked_c) __attribute__((always_inline)) {
    constexpr int QI = decltype(qi_c)::value;
    constexpr bool MASKED = decltype(masked_c)::value;
    const int phase = b % phases;
    const int lane_tab = QI % 2 ? lane_tab_odd : lane_tab_even;
    const f16x8 ind0 = *(const f16x8 *)(s_tab + (phase * 2 + 0) * tab_stride + lane_tab);
    const f16x8 ind1 = *(const f16x8 *)(s_tab + (phase * 2 + 1) * tab_stride + lane_tab);
    const float off = kHalfShift - m_run[QI];
    const int k0 = block_key0(b) + 4 * half;
    // two halves of 8 logits: exp2, (masked: window keys go to the row sum only), fp16 pack, indicator MFMA
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      float e[8];
#pragma unroll
      for (int v = 0; v < 8; ++v) e[v] = fast_exp2(__builtin_fmaf(acc[8 * j + v], c1, off));
      if constexpr (MASKED) {
        float lw = 0.f;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
          const int r = 8 * j + v;
          const bool prefix = k0 + 8 * (r / 4) + (r % 4) < P;
          lw += prefix ? 0.f : e[v];
          e[v] = prefix ? e[v] : 0.f;
        }
        l_run[QI] += lw;
      }
      f16x8 bj;
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const f16x2 h2 = __builtin_convertvector(f32x2{e[2 * p], e[2 * p + 1]}, f16x2);
        bj[2 * p] = h2[0]; bj[2 * p + 1] = h2[1];
      }
      acc2[QI / 2] = __builtin_amdgcn_mfma_f32_32x32x16_f16(j == 0 ? ind0 : ind1, bj, acc2[QI / 2], 0, 0, 0);
    }
  };
  // part 3: at the end of a period (or of the range) write E and the maximum it is relative to.
  // E layout [problem][period][row][16 slots]: registers 0..3 of a lane are slots 4*half + 0..3 and
  // registers 4..7 slots 8 + 4*half + 0..3 (nslots <= 16), so a lane stores two 16-byte pieces.
  auto flush_if_period_done = [&](int b, auto qi_c) __attribute__((always_inline)) {
    constexpr int QI = decltype(qi_c)::value;
    if ((b + 1) % phases != 0 && b + 1 != nblk) return;
    const int period = block_key0(b) / pk;
    const int row = (wq * NQW + QI) * 32 + n;
    constexpr int A = QI / 2, R0 = 8 * (QI % 2);
    f32x4 lo = {acc2[A][R0 + 0], acc2[A][R0 + 1], acc2[A][R0 + 2], acc2[A][R0 + 3]};
    f32x4 hi = {acc2[A][R0 + 4], acc2[A][R0 + 5], acc2[A][R0 + 6], acc2[A][R0 + 7]};
    l_run[QI] += ((lo.x + lo.y) + (lo.z + lo.w)) + ((hi.x + hi.y) + (hi.z + hi.w));
    if (period < a.n_periods) {
      const int64_t pr0 = ((int64_t)problem * a.n_periods + period) * a.rows_pad;  // wavefront-uniform
      char *ebase = (char *)(a.e_buf + pr0 * 16);
      const uint32_t eoff = (uint32_t)(row * 64 + half * 16);
      *(f32x4 *)(ebase + eoff) = lo;
      *(f32x4 *)(ebase + eoff + 32) = hi;
      if (half == 0) *(float *)((char *)(a.m_period + pr0) + (uint32_t)(row * 4)) = m_run[QI];
    }
#pragma unroll
    for (int v = 0; v < 8; ++v) acc2[A][R0 + v] = 0.f;
  };

  // Operand fragments of K are read just in time: a ring of four 16-byte fragments, each refilled four
  // MFMAs ahead of its use (same block, the next row block of the same key block, or the next key block).
  // Because a tile is still being read while its last key block is processed, the slot refilled at a tile
  // transition is the one of the tile before it.
  u32x4 kf[4];
  f32x16 accs[2];
  auto micro = [&](int b, auto qi_c, auto par_c, auto has_prev_c, auto masked_c) __attribute__((always_inline)) {
    constexpr int QI = decltype(qi_c)::value, PAR = decltype(par_c)::value;
    constexpr bool HAS_PREV = decltype(has_prev_c)::value;
    constexpr int PQI = QI > 0 ? QI - 1 : NQW - 1;
    const int pb = QI > 0 ? b : b - 1;
    if constexpr (QI == 0) {
      if ((b + 1) % KBT == 0 && (b + 1) / KBT < nt) {
        const int inext = (b + 1) / KBT;              // tiles <= inext + 1 have been issued
        wait_tile(inext + 1 < nt ? 1 : 0);
        lds_barrier();  // tile inext is in LDS; every wavefront is done with tile inext - 2
        if (inext + 2 < nt) issue_tile(inext + 2);  // into the slot of tile inext - 2
      }
    }
    const int nb = QI == NQW - 1 ? (b + 1 < nblk ? b + 1 : b) : b;  // key block of the next micro-step
#pragma unroll
    for (int v = 0; v < 16; ++v) accs[PAR][v] = 0.f;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      mma<DT>(accs[PAR], kf[ks % 4], qf[QI][ks]);  // D[key][row]
      kf[ks % 4] = ks + 4 < NKS ? *frag_ptr(b, ks + 4) : *frag_ptr(nb, ks + 4 - NKS);
    }
    if constexpr (HAS_PREV) {
      update_max(accs[PAR ^ 1], pb, std::integral_constant<int, PQI>{}, masked_c);
      accumulate(accs[PAR ^ 1], pb, std::integral_constant<int, PQI>{}, masked_c);
      constexpr int kValuPerMfma = (16 * 4) / NKS + 1;
#pragma unroll
      for (int r = 0; r < NKS; ++r) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, kValuPerMfma, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
      flush_if_period_done(pb, std::integral_constant<int, PQI>{});
    }
  };
  auto run_micro = [&](int b, auto qi_c, auto par_c) __attribute__((always_inline)) {
    constexpr int QI = decltype(qi_c)::value;
    if (block_masked(QI > 0 ? b : b - 1)) micro(b, qi_c, par_c, std::true_type{}, std::true_type{});
    else micro(b, qi_c, par_c, std::true_type{}, std::false_type{});
  };
  // all row blocks of key block b; PAR0 = parity of micro-step b * NQW
  auto run_block = [&](int b, auto par0_c) __attribute__((always_inline)) {
    constexpr int PAR0 = decltype(par0_c)::value;
    run_micro(b, std::integral_constant<int, 0>{}, std::integral_constant<int, PAR0>{});
    if constexpr (NQW > 1) run_micro(b, std::integral_constant<int, 1>{}, std::integral_constant<int, PAR0 ^ 1>{});
    if constexpr (NQW > 2) {
      run_micro(b, std::integral_constant<int, 2>{}, std::integral_constant<int, PAR0>{});
      run_micro(b, std::integral_constant<int, 3>{}, std::integral_constant<int, PAR0 ^ 1>{});
    }
  };

  wait_tile(nt - 1 < 2 ? nt - 1 : 2);  // tiles 0..2 issued
  lds_barrier();                        // tile 0 and the indicator table are in LDS
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) kf[ks] = *frag_ptr(0, ks % NKS);
  // key block 0: its first micro-step has no predecessor
  micro(0, std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, std::false_type{}, std::false_type{});
  if constexpr (NQW > 1) run_micro(0, std::integral_constant<int, 1>{}, std::integral_constant<int, 1>{});
  if constexpr (NQW > 2) {
    run_micro(0, std::integral_constant<int, 2>{}, std::integral_constant<int, 0>{});
    run_micro(0, std::integral_constant<int, 3>{}, std::integral_constant<int, 1>{});
  }
  for (int b = 1; b < nblk; b += 2) {
    run_block(b, std::integral_constant<int, NQW & 1>{});          // odd b: parity of b * NQW is NQW & 1
    if (b + 1 < nblk) run_block(b + 1, std::integral_constant<int, 0>{});
  }
  {
    // the last micro-step (nblk-1, NQW-1) still owes its epilogue
    constexpr int LQ = NQW - 1;
    const int lb = nblk - 1;
    auto finish = [&](f32x16 &last) __attribute__((always_inline)) {
      if (block_masked(lb)) {
        update_max(last, lb, std::integral_constant<int, LQ>{}, std::true_type{});
        accumulate(last, lb, std::integral_constant<int, LQ>{}, std::true_type{});
      } else {
        update_max(last, lb, std::integral_constant<int, LQ>{}, std::false_type{});
        accumulate(last, lb, std::integral_constant<int, LQ>{}, std::false_type{});
      }
    };
    if (((lb * NQW + LQ) & 1) == 0) finish(accs[0]);
    else finish(accs[1]);
    flush_if_period_done(lb, std::integral_constant<int, LQ>{});
  }

  // per-range (max, sum) of every row for the merge kernel; sums carry the 2^kHalfShift scale throughout
#pragma unroll
  for (int qi = 0; qi < NQW; ++qi) {
    const float l = l_run[qi] + __shfl_xor(l_run[qi], 32);
    if (half == 0) {
      const int row = (wq * NQW + qi) * 32 + n;
      a.part_stats[(problem * a.max_split + split) * a.rows_pad + row] = make_float2(m_run[qi], l);
    }
  }
}

template <int HD, int NQW>
int launch_fused_cfg(const ScoreArgs &a, dim3 grid, hipStream_t s) {
  static bool attr_done = false;
  auto kern = score_fused_kernel<HD, NQW>;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            kFusedLdsBytes) != hipSuccess)
      return CHUNKKV_ERR_LAUNCH;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, grid, dim3(kThreads), kFusedLdsBytes, s, a);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

}  // namespace ckv
