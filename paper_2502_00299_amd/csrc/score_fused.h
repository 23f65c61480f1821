// Single-pass observation-window scoring (Algorithm 1, first two steps) for bf16 and fp16 caches.
//
// K is streamed ONCE.  The kernel is an attention forward pass whose "value" matrix is the 0/1 indicator
// of chunk membership: for every window row r it keeps a reference m_r (online softmax), forms
// e = exp2(logit*scale*log2e + 12 - m_r) for the 32 keys of a block, casts e to fp16 and multiplies it with
// the block's indicator fragments on the matrix cores, so the accumulator holds, per row, the sum of e over
// each chunk of the current PERIOD of lcm(32, c) keys (at most 16 chunk slots).  The reference is lazy: it
// moves only when a block maximum exceeds it by more than kLazy, and the accumulators are rescaled only
// then.  At the end of a period the per-(chunk, row) sums E and the reference they are relative to are
// written out; the row's total sum follows from the E sums (plus the window keys, which belong to no
// chunk).  Afterwards a merge kernel turns the per-range (reference, sum) pairs into
// ref_r = m_r + log2(sum_r) and a small reduction kernel forms
//     score[chunk] = sum_r E[chunk][r] * exp2(m_period[r] - ref_r).
// Nothing is approximated except the fp16 rounding of e (relative 2^-11, the same values feed numerator
// and denominator); chunk scores stay well inside the 1e-3 tolerance.
//
// Ring, swizzle and waits are those of the two-pass kernels (score_impl.h), with buffer loads as the DMA
// instruction.  The work advances in steps (one 32-key block against one 32-row block); the body of a step
// finishes its logits while the matrix cores compute the next step's.  Every wavefront owns its 32*NQW
// rows for all keys of the workgroup's range, so there is no cross-wavefront reduction and no barrier
// besides the ring's.
#pragma once
#include "score_impl.h"

namespace ckv {

typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kFusedTableBytes = 16384;  // indicator fragments: 2 KB per 32-key phase of a period, <= 8 phases
constexpr int kFusedLdsBytes = kRing * kTileBytes + kFusedTableBytes;
constexpr float kHalfShift = 12.f;      // e is scaled by 2^12 before the fp16 cast (denormals below 2^-26)
constexpr float kLazy = 2.f;            // slack of the running reference, log2 units

typedef unsigned int u32x3 __attribute__((ext_vector_type(3)));
constexpr int kEBytesPerRow = 48;  // 16 chunk slots x 3 bytes

// four non-negative finite fp32 values -> their rounded upper three bytes, packed into three dwords
__device__ __forceinline__ u32x3 pack24(f32x4 v) {
  const uint32_t a = __float_as_uint(v.x) + 0x80u, b = __float_as_uint(v.y) + 0x80u;
  const uint32_t c = __float_as_uint(v.z) + 0x80u, d = __float_as_uint(v.w) + 0x80u;
  return u32x3{__builtin_amdgcn_perm(b, a, 0x05030201u), __builtin_amdgcn_perm(c, b, 0x06050302u),
               __builtin_amdgcn_perm(d, c, 0x07060503u)};
}

template <int DT, int HD, int NQW>
__global__ __launch_bounds__(kThreads, (NQW >= 4 ? 1 : 2)) void score_fused_kernel(ScoreArgs a) {
  static_assert(is_16bit(DT), "the single-pass kernel takes bf16 or fp16 caches");
  constexpr int ROWB = HD * 2;
  constexpr int NSEG = ROWB / 16;
  constexpr int NKS = ROWB / 32;
  constexpr int TK = kTileBytes / ROWB;
  constexpr int KBT = TK / 32;
  constexpr int ESZ = 2;

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
  const char *kbase = (const char *)pick(a.k, z) + (pick(a.seq.kv_base, bl) + (int64_t)h * a.kv_stride_head) * ESZ;
  const int64_t ktok = a.kv_stride_tok * ESZ;
  const float c1 = a.scale_log2e;

  // ---- K tiles: HBM -> LDS ring (ring, swizzle and waits as in score_impl.h).  The loads are buffer
  // loads with an LDS destination: the descriptor covers exactly the L rows of this (sequence, kv-head),
  // so rows past the end of the sequence read as zero instead of being clamped.
  const __amdgpu_buffer_rsrc_t krsrc =
      __builtin_amdgcn_make_buffer_rsrc((void *)kbase, 0, (int)((uint32_t)(L - 1) * (uint32_t)ktok + ROWB), 0x00020000);
  uint32_t klane[kLoadsPerWave];  // lane's byte offset inside a tile: key row and swizzled 16-byte segment
#pragma unroll
  for (int j = 0; j < kLoadsPerWave; ++j) {
    const int key = (wave * kLoadsPerWave + j) * (1024 / ROWB) + lane / NSEG, segp = lane % NSEG;
    klane[j] = (uint32_t)(key * (int)ktok + ((segp ^ (key & 7)) * 16));
  }
  auto issue_tile = [&](int i) __attribute__((always_inline)) {
    const uint32_t tile_off = (uint32_t)(range0 + i * TK) * (uint32_t)ktok;
    char *slot = smem + (i % kRing) * kTileBytes;
#pragma unroll
    for (int j = 0; j < kLoadsPerWave; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc, (__attribute__((address_space(3))) void *)(slot + (wave * kLoadsPerWave + j) * 1024),
                                               16, klane[j], tile_off, 0, 0);
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

  // ---- indicator fragments.  Entry (phase, kgroup, slot row, j) holds, for the 8 k-positions e of
  // indicator MFMA j and lane half kgroup, 1.0 where the key of accumulator register 8j+e (block-relative
  // key 8*((8j+e)/4) + 4*kgroup + (8j+e)%4) belongs to chunk slot `slot row` of the period.  Slot rows
  // nslots..31 are zero; every lane reads an entry of its own (no two lanes share an address).
  {
    const int entries = phases * 128;
    for (int en = tid; en < entries; en += kThreads) {
      const int j = en & 1, slot = (en >> 1) & 31, kg = (en >> 6) & 1, phase = en >> 7;
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
  const uint32_t lane_tab = (uint32_t)(kRing * kTileBytes + (half * 32 + n) * 32);
  constexpr uint32_t kPhaseBytes = 2048;

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
  // Indicator accumulators, one 32x32 tile per row block: a period has at most 16 chunk slots, so only
  // registers 0..7 carry sums (register v <-> chunk slot 8*(v/4) + 4*half + v%4); the tile is kept whole
  // so that every update is a whole-vector operation.
  constexpr int NA = NQW;
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

  // ---- K operand fragments.  Lane n of a fragment read takes key row n of the block, 16-byte segment
  // (2*ks + half) ^ (n & 7); ks and ks + 4 differ by 128 bytes, so four lane offsets serve all ks and the
  // tile slot and the block within the tile are a wavefront-uniform term plus a constant.
  uint32_t kaddr[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) kaddr[j] = (uint32_t)((n * NSEG + (((2 * j + half) ^ (n & 7)) & (NSEG - 1))) * 16);
  auto frag = [&](uint32_t blk_off, int ks) __attribute__((always_inline)) {
    return *(const u32x4 *)(smem + (kaddr[ks % 4] + blk_off + (uint32_t)((ks / 4) * 128)));
  };

  // The pipeline advances in micro-steps: step (b, qi) is key block b against row block qi of this
  // wavefront; inside a tile the step index idx = kb * NQW + qi is a compile-time constant.  The body of a
  // step finishes the step's logits (running maximum, exponentials, indicator MFMAs) while the matrix
  // cores compute the logits of the following step; K fragments are read just in time into a ring of four
  // registers quads, each refilled four MFMAs ahead of its use.
  constexpr int M = KBT * NQW;  // steps per tile (even)
  u32x4 kf[4];
  f32x16 accs[2];
  f16x8 ind0, ind1;
  // MFMAs ks0..ks1-1 of a step whose block sits at LDS offset off_s; off_n is the block of the step after it
  auto mfma_part = [&](f32x16 &acc, auto qi_c, auto ks0_c, auto ks1_c, uint32_t off_s, uint32_t off_n)
      __attribute__((always_inline)) {
    constexpr int QI = decltype(qi_c)::value, KS0 = decltype(ks0_c)::value, KS1 = decltype(ks1_c)::value;
#pragma unroll
    for (int ks = KS0; ks < KS1; ++ks) {
      if (ks == 0) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
      }
      mma<DT>(acc, kf[ks % 4], qf[QI][ks]);  // D[key][row]
      kf[ks % 4] = ks + 4 < NKS ? frag(off_s, ks + 4) : frag(off_n, ks + 4 - NKS);
    }
  };

  int ph = 0;                      // key block within the period
  int period = range0 / pk;        // period of the current key block
  uint32_t tab_off = 0;            // ph * kPhaseBytes
  // E and m_period of this problem (byte offsets inside stay below 2^32: n_periods * rows_pad * kEBytesPerRow)
  char *e_problem = (char *)a.e_buf + (int64_t)problem * a.n_periods * a.rows_pad * kEBytesPerRow;
  char *m_problem = (char *)a.m_period + (int64_t)problem * a.n_periods * a.rows_pad * 4;
  const uint32_t lane_eoff = (uint32_t)((wq * NQW * 32 + n) * kEBytesPerRow + half * (kEBytesPerRow / 2));
  const uint32_t lane_moff = (uint32_t)((wq * NQW * 32 + n) * 4);

  // CLEAN: the step belongs to a tile whose keys are all prefix keys and that is not among the last tiles
  // of the range, so nothing has to be masked and the range cannot end here.
  auto body = [&](int T, uint32_t toff, uint32_t toff_next, auto idx_c, auto masked_c, auto clean_c) __attribute__((always_inline)) {
    constexpr bool CLEAN = decltype(clean_c)::value;
    constexpr int IDX = decltype(idx_c)::value, KB = IDX / NQW, QI = IDX % NQW, PAR = IDX & 1;
    constexpr bool MASKED = decltype(masked_c)::value;
    constexpr int I1 = (IDX + 1) % M, I2 = (IDX + 2) % M;       // the next two steps
    constexpr bool W1 = IDX + 1 >= M, W2 = IDX + 2 >= M;        // ... lie in the next tile
    constexpr int QI1 = I1 % NQW;
    const uint32_t off1 = (W1 ? toff_next : toff) + (uint32_t)((I1 / NQW) * 32 * ROWB);
    const uint32_t off2 = (W2 ? toff_next : toff) + (uint32_t)((I2 / NQW) * 32 * ROWB);
    const int b = T * KBT + KB;
    f32x16 &acc = accs[PAR];
    constexpr int KSA = NKS >= 8 ? 2 : 1;  // MFMAs of the next step issued beside the maximum search

    // indicator fragments of this key block (the same for all its row blocks), needed in part 2
    if constexpr (QI == 0) {
      const uint32_t taddr = lane_tab + tab_off;
      ind0 = *(const f16x8 *)(smem + taddr);
      ind1 = *(const f16x8 *)(smem + taddr + 16);
    }

    // part 1: new running maximum of the row
    mfma_part(accs[PAR ^ 1], std::integral_constant<int, QI1>{}, std::integral_constant<int, 0>{},
              std::integral_constant<int, KSA>{}, off1, off2);
    const int k0 = range0 + b * 32 + 4 * half;
    if constexpr (MASKED) {
      // only the last blocks of a sequence come here: mask the keys behind the row's own position
      const int row = (wq * NQW + QI) * 32 + n;
      const int lim = P + (row < nrows ? row % w : 0);
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[v] = k0 + 8 * (v / 4) + (v % 4) <= lim ? acc[v] : -3.0e38f;
    }
    // block maximum as a shallow tree
    const float t0 = fmaxf(fmaxf(acc[0], acc[1]), acc[2]), t1 = fmaxf(fmaxf(acc[3], acc[4]), acc[5]);
    const float t2 = fmaxf(fmaxf(acc[6], acc[7]), acc[8]), t3 = fmaxf(fmaxf(acc[9], acc[10]), acc[11]);
    const float t4 = fmaxf(fmaxf(acc[12], acc[13]), acc[14]);
    float bm = fmaxf(fmaxf(fmaxf(t0, t1), t2), fmaxf(fmaxf(t3, t4), acc[15]));
    // both lane halves of a row share one reference: exchange across the halves without LDS
    const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(bm), __float_as_uint(bm), false, false);
    bm = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
    // The reference m_run need not be the exact maximum: it moves only when the block maximum exceeds it
    // by more than kLazy (then it is set one above the maximum), so e stays below 2^kLazy and the fp16
    // products below 2^(kHalfShift + kLazy); after the first blocks of a range this is rare.
    const float cand = __builtin_fmaf(bm, c1, -kLazy);
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x002, 10, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    if constexpr (KSA > 1) {
      __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
      __builtin_amdgcn_sched_group_barrier(0x002, 10, 0);
      __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
    }
    if (__builtin_amdgcn_ballot_w64(cand > m_run[QI]) != 0) {
      const float m_new = cand > m_run[QI] ? cand + (kLazy + 1.f) : m_run[QI];
      const float f = fast_exp2(m_run[QI] - m_new);
      acc2[QI] = acc2[QI] * f;
      l_run[QI] *= f;
      m_run[QI] = m_new;
    }

    // part 2: e = exp2(...), fp16 pack, two indicator MFMAs, beside the remaining MFMAs of the next step
    mfma_part(accs[PAR ^ 1], std::integral_constant<int, QI1>{}, std::integral_constant<int, KSA>{},
              std::integral_constant<int, NKS>{}, off1, off2);
    const float off = kHalfShift - m_run[QI];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      float e[8];
#pragma unroll
      for (int v = 0; v < 8; ++v) e[v] = fast_exp2(__builtin_fmaf(acc[8 * j + v], c1, off));
      if constexpr (MASKED) {
        // window keys count for the row sum but belong to no chunk
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
      acc2[QI] = __builtin_amdgcn_mfma_f32_32x32x16_f16(j == 0 ? ind0 : ind1, bj, acc2[QI], 0, 0, 0);
    }
    if constexpr (!MASKED) {
      constexpr int NM = NKS - KSA + 2;               // MFMAs of this region
      constexpr int kValuPerMfma = (40 + NM - 1) / NM;  // 16 fma, 16 exp2, 8 packs, a few more
#pragma unroll
      for (int r = 0; r < NM; ++r) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, kValuPerMfma, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
      }
    }

    // part 3: at the end of a period (or of the range) write E and the reference it is relative to.
    // Registers 0..3 of a lane are slots 4*half + 0..3 and registers 4..7 slots 8 + 4*half + 0..3
    // (nslots <= 16).  E row layout (kEBytesPerRow = 48): the 8 values of lane half 0, then those of half 1,
    // each as the upper three bytes of its fp32 (rounded: 16 mantissa bits, relative 2^-17), 24 bytes per lane.
    if (ph == phases - 1 || (!CLEAN && b == nblk - 1)) {
      f32x4 lo = {acc2[QI][0], acc2[QI][1], acc2[QI][2], acc2[QI][3]};
      f32x4 hi = {acc2[QI][4], acc2[QI][5], acc2[QI][6], acc2[QI][7]};
      l_run[QI] += ((lo.x + lo.y) + (lo.z + lo.w)) + ((hi.x + hi.y) + (hi.z + hi.w));
      if (period < a.n_periods) {
        const uint32_t prow = (uint32_t)period * (uint32_t)a.rows_pad + (uint32_t)(QI * 32);  // wavefront-uniform
        const uint32_t eoff = prow * (uint32_t)kEBytesPerRow + lane_eoff;
        *(u32x3 *)(e_problem + eoff) = pack24(lo);
        *(u32x3 *)(e_problem + eoff + 12) = pack24(hi);
        if (half == 0) *(float *)(m_problem + (prow * 4u + lane_moff)) = m_run[QI];
      }
      acc2[QI] = f32x16{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    }
    if constexpr (QI == NQW - 1) {
      // the key block is done: advance the period phase
      const bool wrap = ph == phases - 1;
      ph = wrap ? 0 : ph + 1;
      tab_off = wrap ? 0u : tab_off + kPhaseBytes;
      period += wrap ? 1 : 0;
    }
  };

  wait_tile(nt - 1 < 2 ? nt - 1 : 2);  // tiles 0..2 issued
  lds_barrier();                        // tile 0 and the indicator table are in LDS
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) kf[ks] = frag(0u, ks % NKS);
  {
    // logits of step 0; the step after it is in tile 0 as well
    constexpr uint32_t kOff1 = (uint32_t)((1 / NQW) * 32 * ROWB);
    mfma_part(accs[0], std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{},
              std::integral_constant<int, NKS>{}, 0u, kOff1);
  }
  // Tiles that need no checks: all their keys are prefix keys and three more tiles follow in the range.
  int n_clean = (P - range0) / TK;
  n_clean = n_clean < nt - 3 ? n_clean : nt - 3;
  n_clean = n_clean > 0 ? n_clean : 0;
  auto for_steps = [&](auto f) __attribute__((always_inline)) {
    f(std::integral_constant<int, 0>{});
    f(std::integral_constant<int, 1>{});
    if constexpr (M > 2) { f(std::integral_constant<int, 2>{}); f(std::integral_constant<int, 3>{}); }
    if constexpr (M > 4) {
      f(std::integral_constant<int, 4>{}); f(std::integral_constant<int, 5>{});
      f(std::integral_constant<int, 6>{}); f(std::integral_constant<int, 7>{});
    }
    if constexpr (M > 8) {
      f(std::integral_constant<int, 8>{}); f(std::integral_constant<int, 9>{});
      f(std::integral_constant<int, 10>{}); f(std::integral_constant<int, 11>{});
      f(std::integral_constant<int, 12>{}); f(std::integral_constant<int, 13>{});
      f(std::integral_constant<int, 14>{}); f(std::integral_constant<int, 15>{});
    }
    static_assert(M <= 16, "steps per tile");
  };
  int T = 0;
  for (; T < n_clean; ++T) {
    const uint32_t toff = (uint32_t)((T % kRing) * kTileBytes), toff_next = (uint32_t)(((T + 1) % kRing) * kTileBytes);
    for_steps([&](auto idx_c) __attribute__((always_inline)) {
      constexpr int IDX = decltype(idx_c)::value;
      if constexpr (IDX == M - 2) {
        // the refills of this step start to read tile T + 1
        wait_tile(1);      // tiles <= T + 2 have been issued
        // Tile T + 1 is in LDS; every wavefront is done with tile T - 1, whose fragments the MFMAs consumed
        // a tile ago.  The LDS reads in flight are prefetches of tiles T and T + 1, so the barrier does not
        // wait for them (a wait here would drain the fragment ring once per tile).
        __builtin_amdgcn_s_barrier();
        issue_tile(T + 3);
      }
      body(T, toff, toff_next, idx_c, std::false_type{}, std::true_type{});
    });
  }
  for (; T < nt; ++T) {
    const uint32_t toff = (uint32_t)((T % kRing) * kTileBytes), toff_next = (uint32_t)(((T + 1) % kRing) * kTileBytes);
    const int nb_t = nblk - T * KBT;  // key blocks of this tile that hold keys of the sequence (>= 1)
    for_steps([&](auto idx_c) __attribute__((always_inline)) {
      constexpr int IDX = decltype(idx_c)::value;
      if (IDX / NQW >= nb_t) return;
      if constexpr (IDX == M - 2) {
        if (T + 1 < nt) {
          wait_tile(T + 2 < nt ? 1 : 0);
          __builtin_amdgcn_s_barrier();
          if (T + 3 < nt) issue_tile(T + 3);
        }
      }
      if (range0 + (T * KBT + IDX / NQW) * 32 + 32 > P) body(T, toff, toff_next, idx_c, std::true_type{}, std::false_type{});
      else body(T, toff, toff_next, idx_c, std::false_type{}, std::false_type{});
    });
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

template <int DT, int HD, int NQW>
int launch_fused_cfg(const ScoreArgs &a, dim3 grid, hipStream_t s) {
  static bool attr_done = false;
  auto kern = score_fused_kernel<DT, HD, NQW>;
  if (!attr_done) {
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            kFusedLdsBytes) != hipSuccess)
      return CHUNKKV_ERR_LAUNCH;
    attr_done = true;
  }
  const int lds_bytes = kRing * kTileBytes + a.period_keys / 32 * 2048;  // ring + indicator table
  hipLaunchKernelGGL(kern, grid, dim3(kThreads), lds_bytes, s, a);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

// every compiled geometry of one storage type
template <int DT>
int launch_fused_dt(int head_dim, const ScoreGeom &g, const ScoreArgs &a, dim3 grid, hipStream_t s) {
  if (g.wq != 4) return CHUNKKV_ERR_UNSUPPORTED;
  if (head_dim == 128) {
    if (g.nqw == 1) return launch_fused_cfg<DT, 128, 1>(a, grid, s);
    if (g.nqw == 2) return launch_fused_cfg<DT, 128, 2>(a, grid, s);
    if (g.nqw == 4) return launch_fused_cfg<DT, 128, 4>(a, grid, s);
  } else if (head_dim == 64) {
    if (g.nqw == 1) return launch_fused_cfg<DT, 64, 1>(a, grid, s);
    if (g.nqw == 2) return launch_fused_cfg<DT, 64, 2>(a, grid, s);
    if (g.nqw == 4) return launch_fused_cfg<DT, 64, 4>(a, grid, s);
  }
  return CHUNKKV_ERR_UNSUPPORTED;
}

}  // namespace ckv
