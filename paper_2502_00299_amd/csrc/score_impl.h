// Observation-window scoring (Algorithm 1, first two steps, with the row softmax the text implies).
//
// For one (leader layer, sequence, kv-head) the g*w window rows are multiplied with every key on the
// matrix cores (bf16: v_mfma_f32_32x32x16_bf16, f32: v_mfma_f32_32x32x2_f32; fp32 accumulation).
// The exact softmax needs each row's maximum and sum over ALL visible keys before any column can be
// normalised, so the work is two passes over K:
//   pass 0  (keys x rows orientation: a lane owns one window row)  streams K, keeps a running
//           (max, sum) per row in registers, and writes one partial pair per row and key range;
//   -----   a tiny kernel merges the partial pairs into ref_r = max_r + log2(sum_r) (or, when the caller
//           supplies each row's log-sum-exp, converts that and pass 0 does not run at all);
//   pass 1  (rows x keys orientation: a lane owns one key)  streams K again with the accumulators
//           started at -ref_r/(scale*log2e) (kept in registers for bf16 caches, where they are the C
//           operand of a block's first MFMA), so p = exp2(acc*scale*log2e); p is summed over the rows in
//           registers, across the two lane halves by one shuffle, across wavefronts in LDS, and once
//           per super-tile of kSuperKeys keys the per-token importance is reduced to chunk sums with a
//           fixed-order segmented sum in LDS (super-tiles advance by a multiple of c, so no chunk
//           straddles two of them and no atomics are needed: results are deterministic).
//
// K streaming: tiles of 16 KB travel HBM -> LDS directly (buffer loads with an LDS destination, 16 bytes
// per lane, no register staging; the buffer descriptor covers the rows of one sequence and kv-head, so
// rows past the end read as zero) into a ring of kRing slots, three or four tiles in flight per workgroup.
// Being buffer and not flat-segment instructions they leave the LDS counter's ordering exact, so the
// compiler's waits before the operand reads name just the read that is needed.  A wavefront
// instruction fills 1 KB of a slot in lane order, so the XOR swizzle of the 16-byte row segments by
// key index is applied on the global-address side; the MFMA operand reads (one 16-byte segment per
// lane, 32 keys per instruction) then hit distinct banks.  Completion is tracked with explicit
// s_waitcnt vmcnt(n) and raw s_barrier: a fenced barrier would drain the ring on every tile.
//
// The block loop is software-pipelined one key block deep: a step issues the MFMAs of block b, the
// LDS reads of block b+1's operand fragments (each behind the MFMAs that consumed the old fragment)
// and the exp/sum epilogue of block b-1 as one straight-line region, with scheduling hints that
// alternate one MFMA with a handful of VALU instructions, so the matrix pipe and the vector ALU of a
// wavefront work at the same time.  The window queries stay in registers as operand fragments.
#pragma once
#include <mutex>
#include <type_traits>

#include "internal.h"

namespace ckv {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr float kNegBig = -1.0e30f;
constexpr int kRing = 4;                                          // LDS slots of kTileBytes
constexpr int kLoadsPerWave = kTileBytes / 1024 / (kThreads / 64);  // 1 KB loads a wavefront issues per tile
// [4][kSuperKeys] partial column sums + [kSuperKeys] importance + [kMaxRows] accumulator start values
constexpr int kScoreMiscBytes = 4 * kSuperKeys * 4 + kSuperKeys * 4 + kMaxRows * 4;
constexpr int kScoreLdsBytes = kRing * kTileBytes + kScoreMiscBytes;

// 16-bit storage types share every layout (8 elements per 16-byte fragment); only the MFMA differs
constexpr bool is_16bit(int dt) { return dt == CHUNKKV_BF16 || dt == CHUNKKV_F16; }

template <int DT>
__device__ __forceinline__ void mma(f32x16 &acc, const u32x4 &a, const u32x4 &b) {
  if constexpr (DT == CHUNKKV_BF16) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                  acc, 0, 0, 0);
  } else if constexpr (DT == CHUNKKV_F16) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b),
                                                 acc, 0, 0, 0);
  } else {
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  }
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// s_waitcnt immediate (gfx9 encoding) that waits only for the vector-memory counter to drop to n.
constexpr int vmcnt_imm(int n) { return (n & 0xF) | ((n >> 4) << 14) | 0x0F70; }
// Wavefront-local LDS traffic finished, then workgroup barrier.  No memory fence: outstanding
// global->LDS tile loads stay in flight.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
  __builtin_amdgcn_s_barrier();
}

// DT: chunkkv_dtype, HD: head dim, NQW: 32-row blocks per wavefront, WQ: wavefronts splitting the rows.
// Two workgroups per CU, except where the operand fragments alone need more than half the register file
// (four row blocks per wavefront; fp32 operands at head_dim 128).
template <int DT, int HD, int NQW, int WQ, int PASS>
__global__ __launch_bounds__(kThreads, ((NQW >= 4 || (DT == CHUNKKV_F32 && HD == 128)) ? 1 : 2)) void score_kernel(ScoreArgs a) {
  constexpr int ESZ = is_16bit(DT) ? 2 : 4;
  constexpr int ROWB = HD * ESZ;
  constexpr int NSEG = ROWB / 16;
  constexpr int NKS = ROWB / 32;
  constexpr int TK = kTileBytes / ROWB;                // keys per tile
  constexpr int KBT = TK / 32;                         // 32-key blocks per tile
  constexpr int WK = (4 / WQ) < KBT ? (4 / WQ) : KBT;  // wavefronts splitting the key blocks of a tile
  constexpr int KPW = KBT / WK;                        // key blocks of a tile one wavefront handles
  static_assert(KBT >= 1 && KBT % WK == 0 && ROWB <= 1024 && kSuperKeys % TK == 0, "tile geometry");

  extern __shared__ __align__(16) char smem[];
  float *s_part = (float *)(smem + kRing * kTileBytes);  // [WQ][kSuperKeys] partial column sums
  float *s_imp = s_part + 4 * kSuperKeys;                // [kSuperKeys] importance of the super-tile
  float *s_start = s_imp + kSuperKeys;                   // [rows] pass 1: -ref_r / (scale*log2e)

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, half = lane >> 5;
  const int wq = wave % WQ, wk = wave / WQ;
  const bool active = (4 / WQ == WK) ? true : (wk < WK);  // wavefronts beyond the key blocks only load
  const int bl = blockIdx.y / a.n_kv_heads, h = blockIdx.y % a.n_kv_heads, z = blockIdx.z;
  const int split = blockIdx.x;
  const int g = a.n_q_heads / a.n_kv_heads, w = a.window, c = a.chunk;
  const int L = pick(a.seq.seqlen, bl), P = L - w, nrows = g * w;
  const int64_t problem = ((int64_t)(a.leader0 + z) * a.batch_total + (a.batch0 + bl)) * a.n_kv_heads + h;

  // Work units: pass 0 walks tiles of TK keys over [0, L); pass 1 walks super-tiles over [0, P), each
  // advancing `sstride` keys (a multiple of c when chunk sums are fused) and made of `spt` tiles.
  const int sstride = PASS == 0 ? TK : (a.fuse_chunks ? (kSuperKeys / c) * c : kSuperKeys);
  const int spt = (sstride + TK - 1) / TK;
  const int span = PASS == 0 ? L : P;
  const int nunits = (span + sstride - 1) / sstride;
  const int u0 = split * a.tiles_per_wg;
  const int u1 = u0 + a.tiles_per_wg < nunits ? u0 + a.tiles_per_wg : nunits;
  if (u0 >= nunits) return;
  // tiles of this workgroup, numbered 0..nt-1: tile i belongs to unit u0 + i/spt, position i%spt;
  // the last unit stops at the end of the span
  const int last_keys = (span - (u1 - 1) * sstride) < sstride ? (span - (u1 - 1) * sstride) : sstride;
  const int nt = (u1 - 1 - u0) * spt + (last_keys + TK - 1) / TK;
  const int nblk = nt * KPW;  // key blocks this wavefront walks: block b = (tile b / KPW, kb = wk + (b % KPW) * WK)
  auto tile_key0 = [&](int i) __attribute__((always_inline)) { return (u0 + i / spt) * sstride + (i % spt) * TK; };

  const char *qbase = (const char *)pick(a.q, z) + ((int64_t)(a.batch0 + bl) * a.n_q_heads + (int64_t)h * g) * w * ROWB;
  const char *kbase = (const char *)pick(a.k, z) + (pick(a.seq.kv_base, bl) + (int64_t)h * a.kv_stride_head) * ESZ;
  const int64_t ktok = a.kv_stride_tok * ESZ;
  const float c1 = a.scale_log2e;

  // Tile i -> ring slot i % kRing.  Lane l of a 1 KB group lands at byte 16*l of the group, i.e. at
  // (key, segment position l % NSEG); it fetches segment (position ^ key&7) of that key.  The loads are
  // buffer loads with an LDS destination; the descriptor covers exactly the L rows of this (sequence,
  // kv-head), so rows past the end read as zero (their results are masked) and nothing is clamped.  The
  // lane's byte offset inside a tile is the same for every tile: scalar tile offset + 32-bit lane offset.
  const __amdgpu_buffer_rsrc_t krsrc =
      __builtin_amdgcn_make_buffer_rsrc((void *)kbase, 0, (int)((uint32_t)(L - 1) * (uint32_t)ktok + ROWB), 0x00020000);
  uint32_t lane_off[kLoadsPerWave];
#pragma unroll
  for (int j = 0; j < kLoadsPerWave; ++j) {
    const int key = (wave * kLoadsPerWave + j) * (1024 / ROWB) + lane / NSEG, segp = lane % NSEG;
    lane_off[j] = (uint32_t)(key * (int)ktok + ((segp ^ (key & 7)) * 16));
  }
  auto issue_tile = [&](int i) __attribute__((always_inline)) {
    const uint32_t tile_off = (uint32_t)tile_key0(i) * (uint32_t)ktok;  // wavefront-uniform
    char *slot = smem + (i % kRing) * kTileBytes;
#pragma unroll
    for (int j = 0; j < kLoadsPerWave; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc, (__attribute__((address_space(3))) void *)(slot + (wave * kLoadsPerWave + j) * 1024),
                                               16, lane_off[j], tile_off, 0, 0);
  };
  // tile i has landed once at most min(2, tiles issued after it) newer tile loads are outstanding
  auto wait_tile = [&](int i) __attribute__((always_inline)) {
    const int newer = nt - 1 - i;
    if (newer >= 2) __builtin_amdgcn_s_waitcnt(vmcnt_imm(2 * kLoadsPerWave));
    else if (newer == 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kLoadsPerWave));
    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  };
#pragma unroll
  for (int s = 0; s < kRing - 1; ++s)
    if (s < nt) issue_tile(s);

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

  // pass 0 state: running (max, sum) of the lane's row and the last key the row may see
  float m_run[NQW], l_run[NQW];
  int lim[NQW];
#pragma unroll
  for (int qi = 0; qi < NQW; ++qi) {
    m_run[qi] = kNegBig;
    l_run[qi] = 0.f;
    const int row = (wq * NQW + qi) * 32 + n;
    lim[qi] = P + (row < nrows ? row % w : 0);
  }
  // pass 1: accumulator start values, so that acc*c1 = logit*c1 - ref (padding rows end at -1e30)
  if constexpr (PASS == 1) {
    for (int r = tid; r < WQ * NQW * 32; r += kThreads)
      s_start[r] = (r < nrows ? -a.refs[problem * a.rows_pad + r] : kNegBig) / c1;
  }

  // Lane's LDS address of fragment segment ks of key block b: row n of the block, 16-byte segment
  // (2*ks + half) ^ (n & 7).  ks and ks + 4 differ by 128 bytes, so four lane offsets serve every ks and the
  // ring slot and the block within the tile are one wavefront-uniform term.
  uint32_t kaddr[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) kaddr[j] = (uint32_t)((n * NSEG + (((2 * j + half) ^ (n & 7)) & (NSEG - 1))) * 16);
  auto block_off = [&](int b) __attribute__((always_inline)) {
    const int kb = wk + (b % KPW) * WK;
    return (uint32_t)(((b / KPW) % kRing) * kTileBytes + kb * 32 * ROWB);
  };
  auto frag_at = [&](uint32_t boff, int ks) __attribute__((always_inline)) {
    return (const u32x4 *)(smem + (kaddr[ks % 4] + boff + (uint32_t)((ks / 4) * 128)));
  };
  // pass 0: does key block b touch keys a window row may not see (or keys past the sequence)?
  auto block_masked = [&](int b) __attribute__((always_inline)) { return PASS == 0 && tile_key0(b / KPW) + TK > P; };

  // exp/sum epilogue of key block b whose logits are in acc
  auto epilogue = [&](f32x16 (&acc)[NQW], int b, auto masked_c) {
    constexpr bool MASKED = decltype(masked_c)::value;
    const int i = b / KPW, kb = wk + (b % KPW) * WK;
    if constexpr (PASS == 0) {
      // lane: row n of block qi; registers: keys kb*32 + 8*(v/4) + 4*half + v%4
#pragma unroll
      for (int qi = 0; qi < NQW; ++qi) {
        if constexpr (MASKED) {
          const int kbase0 = tile_key0(i) + kb * 32 + 4 * half;
#pragma unroll
          for (int v = 0; v < 16; ++v) acc[qi][v] = kbase0 + 8 * (v / 4) + (v % 4) <= lim[qi] ? acc[qi][v] : -3.0e38f;
        }
        float bm = acc[qi][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) bm = fmaxf(bm, acc[qi][v]);
        const float m_new = fmaxf(m_run[qi], bm * c1);
        float sum[4] = {0.f, 0.f, 0.f, 0.f};  // four independent chains, fixed order
#pragma unroll
        for (int v = 0; v < 16; ++v) sum[v & 3] += fast_exp2(__builtin_fmaf(acc[qi][v], c1, -m_new));
        l_run[qi] = __builtin_fmaf(l_run[qi], fast_exp2(m_run[qi] - m_new), (sum[0] + sum[1]) + (sum[2] + sum[3]));
        m_run[qi] = m_new;
      }
    } else {
      // lane: key kb*32 + n; registers: rows 8*(v/4) + 4*half + v%4 of block qi
      float cs[4] = {0.f, 0.f, 0.f, 0.f};  // four independent chains, fixed order
#pragma unroll
      for (int qi = 0; qi < NQW; ++qi)
#pragma unroll
        for (int v = 0; v < 16; ++v) cs[v & 3] += fast_exp2(acc[qi][v] * c1);
      float colsum = (cs[0] + cs[1]) + (cs[2] + cs[3]);
      colsum += __shfl_xor(colsum, 32);
      if (half == 0) s_part[wq * kSuperKeys + (i % spt) * TK + kb * 32 + n] = colsum;
    }
  };

  // pass 1, after the epilogue of the last key block of a super-tile: importance, then chunk sums
  auto flush_if_unit_done = [&](int b) __attribute__((always_inline)) {
    if constexpr (PASS == 1) {
      const int i = b / KPW;
      if ((b + 1) % KPW != 0 || !((i + 1) % spt == 0 || i + 1 == nt)) return;
      const int ukey0 = (u0 + i / spt) * sstride;
      lds_barrier();
      if (tid < kSuperKeys) {
        float imp = 0.f;
#pragma unroll
        for (int q = 0; q < WQ; ++q) imp += s_part[q * kSuperKeys + tid];
        const int key = ukey0 + tid;
        const bool owned = tid < sstride && key < P;
        imp = owned ? imp : 0.f;
        s_imp[tid] = imp;
        if (owned && a.token_imp) a.token_imp[problem * a.imp_pitch + key] = imp;
      }
      lds_barrier();
      if (a.fuse_chunks) {
        const int nch = sstride / c;
        if (tid < nch) {
          const int cidx = ukey0 / c + tid;
          if ((int64_t)cidx * c < P) {
            float sum = 0.f;
            for (int e = 0; e < c; ++e) sum += s_imp[tid * c + e];
            a.chunk_scores[problem * a.score_cap + cidx] = sum;
          }
        }
      }
    }
  };

  // One pipeline step (see the file header).  HAS_PREV / MASKED are compile-time so that the MFMAs,
  // the fragment reads and the epilogue form one basic block the scheduler can interleave.
  // pass 1: the accumulator start values stay in registers where the register file has room for them
  // (16-bit types: every geometry; fp32 operands are twice as large), otherwise they are re-read from LDS per step
  constexpr bool kStartInRegs = PASS == 1 && is_16bit(DT);
  f32x16 start[kStartInRegs ? NQW : 1];
  u32x4 kf[NKS];
  auto step = [&](int b, f32x16 (&cur)[NQW], f32x16 (&prev)[NQW], auto has_prev_c, auto masked_c) {
    constexpr bool HAS_PREV = decltype(has_prev_c)::value;
    if ((b + 1) % KPW == 0 && (b + 1) / KPW < nt) {
      const int inext = (b + 1) / KPW;
      wait_tile(inext);
      lds_barrier();  // tile inext is in LDS; every wavefront holds its fragments of tile inext-1
      if (inext - 1 + kRing < nt) issue_tile(inext - 1 + kRing);  // refill the slot of tile inext-1
    }
    if (active) {
      const int bn = b + 1 < nblk ? b + 1 : b;  // the last step re-reads its own block (unused)
      const uint32_t boff_next = block_off(bn);
#pragma unroll
      for (int qi = 0; qi < NQW; ++qi) {
        if constexpr (PASS == 1) {
          if constexpr (kStartInRegs) {
            cur[qi] = start[qi];  // becomes the C operand of the first MFMA, no copy
          } else {
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
              const f32x4 st = *(const f32x4 *)(s_start + (wq * NQW + qi) * 32 + 8 * v4 + 4 * half);
              cur[qi][4 * v4 + 0] = st.x; cur[qi][4 * v4 + 1] = st.y; cur[qi][4 * v4 + 2] = st.z; cur[qi][4 * v4 + 3] = st.w;
            }
          }
        } else {
#pragma unroll
          for (int v = 0; v < 16; ++v) cur[qi][v] = 0.f;
        }
      }
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
        for (int qi = 0; qi < NQW; ++qi) {
          if constexpr (PASS == 0) mma<DT>(cur[qi], kf[ks], qf[qi][ks]);   // D[key][row]
          else mma<DT>(cur[qi], qf[qi][ks], kf[ks]);                       // D[row][key]
        }
        kf[ks] = *frag_at(boff_next, ks);
      }
      if constexpr (HAS_PREV) epilogue(prev, b - 1, masked_c);
      if constexpr (is_16bit(DT) && HAS_PREV) {
        // one MFMA, then its share of the epilogue's VALU instructions; a fragment read per MFMA group
        constexpr int kValuPerMfma = (NQW * 16 * 7 / 2) / (NKS * NQW) + 1;
#pragma unroll
        for (int r = 0; r < NKS * NQW; ++r) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, kValuPerMfma, 0);
          if (r % NQW == NQW - 1) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
      }
    }
    if constexpr (HAS_PREV) flush_if_unit_done(b - 1);
  };
  auto run_step = [&](int b, f32x16 (&cur)[NQW], f32x16 (&prev)[NQW]) {
    if (block_masked(b - 1)) step(b, cur, prev, std::true_type{}, std::true_type{});
    else step(b, cur, prev, std::true_type{}, std::false_type{});
  };

  wait_tile(0);
  lds_barrier();  // every wavefront's part of tile 0 and the start values are in LDS
  if (kRing - 1 < nt) issue_tile(kRing - 1);
  if constexpr (PASS == 1 && kStartInRegs) {
#pragma unroll
    for (int qi = 0; qi < NQW; ++qi)
#pragma unroll
      for (int v4 = 0; v4 < 4; ++v4) {
        const f32x4 st = *(const f32x4 *)(s_start + (wq * NQW + qi) * 32 + 8 * v4 + 4 * half);
        start[qi][4 * v4 + 0] = st.x; start[qi][4 * v4 + 1] = st.y; start[qi][4 * v4 + 2] = st.z; start[qi][4 * v4 + 3] = st.w;
      }
  }
  if (active) {
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) kf[ks] = *frag_at(block_off(0), ks);
  }
  f32x16 accA[NQW], accB[NQW];
  step(0, accA, accB, std::false_type{}, std::false_type{});
  for (int b = 1; b < nblk; b += 2) {
    run_step(b, accB, accA);
    if (b + 1 < nblk) run_step(b + 1, accA, accB);
  }
  auto last_epilogue = [&](f32x16 (&last)[NQW]) {
    if (block_masked(nblk - 1)) epilogue(last, nblk - 1, std::true_type{});
    else epilogue(last, nblk - 1, std::false_type{});
  };
  if (active) {
    if ((nblk - 1) % 2 == 0) last_epilogue(accA);
    else last_epilogue(accB);
  }
  flush_if_unit_done(nblk - 1);

  if constexpr (PASS == 0) {
    float2 *s_st = (float2 *)s_part;  // [4 wavefronts][32 rows]
#pragma unroll
    for (int qi = 0; qi < NQW; ++qi) {
      // merge the two lane halves (same row, different keys)
      const float m_o = __shfl_xor(m_run[qi], 32), l_o = __shfl_xor(l_run[qi], 32);
      float m = fmaxf(m_run[qi], m_o);
      float l = l_run[qi] * fast_exp2(m_run[qi] - m) + l_o * fast_exp2(m_o - m);
      if constexpr (4 / WQ > 1) {
        // NQW == 1 here: merge the wavefronts that split the keys (idle ones carry (-big, 0))
        if (half == 0) s_st[wave * 32 + n] = make_float2(m, l);
        __syncthreads();
        if (wk == 0) {
          for (int o = 1; o < 4 / WQ; ++o) {
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

template <int DT, int HD, int NQW, int WQ>
int launch_score_cfg(int pass, const ScoreArgs &a, dim3 grid, hipStream_t s) {
  static std::once_flag once;
  static hipError_t attr_rc[2] = {hipSuccess, hipSuccess};
  auto k0 = score_kernel<DT, HD, NQW, WQ, 0>;
  auto k1 = score_kernel<DT, HD, NQW, WQ, 1>;
  std::call_once(once, [&] {   // both passes, once per process, whichever thread comes first
    attr_rc[0] = hipFuncSetAttribute(reinterpret_cast<const void *>(k0), hipFuncAttributeMaxDynamicSharedMemorySize, kScoreLdsBytes);
    attr_rc[1] = hipFuncSetAttribute(reinterpret_cast<const void *>(k1), hipFuncAttributeMaxDynamicSharedMemorySize, kScoreLdsBytes);
  });
  if (attr_rc[pass] != hipSuccess) return CHUNKKV_ERR_LAUNCH;
  hipLaunchKernelGGL(pass == 0 ? k0 : k1, grid, dim3(kThreads), kScoreLdsBytes, s, a);
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
