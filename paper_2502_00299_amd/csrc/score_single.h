// Single-pass observation-window scoring (Algorithm 1, first two steps) for bf16 and fp16 caches, head_dim 128,
// chunk sizes that divide 80 into a multiple of four chunks (5, 10, 20).
//
// K is streamed ONCE and nothing is rounded below fp32.  For every window row r the kernel keeps a reference
// m_r and forms e = exp2(logit * scale * log2e - m_r) in fp32 for every key; the e of one chunk are added up in
// registers, so after a PERIOD of 160 keys a lane holds the sums E[chunk][r] of the chunks it owns, relative to
// m_r.  These per-(chunk, row) sums and the reference they are relative to go to the workspace; the row's total
// follows from them (plus the window keys, which belong to no chunk).  A second, small kernel
// (single_scores_kernel in score_misc.hip) merges the per-range (reference, sum) pairs of a row into
// ref_r = m_r + log2(sum_r) and forms score[chunk] = sum_r E[chunk][r] * exp2(m[chunk][r] - ref_r).
//
// Who owns which key.  The logits come from v_mfma_f32_32x32x16 with the keys as the M dimension: a lane owns
// one window row (N index) and, of the 32 keys of a block, the 16 whose M index has bit 2 equal to its lane
// half.  Which key sits at which M index is the kernel's choice (the operand fragments are read from LDS row
// by row), and it is chosen so that both lane halves see the SAME chunk pattern in their registers: the chunks
// of a period alternate between the halves (half h owns chunks h, h + 2, ...), and register v of step t of a
// period holds position u = 16 t + v of the lane half's own sequence of 80 keys.  Position u belongs to own
// chunk u / c: a compile-time function of (t, v), so every exponential is added to its chunk's register with
// one plain add, no matrix product and no cross-lane traffic.
//
// The reference is lazy.  fp32 has room for e up to 2^100 before the sums are in danger, so the reference moves
// only when a step's sum reaches that bound (the first step of a range always does, its reference starts at
// -1e30); the step is then redone against the step's own maximum and the lane's sums are rescaled.  On ordinary
// inputs that happens once per range.  Values more than 2^126 below the reference vanish: their probability is
// below what fp32 chunk scores can represent.
//
// K: HBM -> LDS by buffer loads with an LDS destination (16 bytes per lane, rows past the end of the sequence
// read as zero).  The ring holds two periods; a period is 5 slots of 32 key rows, slot t holding the rows of
// step t in M-index order, so the permutation above lives in the global addresses of the loads and the operand
// reads are "lane register + compile-time slot offset".  The 16-byte segments of a row are XOR-swizzled by the
// M index (global-address side), so the reads of 16 consecutive lanes hit distinct banks.  One barrier per
// period: when every wavefront has read the last slot of period p, the loads of period p + 1 (issued a period
// earlier) are waited for and the whole of period p + 2 is issued into the half that p occupied, so 40 KB per
// workgroup are in flight for a full period.
//
// A wavefront holds NQ blocks of 32 window rows as resident operand fragments and the four wavefronts of a
// workgroup split the rows, so each K fragment read from LDS feeds NQ matrix instructions.  The work advances
// in micro-steps (one 32-key block against one 32-row block).  The instruction stream of a micro-step is laid
// out by hand: eight slots of one matrix instruction of the NEXT micro-step and the vector work of two keys of
// THIS one.  The kernel is bound by vector-instruction issue (16 scalings, 16 exponentials and 16 adds per
// micro-step and lane against 8 matrix instructions), which is why everything that is not one of those three
// has been moved out of the steady state.
#pragma once
#include <mutex>
#include <type_traits>

#include "score_impl.h"

namespace ckv {

constexpr int kSpPeriod = 160;                          // keys per period
constexpr int kSpHalf = 80;                             // keys of a period one lane half owns
constexpr int kSpSteps = 5;                             // 32-key blocks per period
constexpr int kSpStepBytes = 32 * 256;                  // one ring slot: 32 rows of 128 16-bit values
constexpr int kSpPeriodBytes = kSpSteps * kSpStepBytes; // 40 KB
constexpr int kSpRingBytes = 2 * kSpPeriodBytes;        // two periods
constexpr float kSpBig = 1.2676506e30f;                 // 2^100: a step whose sum reaches this is redone
constexpr int kSpLoadsPerPeriod = 2 * kSpSteps;         // 1 KB loads a wavefront issues per period
constexpr int kSpMaxSeg = 5;                            // chunk segments 16 consecutive keys can touch (c >= 5)

typedef unsigned int u32x3 __attribute__((ext_vector_type(3)));

// four non-negative finite fp32 values -> their rounded upper three bytes, packed into three dwords
__device__ __forceinline__ u32x3 pack24(float x, float y, float z, float w) {
  const uint32_t a = __float_as_uint(x) + 0x80u, b = __float_as_uint(y) + 0x80u;
  const uint32_t c = __float_as_uint(z) + 0x80u, d = __float_as_uint(w) + 0x80u;
  return u32x3{__builtin_amdgcn_perm(b, a, 0x05030201u), __builtin_amdgcn_perm(c, b, 0x06050302u),
               __builtin_amdgcn_perm(d, c, 0x07060503u)};
}

// eight non-negative finite fp32 values -> their upper 20 bits below the sign (8 exponent, 12 mantissa bits,
// rounded: relative 2^-13), packed into five dwords
__device__ __forceinline__ void pack20(const float (&v)[8], u32x4 &lo, uint32_t &hi) {
  uint32_t q[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) q[i] = (__float_as_uint(v[i]) + 0x400u) >> 11;
  lo.x = q[0] | (q[1] << 20);
  lo.y = (q[1] >> 12) | (q[2] << 8) | (q[3] << 28);
  lo.z = (q[3] >> 4) | (q[4] << 16);
  lo.w = (q[4] >> 16) | (q[5] << 4) | (q[6] << 24);
  hi = (q[6] >> 8) | (q[7] << 12);
}

// period-relative key of position u of lane half 0's own sequence (lane half 1: + C)
template <int C>
__host__ __device__ constexpr int sp_key(int u) { return 2 * C * (u / C) + u % C; }

template <int DT>
__device__ __forceinline__ f32x16 mma0(const u32x4 &a, const u32x4 &b) {  // first product of a chain: C = 0
  const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if constexpr (DT == CHUNKKV_BF16)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), z, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), z, 0, 0, 0);
}

// DT: chunkkv_dtype (16-bit), C: chunk size, NQ: 32-row blocks per wavefront (rows_pad = 128 * NQ)
template <int DT, int C, int NQ>
__global__ __launch_bounds__(kThreads, 2) void score_single_kernel(ScoreArgs a) {
  static_assert(is_16bit(DT), "the single-pass kernel takes bf16 or fp16 caches");
  static_assert(kSpHalf % C == 0 && (kSpHalf / C) % 4 == 0 && kSpHalf / C <= 16, "chunk size");
  static_assert(NQ == 1 || NQ == 2, "row blocks per wavefront");
  constexpr int S = kSpHalf / C;  // chunks per lane half and period
  constexpr int ROWB = 256, NKS = 8, ESZ = 2;

  extern __shared__ __align__(16) char smem[];   // kSpRingBytes

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wavefront-uniform, and known to be
  const int n = lane & 31, half = lane >> 5;
  const int bl = blockIdx.y / a.n_kv_heads, h = blockIdx.y % a.n_kv_heads, z = blockIdx.z;
  const int split = blockIdx.x;
  const int g = a.n_q_heads / a.n_kv_heads, w = a.window;
  const int L = pick(a.seq.seqlen, bl), P = L - w, nrows = g * w;
  const int64_t problem = ((int64_t)(a.leader0 + z) * a.batch_total + (a.batch0 + bl)) * a.n_kv_heads + h;

  const int np_total = (L + kSpPeriod - 1) / kSpPeriod;
  const int ppr = single_periods_per_range(np_total);
  const int u0 = split * ppr;
  const int u1 = u0 + ppr < np_total ? u0 + ppr : np_total;
  if (u0 >= np_total) return;
  const int np = u1 - u0;               // periods of this workgroup
  const int range0 = u0 * kSpPeriod;    // its first key

  const char *qbase = (const char *)pick(a.q, z) + ((int64_t)(a.batch0 + bl) * a.n_q_heads + (int64_t)h * g) * w * ROWB;
  const char *kbase = (const char *)pick(a.k, z) + (pick(a.seq.kv_base, bl) + (int64_t)h * a.kv_stride_head) * ESZ;
  const int64_t ktok = a.kv_stride_tok * ESZ;
  const float c1 = a.scale_log2e;

  // ---- K: HBM -> LDS.  Load j of a wavefront fills rows 8 wave + 4 j .. + 3 of a slot; lane l lands at row
  // 8 wave + 4 j + l / 16, 16-byte position l % 16, and fetches the segment that position holds after the
  // swizzle, of the key that M index stands for in step t.  M index 8 wave + 4 j + b is position
  // u = 16 t + 4 wave + b of lane half j, so the two loads of a step differ by a lane constant.
  const __amdgpu_buffer_rsrc_t krsrc =
      __builtin_amdgcn_make_buffer_rsrc((void *)kbase, 0, (int)((uint32_t)(L - 1) * (uint32_t)ktok + ROWB), 0x00020000);
  uint32_t klane[kSpSteps], kdelta;
  {
    const int b = lane / 16, pos = lane % 16;
    const int seg0 = pos ^ (8 * (wave & 1) + b), seg1 = seg0 ^ 4;   // M index & 15 = 8 (wave & 1) + 4 j + b
#pragma unroll
    for (int t = 0; t < kSpSteps; ++t) {
      const int u = 16 * t + 4 * wave + b;
      klane[t] = (uint32_t)((2 * C * (u / C) + u % C) * (int)ktok + seg0 * 16);
    }
    kdelta = (uint32_t)(C * (int)ktok + (seg1 - seg0) * 16);
  }
  // all five slots of period prel, into ring half prel & 1
  auto issue_period = [&](int prel) __attribute__((always_inline)) {
    const uint32_t off = (uint32_t)(range0 + prel * kSpPeriod) * (uint32_t)ktok;  // wavefront-uniform
    char *dst = smem + (prel & 1) * kSpPeriodBytes + wave * 2048;
#pragma unroll
    for (int t = 0; t < kSpSteps; ++t) {
      __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc, (__attribute__((address_space(3))) void *)(dst + t * kSpStepBytes), 16,
                                               klane[t], off, 0, 0);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc, (__attribute__((address_space(3))) void *)(dst + t * kSpStepBytes + 1024),
                                               16, klane[t] + kdelta, off, 0, 0);
    }
  };
  issue_period(0);
  if (np > 1) issue_period(1);

  // wavefronts whose rows are all padding only move K
  const bool active = wave * NQ * 32 < nrows;

  // ---- window queries: resident operand fragments (lane n: row n of the block, elements 16 ks + 8 half ..)
  u32x4 qf[NQ][NKS];
#pragma unroll
  for (int qi = 0; qi < NQ; ++qi) {
    const int row = (wave * NQ + qi) * 32 + n;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      qf[qi][ks] = u32x4{0, 0, 0, 0};
      if (row < nrows) qf[qi][ks] = *(const u32x4 *)(qbase + (int64_t)row * ROWB + (2 * ks + half) * 16);
    }
  }
  float m_run[NQ], l_run[NQ], slot[NQ][S];
  int lim[NQ];  // last key the row may see
#pragma unroll
  for (int qi = 0; qi < NQ; ++qi) {
    m_run[qi] = kNegBig;
    l_run[qi] = 0.f;
#pragma unroll
    for (int s = 0; s < S; ++s) slot[qi][s] = 0.f;
    const int row = (wave * NQ + qi) * 32 + n;
    lim[qi] = P + (row < nrows ? row % w : 0);
  }

  // ---- K operand fragments: lane (n, half) reads row n of a slot, segment 2 ks + half, at its swizzled position.
  // kaddr points into the ring half the reads currently go to; it is flipped (all values are below 8 KB, the
  // half offset 0xA000 has no bit in common with them) when the reads cross into the next period.
  uint32_t kaddr[NKS];
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) kaddr[ks] = (uint32_t)(n * ROWB + (((2 * ks + half) ^ (n & 15)) * 16));
  static_assert(kSpPeriodBytes == 0xA000 && 32 * ROWB <= 0x2000, "ring half flip");
  auto frag = [&](auto t_c, int ks) __attribute__((always_inline)) {
    constexpr int T = decltype(t_c)::value;
    return *(const u32x4 *)(smem + (kaddr[ks] + (uint32_t)(T * kSpStepBytes)));
  };

  // Two accumulator tiles: the matrix instructions of micro-step mu + 1 (one key block against one row block)
  // fill one while the exponentials of micro-step mu read the other.  All eight K fragments of the current
  // block are resident; fragment ks is re-read for the next block right behind its last product.
  f32x16 acc[2];
  u32x4 kf[NKS];
  // E and the references of this problem (byte offsets inside stay below 2^32).  Layout per period, with a
  // group = eight chunk sums of one lane half as 20-bit floats: [lane half][group][rows_pad] x 16 bytes, then
  // [lane half][group][rows_pad] x 4 bytes (c = 20 has four sums per lane half: [lane half][rows_pad] x 12 bytes,
  // 24-bit floats); m [rows_pad] floats.  Consecutive lanes write consecutive pieces.
  constexpr int G8 = S / 8;                                  // groups of eight sums per lane half
  constexpr int kPeriodRowBytes = S == 4 ? 24 : 2 * G8 * 20;  // E bytes per period and row
  char *e_problem = (char *)a.e_buf + (int64_t)problem * a.n_periods * a.rows_pad * kPeriodRowBytes;
  char *m_problem = (char *)a.m_period + (int64_t)problem * a.n_periods * a.rows_pad * 4;
  const uint32_t lane_row = (uint32_t)(wave * NQ * 32 + n);
  const uint32_t lane_m = lane_row * 4u;
  const int key_half = C * half;  // period-relative key of the lane half's position 0

  // logits of one micro-step; REFILL: the fragments are re-read from slot TR behind their product
  auto chain = [&](f32x16 &dst, auto qi_c, auto refill_c, auto tr_c) __attribute__((always_inline)) {
    constexpr int QI = decltype(qi_c)::value;
    constexpr bool REFILL = decltype(refill_c)::value;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      if (ks == 0) dst = mma0<DT>(kf[0], qf[QI][0]);
      else mma<DT>(dst, kf[ks], qf[QI][ks]);  // D[key][row]
      if constexpr (REFILL) kf[ks] = frag(tr_c, ks);
    }
  };

  // exponentials of one micro-step against the current reference: sums per chunk segment of the step (seg[]),
  // window keys (lw, masked periods only)
  auto exps = [&](const f32x16 &x, auto qi_c, int pkey0, auto t_c, auto masked_c, float (&seg)[kSpMaxSeg], float &lw)
      __attribute__((always_inline)) {
    constexpr int T = decltype(t_c)::value, QI = decltype(qi_c)::value;
    constexpr bool MASKED = decltype(masked_c)::value;
    const float negm = -m_run[QI];
    lw = 0.f;
    constexpr int U0 = 16 * T;
#pragma unroll
    for (int v4 = 0; v4 < 16; v4 += 4) {
      float e[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) e[i] = __builtin_fmaf(x[v4 + i], c1, negm);
#pragma unroll
      for (int i = 0; i < 4; ++i) e[i] = fast_exp2(e[i]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int u = U0 + v4 + i, sg = u / C - U0 / C;
        if constexpr (MASKED) {
          const int key = pkey0 + key_half + sp_key<C>(u);
          lw += (key >= P && key <= lim[QI]) ? e[i] : 0.f;   // window keys count for the row sum only
          e[i] = key < P ? e[i] : 0.f;
        }
        const bool first = v4 + i == 0 || (u % C == 0);
        seg[sg] = first ? e[i] : seg[sg] + e[i];
      }
    }
  };

  // The unmasked micro-step in issue order: eight slots of one matrix instruction of the NEXT micro-step (with
  // its fragment re-read) and the vector work of two keys of THIS one, software-pipelined over the slots (the
  // scaling of slot k + 1, the exponentials of slot k, the adds of slot k - 1), so that nothing in a slot
  // waits for anything in the same slot and the vector work of a slot takes about as long as its matrix
  // instruction.  Fences keep the compiler from regrouping the slots.
  auto fused = [&](f32x16 &dst, const f32x16 &x, auto qnx_c, auto refill_c, auto tr_c, auto qi_c, auto t_c,
                   float (&seg)[kSpMaxSeg]) __attribute__((always_inline)) {
    constexpr int T = decltype(t_c)::value, QI = decltype(qi_c)::value, QNX = decltype(qnx_c)::value;
    constexpr bool REFILL = decltype(refill_c)::value;
    constexpr int U0 = 16 * T;
    const float negm = -m_run[QI];
    float xs[2], es[2];
    xs[0] = __builtin_fmaf(x[0], c1, negm);
    xs[1] = __builtin_fmaf(x[1], c1, negm);
#pragma unroll
    for (int k = 0; k <= NKS; ++k) {
      if (k < NKS) {
        if (k == 0) dst = mma0<DT>(kf[0], qf[QNX][0]);
        else mma<DT>(dst, kf[k], qf[QNX][k]);
        if constexpr (REFILL) kf[k] = frag(tr_c, k);
      }
      // adds of slot k - 1
      if (k >= 1) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          const int v = 2 * (k - 1) + i, u = U0 + v, sg = u / C - U0 / C;
          const bool first = v == 0 || (u % C == 0);
          seg[sg] = first ? es[i] : seg[sg] + es[i];
        }
      }
      // exponentials of slot k
      if (k < NKS) {
        es[0] = fast_exp2(xs[0]);
        es[1] = fast_exp2(xs[1]);
      }
      // scaling of slot k + 1
      if (k + 1 < NKS) {
        xs[0] = __builtin_fmaf(x[2 * k + 2], c1, negm);
        xs[1] = __builtin_fmaf(x[2 * k + 3], c1, negm);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // One micro-step: (ring hand-over at the micro-step whose reads cross into the next period,) the matrix work
  // of the micro-step after it, the exponentials of this one.
  // prel: period relative to the range; T: step within the period; QI: row block; TILE: accumulator tile that
  // holds this micro-step's logits.
  auto micro = [&](int prel, auto t_c, auto qi_c, auto tile_c, auto masked_c) __attribute__((always_inline)) {
    constexpr int T = decltype(t_c)::value, QI = decltype(qi_c)::value, TILE = decltype(tile_c)::value;
    constexpr bool MASKED = decltype(masked_c)::value;
    constexpr bool STEP_END = QI == NQ - 1;                 // the next micro-step belongs to the next step
    constexpr int TNX = STEP_END ? (T + 1) % kSpSteps : T;  // its step ...
    constexpr int QNX = STEP_END ? 0 : QI + 1;              // ... and row block
    // if it is the last use of its block's fragments they are re-read for the block after (slot TR)
    constexpr bool REFILL = QNX == NQ - 1;
    constexpr int TR = (TNX + 1) % kSpSteps;
    // This micro-step's re-reads are the first that touch the next period: every wavefront has then read the
    // last slot of this period.  The loads of the next period, issued a period ago, are waited for; behind the
    // barrier the half this period occupied is free and takes the period after next.
    if constexpr (REFILL && TR == 0) {
      __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      __builtin_amdgcn_s_barrier();
      if (prel + 2 < np) issue_period(prel + 2);
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) kaddr[ks] ^= (uint32_t)kSpPeriodBytes;
    }
    if (active) {
      // (at the very end of the range the matrix work multiplies stale rows of the ring: in bounds, never used)
      const int pkey0 = range0 + prel * kSpPeriod;
      float seg[kSpMaxSeg], lw = 0.f;
      constexpr int NSEG = (16 * T + 15) / C - (16 * T) / C + 1;
      static_assert(NSEG <= kSpMaxSeg, "segments per step");
      if constexpr (MASKED) {
        chain(acc[TILE ^ 1], std::integral_constant<int, QNX>{}, std::integral_constant<bool, REFILL>{},
              std::integral_constant<int, TR>{});
        exps(acc[TILE], qi_c, pkey0, t_c, masked_c, seg, lw);
      } else {
        fused(acc[TILE ^ 1], acc[TILE], std::integral_constant<int, QNX>{}, std::integral_constant<bool, REFILL>{},
              std::integral_constant<int, TR>{}, qi_c, t_c, seg);
      }
      float tot = seg[0];
#pragma unroll
      for (int sg = 1; sg < NSEG; ++sg) tot += seg[sg];
      if constexpr (MASKED) tot += lw;
      if (__builtin_amdgcn_ballot_w64(tot >= kSpBig) != 0) {
        // rare: a sum reached 2^100 (always on the first step of a range).  Lanes that did move their
        // reference to the step's own maximum, rescale what they hold and redo the step.
        float bm = -3.0e38f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          float xv = acc[TILE][v];
          if constexpr (MASKED) xv = (pkey0 + key_half + sp_key<C>(16 * T + v)) <= lim[QI] ? xv : -3.0e38f;
          bm = fmaxf(bm, xv);
        }
        // the two lane halves of a row move together, so a row has one reference per period
        bm = fmaxf(bm, __shfl_xor(bm, 32));
        const bool mine = __shfl_xor(tot, 32) >= kSpBig || tot >= kSpBig;
        const float m_new = mine ? bm * c1 : m_run[QI];
        const float f = fast_exp2(m_run[QI] - m_new);
#pragma unroll
        for (int s = 0; s < S; ++s) slot[QI][s] *= f;
        l_run[QI] *= f;
        m_run[QI] = m_new;
        exps(acc[TILE], qi_c, pkey0, t_c, masked_c, seg, lw);
      }
      // commit: every segment goes to its chunk's register (the first segment of a chunk in a period starts
      // the register afresh)
#pragma unroll
      for (int sg = 0; sg < NSEG; ++sg) {
        constexpr int SL0 = (16 * T) / C;
        const int sl = SL0 + sg;
        const bool fresh = sl * C >= 16 * T;
        slot[QI][sl] = fresh ? seg[sg] : slot[QI][sl] + seg[sg];
      }
      if constexpr (MASKED) l_run[QI] += lw;
      if constexpr (T == kSpSteps - 1) {
        // end of the period: the sums and the reference they are relative to leave the lane.  Streaming
        // (non-temporal) stores: the 1.2 GB a launch writes is read back by the next kernel only, and a read
        // that follows plain stores of that size runs at 4.5 TB/s instead of 6 (the write-back competes)
        float sum = 0.f;
#pragma unroll
        for (int s = 0; s < S; ++s) sum += slot[QI][s];
        l_run[QI] += sum;
        const uint32_t pbase = (uint32_t)(u0 + prel) * (uint32_t)a.rows_pad;
        const uint32_t rp = (uint32_t)a.rows_pad, row = lane_row + (uint32_t)(QI * 32);
        char *pdst = e_problem + pbase * (uint32_t)kPeriodRowBytes;
        if constexpr (S == 4) {
          __builtin_nontemporal_store(pack24(slot[QI][0], slot[QI][1], slot[QI][2], slot[QI][3]),
                                      (u32x3 *)(pdst + ((uint32_t)half * rp + row) * 12u));
        } else {
#pragma unroll
          for (int g8 = 0; g8 < G8; ++g8) {
            float v8[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) v8[i] = slot[QI][8 * g8 + i];
            u32x4 lo;
            uint32_t hi;
            pack20(v8, lo, hi);
            const uint32_t cell = ((uint32_t)(half * G8 + g8)) * rp + row;
            __builtin_nontemporal_store(lo, (u32x4 *)(pdst + cell * 16u));
            __builtin_nontemporal_store(hi, (uint32_t *)(pdst + (uint32_t)(2 * G8) * rp * 16u + cell * 4u));
          }
        }
        if (half == 0) __builtin_nontemporal_store(m_run[QI], (float *)(m_problem + (pbase * 4u + lane_m + (uint32_t)(QI * 32 * 4))));
      }
    }
  };

  // one step (all row blocks of the wavefront); P0: accumulator tile of the step's first micro-step
  auto step = [&](int prel, auto t_c, auto p0_c, auto masked_c) __attribute__((always_inline)) {
    constexpr int P0 = decltype(p0_c)::value;
    micro(prel, t_c, std::integral_constant<int, 0>{}, std::integral_constant<int, P0>{}, masked_c);
    if constexpr (NQ == 2)
      micro(prel, t_c, std::integral_constant<int, 1>{}, std::integral_constant<int, P0 ^ 1>{}, masked_c);
  };
  // one period; PP: tile of its first micro-step (NQ = 2: always 0; NQ = 1: alternates with the period)
  auto period = [&](int prel, auto pp_c, auto masked_c) __attribute__((always_inline)) {
    constexpr int PP = decltype(pp_c)::value;
    constexpr int ALT = NQ == 1 ? 1 : 0;  // the tile alternates from step to step
    step(prel, std::integral_constant<int, 0>{}, std::integral_constant<int, PP>{}, masked_c);
    step(prel, std::integral_constant<int, 1>{}, std::integral_constant<int, PP ^ ALT>{}, masked_c);
    step(prel, std::integral_constant<int, 2>{}, std::integral_constant<int, PP>{}, masked_c);
    step(prel, std::integral_constant<int, 3>{}, std::integral_constant<int, PP ^ ALT>{}, masked_c);
    step(prel, std::integral_constant<int, 4>{}, std::integral_constant<int, PP>{}, masked_c);
  };

  // ---- prologue: period 0 landed (the loads of period 1 may still be out), fragments of block 0, logits of
  // micro-step 0
  if (np > 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm(kSpLoadsPerPeriod));
  else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
  __builtin_amdgcn_s_barrier();
  if (active) {
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) kf[ks] = frag(std::integral_constant<int, 0>{}, ks);
    chain(acc[0], std::integral_constant<int, 0>{}, std::integral_constant<bool, NQ == 1>{}, std::integral_constant<int, 1>{});
  }

  // periods whose keys are all prefix keys run without masks
  int n_clean = (P - range0) / kSpPeriod;
  n_clean = n_clean < 0 ? 0 : (n_clean > np ? np : n_clean);
  int prel = 0;
  if constexpr (NQ == 2) {
    for (; prel < n_clean; ++prel) period(prel, std::integral_constant<int, 0>{}, std::false_type{});
    for (; prel < np; ++prel) period(prel, std::integral_constant<int, 0>{}, std::true_type{});
  } else {
    for (; prel + 2 <= n_clean; prel += 2) {
      period(prel, std::integral_constant<int, 0>{}, std::false_type{});
      period(prel + 1, std::integral_constant<int, 1>{}, std::false_type{});
    }
    for (; prel < np; ++prel) {
      if (prel & 1) period(prel, std::integral_constant<int, 1>{}, std::true_type{});
      else period(prel, std::integral_constant<int, 0>{}, std::true_type{});
    }
  }

  // per-range (reference, sum) of every row for the merge (the lane halves share the reference)
  if (active) {
#pragma unroll
    for (int qi = 0; qi < NQ; ++qi) {
      const int row = (wave * NQ + qi) * 32 + n;
      const float l = l_run[qi] + __shfl_xor(l_run[qi], 32);
      if (half == 0) a.part_stats[(problem * a.max_split + split) * a.rows_pad + row] = make_float2(m_run[qi], l);
    }
  }
}

template <int DT, int C, int NQ>
int launch_single_cfg(const ScoreArgs &a, dim3 grid, hipStream_t s) {
  static std::once_flag once;
  static hipError_t attr_rc = hipSuccess;
  auto kern = score_single_kernel<DT, C, NQ>;
  std::call_once(once, [&] {
    attr_rc = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, kSpRingBytes);
  });
  if (attr_rc != hipSuccess) return CHUNKKV_ERR_LAUNCH;
  hipLaunchKernelGGL(kern, grid, dim3(kThreads), kSpRingBytes, s, a);
  return hipGetLastError() == hipSuccess ? CHUNKKV_OK : CHUNKKV_ERR_LAUNCH;
}

// every compiled geometry of one storage type: chunk size x row blocks per wavefront
template <int DT>
int launch_single_dt(const ScoreArgs &a, dim3 grid, hipStream_t s) {
  const int nq = a.rows_pad / 128;
  if (nq != 1 && nq != 2) return CHUNKKV_ERR_UNSUPPORTED;
  switch (a.chunk) {
    case 5: return nq == 1 ? launch_single_cfg<DT, 5, 1>(a, grid, s) : launch_single_cfg<DT, 5, 2>(a, grid, s);
    case 10: return nq == 1 ? launch_single_cfg<DT, 10, 1>(a, grid, s) : launch_single_cfg<DT, 10, 2>(a, grid, s);
    case 20: return nq == 1 ? launch_single_cfg<DT, 20, 1>(a, grid, s) : launch_single_cfg<DT, 20, 2>(a, grid, s);
    default: return CHUNKKV_ERR_UNSUPPORTED;
  }
}

}  // namespace ckv
