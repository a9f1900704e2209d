// Fused quantized attention kernel for gfx950: the inner loop and epilogue of the paper's
// Algorithm 1.  One workgroup (4 wavefronts) owns one 128-query smoothing block of one
// (batch, head); each wavefront owns 32 queries and walks the 64-key blocks.
//
// The score tile is computed transposed, S^T = K^ Q^^T, with 32x32 MFMAs (v_mfma_i32_32x32x32_i8 in
// the 8-bit mode, the FP6 operand format of v_mfma_f32_32x32x64_f8f6f4 in the 4-bit mode): rows are
// keys, columns are queries, so a lane holds ONE query (column lane%32) and, thanks to the row
// permutation baked into the packed K^ layout, 16 consecutive keys per 32-key tile.  Row max
// and row sum are therefore lane-local plus one exchange between the two lane halves, one
// lane needs one delta_Q and one delta_K per tile (Sec. 3.2's per-thread principle on this
// accumulator layout; finer key scales are a template option), and the FP8 P~ registers are directly the B operand of
// O^T = V^^T P~^T (v_mfma_f32_32x32x64_f8f6f4, K = 64 = one accumulation block).  The
// instruction sums the block's 64 products internally (level 1 of Sec. 3.4) and adds its C
// operand - the running O - in full FP32 (level 2).
#include "sage_common.h"

namespace sage {

struct AttnParams {
  const int8_t* q_codes;
  const int8_t* k_codes;
  const uint8_t* v_codes;
  const float* q_scale;
  const float* k_scale;
  const float* v_scale;
  const float* v_mean;    // null, or the token mean of V to add back (smooth-V option)
  const float* delta_s;
  void* out;
  int H, Hkv, N, Nk, nQb, nKb, total_tiles;   // N queries, Nk keys (of the longest sequence)
  TensorMap om;           // where the rows of `out` start
  float kappa;
  SeqMap seq;             // variable-length batch: N, Nk, nQb, nKb describe the longest sequence
  float* lse;             // null, or where the row log-sum-exp goes
  const float* q_corr;    // kappa * <q_r, mean(K)> per query (read only with lse)
  int B;
  // key range split over several workgroups per tile (few tiles, many keys): partial results, merged by k_merge_splits
  int splits;             // workgroups per tile (1: no split)
  float* part_o;          // [tile * splits + s][128 rows][d]: unnormalized O under the chunk's own exponent offset
  float* part_el;         // [tile * splits + s][128 rows][2]: that offset e and the sum l under it
};

// Split of a tile's key blocks [0, nblk) into chunks, one workgroup each (Sec. 2.1, Eq. 1: the running maximum / sum /
// output of disjoint key sets combine by the same rule that combines consecutive blocks).  Every chunk must start
// with a block in which every query of the tile sees a key, so the chunks divide the first n_vis blocks - those
// with a key visible to the tile's first query - evenly, C = ceil(n_vis / S) blocks each, and the last non-empty
// chunk runs on to nblk; chunks s >= ceil(n_vis / C) are empty.
struct KeyChunk { int j0, j1; };
__host__ __device__ inline KeyChunk key_chunk(int s, int S, int nblk, int n_vis) {
  const int C = (n_vis + S - 1) / S;
  const int used = C > 0 ? (n_vis + C - 1) / C : 0;
  KeyChunk k;
  k.j0 = s * C;
  k.j1 = s + 1 >= used ? nblk : (s + 1) * C;
  if (s >= used) { k.j0 = k.j1 = 0; }
  return k;
}

// Score accumulators of one wavefront for one 64-key block: 2 key tiles x (32 keys x 32
// queries).  ka: the block's K^ chunks already in registers (chunk (s, kt) at ka[2s + kt]); qreg:
// the wavefront's Q^ B-operands (one per 32-channel step).  Element acc[kt][v] belongs to key
// 32*kt + 16*(lane/32) + v of the block and to query lane%32 of the wavefront.
// INT8 mode: v_mfma_i32_32x32x32_i8, int32 accumulators.  INT4 mode: the codes are 6-bit FP6 E2M3
// values and feed v_mfma_f32_32x32x64_f8f6f4 in its FP6 operand format (twice the rate of the 8-bit
// formats); the FP32 accumulators hold the exact integers.  Either way the result is returned as
// raw 32-bit lanes.
// The product is issued one MFMA ("step") at a time so that the steps can be spread between
// pieces of vector work: step I works on key tile I % 2 and contraction piece I / 2 (64 channels
// in the INT4 mode, 32 in the INT8 mode); the first piece of a tile starts from a zero accumulator.
// Operand registers: INT8 mode one 16-byte chunk per (piece, tile); INT4 mode one FP6 payload (24
// bytes in the low 6 dwords of an 8-dword operand) per (piece, tile).
template <bool INT4> struct QkOperand { typedef v4i type; };
template <> struct QkOperand<true> { typedef v8i type; };
template <bool INT4> using qk_operand_t = typename QkOperand<INT4>::type;
template <int D, bool INT4> constexpr int qk_pieces() { return INT4 ? D / 64 : D / 32; }
template <int D, bool INT4> constexpr int qk_steps() { return 2 * qk_pieces<D, INT4>(); }
template <int D, bool INT4> struct KBlockRegs { typedef qk_operand_t<INT4> type[2 * (INT4 ? D / 64 : D / 32)]; };

template <int D, bool INT4, int I>
__device__ __forceinline__ void qk_step(const typename QkOperand<INT4>::type (&ka)[qk_steps<D, INT4>()],
                                        const typename QkOperand<INT4>::type (&qreg)[qk_pieces<D, INT4>()],
                                        v16i (&acc)[2]) {
  constexpr int KT = I & 1, S = I >> 1;
  if constexpr (INT4) {
    v16f c;
#pragma unroll
    for (int v = 0; v < 16; ++v) c[v] = S == 0 ? 0.0f : __int_as_float(acc[KT][v]);
    // operand format 2 = FP6 E2M3 for both A and B
    c = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(ka[S * 2 + KT], qreg[S], c, 2, 2, 0, 0, 0, 0);
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[KT][v] = __float_as_int(c[v]);
  } else {
    v16i c;
#pragma unroll
    for (int v = 0; v < 16; ++v) c[v] = S == 0 ? 0 : acc[KT][v];
    acc[KT] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ka[S * 2 + KT], qreg[S], c, 0, 0, 0);
  }
}
template <int D, bool INT4, int I = 0>
__device__ __forceinline__ void qk_tile(const typename QkOperand<INT4>::type (&ka)[qk_steps<D, INT4>()],
                                        const typename QkOperand<INT4>::type (&qreg)[qk_pieces<D, INT4>()],
                                        v16i (&acc)[2]) {
  if constexpr (I < qk_steps<D, INT4>()) {
    qk_step<D, INT4, I>(ka, qreg, acc);
    qk_tile<D, INT4, I + 1>(ka, qreg, acc);
  }
}

// One (piece, tile) operand out of a packed K^ block or Q^ tile at `base` (LDS or global): INT8
// mode chunk `op`*64 + lane; INT4 mode the lane's 16 bytes of op's first plane and 8 bytes of its
// second plane.
template <bool INT4, typename Ptr>
__device__ __forceinline__ typename QkOperand<INT4>::type load_qk_operand(Ptr base, int op, int lane) {
  if constexpr (INT4) {
    const v4i lo = base[op * (OP6_BYTES / 16) + lane];
    const uint2 hi = *reinterpret_cast<const uint2*>(reinterpret_cast<const char*>(&base[op * (OP6_BYTES / 16) + 64]) + 8 * lane);
    v8i r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = (int)hi.x; r[5] = (int)hi.y; r[6] = 0; r[7] = 0;
    return r;
  } else {
    return base[op * 64 + lane];
  }
}

// The K^ operands of one block out of LDS (blk: the block's packed image).
// INT4 mode: an operand is a 16-byte read plus an 8-byte read (its "tail").  Left free, the compiler pairs the
// tails of two operands into one two-address read and then moves the halves of its result next to their
// operands' first four registers, two vector instructions per operand in a loop that is bound by them.  The
// empty statement after every operand is a fence for memory accesses: reads cannot be merged across it, so
// every tail stays a read of its own that lands where its operand wants it, while the compiler still knows
// about every read and waits for it before the first use.
template <int D, bool INT4, typename Ptr>
__device__ __forceinline__ void read_k_block(Ptr blk, int lane, typename KBlockRegs<D, INT4>::type& ka) {
  constexpr int NS = qk_steps<D, INT4>();
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    ka[i] = load_qk_operand<INT4>(blk, i, lane);
    if constexpr (INT4) asm volatile("" ::: "memory");
  }
}

// Per-wavefront running state of Algorithm 1's inner loop.
template <int D> struct RowState {
  v16f O[D / 32];   // cross-block FP32 accumulator; O[ct][v]: channel 32ct + 8(v/4) + 4(lane/32) + v%4
  float m_run;      // running max of the base-2 scores of this lane's query
  float l_run;      // this lane's share of the running sum of 448 * P~
};

// Quantization granularity of the keys as the kernel sees it (template parameter GM): a lane's 32
// scores of a block are (key tile KT, quad G, R) = key 32 KT + 16 (lane / 32) + 4 G + R, so
//   GM 0: one scale per run of 16 keys = one per key tile  (2 per lane and block; queries in pairs),
//   GM 1: one scale per run of 4 keys  = one per quad      (8 per lane and block; every query its own),
//   GM 2: one scale per key            = one per score     (32 per lane and block; every query its own).
// KeyScales: the block's key scales this lane needs; Factors: c = fl32(fl32(delta_Q delta_K) kappa).
template <int GM> struct KeyScales;
template <> struct KeyScales<0> { float s[2]; };
template <> struct KeyScales<1> { v4f s[2]; };
template <> struct KeyScales<2> { v4f s[2][4]; };
template <int GM> struct Factors;
template <> struct Factors<0> {
  float c[2];
  __device__ __forceinline__ void set(float dq, float kappa, const KeyScales<0>& k) {
    c[0] = __fmul_rn(__fmul_rn(dq, k.s[0]), kappa);
    c[1] = __fmul_rn(__fmul_rn(dq, k.s[1]), kappa);
  }
  __device__ __forceinline__ float at(int kt, int, int) const { return c[kt]; }
};
template <> struct Factors<1> {
  float c[2][4];
  __device__ __forceinline__ void set(float dq, float kappa, const KeyScales<1>& k) {
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int g = 0; g < 4; ++g) c[kt][g] = __fmul_rn(__fmul_rn(dq, k.s[kt][g]), kappa);
    }
  }
  __device__ __forceinline__ float at(int kt, int g, int) const { return c[kt][g]; }
};
template <> struct Factors<2> {
  float c[2][4][4];
  __device__ __forceinline__ void set(float dq, float kappa, const KeyScales<2>& k) {
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
#pragma unroll
        for (int r = 0; r < 4; ++r) c[kt][g][r] = __fmul_rn(__fmul_rn(dq, k.s[kt][g][r]), kappa);
      }
    }
  }
  __device__ __forceinline__ float at(int kt, int g, int r) const { return c[kt][g][r]; }
};
// The 8-bit mode has no Delta-S in its score line: the dequantization product is fused into the exponent's
// argument, 2^(fma(acc, c, -m)), one rounding, whatever the granularity of the key scales (with a scale per key
// nothing is saved - the maximum needs the products anyway - but the value that decides the FP8 code of P~ is
// formed the same way for every group map).
template <bool INT4, int GM> constexpr bool fused_factor() { return !INT4; }

// Middle part of one block of Algorithm 1's inner loop for one wavefront, cut into pieces of four
// keys (one "group": registers 4G..4G+3 of key tile KT) so that MFMAs can be issued between them.
//
// dequant_group: the raw scores of the group are dequantized (+ Delta-S) into sc, in base 2
// (Algorithm 1, score line); MASKED adds the causal diagonal (keys past last_visible) and the
// padded keys (n_keys and beyond).  In the INT8
// mode there is no Delta-S and one positive factor c per key tile, so sc keeps the accumulators
// as floats: the maximum commutes with the factor and the product is fused into the exponent's
// argument (exp_group), one instruction less per score.
template <bool INT4, bool CAUSAL, bool MASKED, int GM, int KT, int G>
__device__ __forceinline__ void dequant_group(const v16i (&raw)[2], v16i (&sc)[2], const Factors<GM>& fac, int half,
                                              int key0, int last_visible, int n_keys) {
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    float x;
    if constexpr (INT4) {
      // On entry sc holds the block's Delta-S values (read from LDS straight into these registers): the score is
      // one fused multiply-add in place (the two-operand encoding, which issues faster than the three-operand
      // one).  Written as an ordinary expression, not as inline assembly: the compiler must see that it reads the
      // accumulators of a matrix instruction, or it cannot keep the wait states that read needs.
      x = __builtin_fmaf(__int_as_float(raw[KT][4 * G + r]), fac.at(KT, G, r), __int_as_float(sc[KT][4 * G + r]));
    }
    else x = (float)raw[KT][4 * G + r];       // 8-bit mode: the factor is applied inside the exponent's argument
    if constexpr (MASKED) {
      const int key = key0 + 32 * KT + 16 * half + 4 * G + r;
      if (key >= n_keys || (CAUSAL && key > last_visible)) x = -INFINITY;
    }
    sc[KT][4 * G + r] = __float_as_int(x);
  }
}

// update_max: running max over the block's 64 dequantized scores of this lane's query (Eq. 1 /
// Algorithm 1); takes the previous block's exponent offset in m_sub and returns the new one there, and
// alpha = 2^(old offset - new offset).
template <int D, bool INT4, int GM, int PVF>
__device__ __forceinline__ float update_max(RowState<D>& st, const v16i (&acc)[2], const Factors<GM>& fac,
                                            float& m_sub) {
  float mx;
  if constexpr (!fused_factor<INT4, GM>()) {
    mx = fmaxf(__int_as_float(acc[0][0]), __int_as_float(acc[1][0]));
#pragma unroll
    for (int v = 1; v < 16; ++v)   // one v_max3_f32 per step
      mx = fmaxf(fmaxf(mx, __int_as_float(acc[0][v])), __int_as_float(acc[1][v]));
  } else if constexpr (GM == 0) {
    // per key tile: max of the accumulators, then the tile's factor (c >= 0, so the order does not
    // matter; a fully masked tile with c = 0 gives NaN, which fmaxf drops)
    float m0 = __int_as_float(acc[0][0]), m1 = __int_as_float(acc[1][0]);
#pragma unroll
    for (int v = 1; v < 16; v += 2) {
      m0 = fmaxf(fmaxf(m0, __int_as_float(acc[0][v])), __int_as_float(acc[0][(v + 1) & 15]));
      m1 = fmaxf(fmaxf(m1, __int_as_float(acc[1][v])), __int_as_float(acc[1][(v + 1) & 15]));
    }
    // |c|: the pipeline's last update works on a stale, fully masked block whose scales are arbitrary
    // bits; -inf * |c| is -inf or NaN (dropped) whatever they are, so the running max stays intact
    mx = fmaxf(__fmul_rn(m0, fabsf(fac.at(0, 0, 0))), __fmul_rn(m1, fabsf(fac.at(1, 0, 0))));
  } else if constexpr (GM == 1) {
    // the same per quad
    mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float a = fmaxf(fmaxf(__int_as_float(acc[kt][4 * g]), __int_as_float(acc[kt][4 * g + 1])),
                              fmaxf(__int_as_float(acc[kt][4 * g + 2]), __int_as_float(acc[kt][4 * g + 3])));
        mx = fmaxf(mx, __fmul_rn(a, fabsf(fac.at(kt, g, 0))));
      }
    }
  } else {
    // a scale per key: the maximum of the products themselves (a masked score is -inf whatever its factor)
    mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
      for (int v = 0; v < 16; v += 2)
        mx = fmaxf(fmaxf(mx, __fmul_rn(__int_as_float(acc[kt][v]), fabsf(fac.at(kt, v / 4, v % 4)))),
                   __fmul_rn(__int_as_float(acc[kt][v + 1]), fabsf(fac.at(kt, (v + 1) / 4, (v + 1) % 4))));
    }
  }
  {
    // the other half of the wavefront holds the other 32 keys of the same query
    const unsigned u = __float_as_uint(mx);
    const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
  }
  const float m_new = fmaxf(st.m_run, mx);
  // The static scale of P~ (Sec. 3.3: *448; *57344 or *127 for the other data types) is folded into the exponent:
  // E = scale * P~ = 2^(S - e), e = m - log2(scale).  Rounded to nearest, e could come out below m - log2(scale) and
  // the row's largest E above the scale - for scores beyond 2^19 far enough to overflow the 8-bit format, whose
  // conversion then gives NaN.  So m is first nudged upward by |m| 2^-22 (two to four units of its last place):
  // E <= scale whatever the roundings; the factor 2^-(2^-22 |m|) on P~ cancels in O / l.  The previous sums are
  // rescaled by the power of two of the offsets' difference (2^-inf = 0 on the first block), so O and l stay
  // sums under the current offset exactly.
  const float e_new = __fmaf_rn(fabsf(m_new), 0x1p-22f, m_new) -
                      (PVF == PV_INT8 ? LOG2_127 : (PVF == PV_E5M2 ? LOG2_57344 : LOG2_448));
  const float alpha = __builtin_amdgcn_exp2f(m_sub - e_new);      // m_sub: the offset of the previous block
  m_sub = e_new;
  st.m_run = m_new;
  return alpha;
}

// exp_group: 448 * P~ = 2^(S - m_sub) for the group (INT8 mode: S = sc * c, fused), its row-sum share
// added to ls, its FP8 codes written into word 4*KT + G of the P~ operand.
template <bool INT4, bool MASKED, int GM, int PVF, int KT, int G>
__device__ __forceinline__ void exp_group(const v16i (&acc)[2], const Factors<GM>& fac, float m_sub, v8i& pb,
                                          float& ls) {
  float e[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const float x = __int_as_float(acc[KT][4 * G + r]);
    float arg;
    if constexpr (!fused_factor<INT4, GM>()) {
      arg = x - m_sub;
    } else {
      arg = __fmaf_rn(x, fac.at(KT, G, r), -m_sub);
      if constexpr (MASKED) arg = x == -INFINITY ? -INFINITY : arg;   // also when c = 0
    }
    e[r] = __builtin_amdgcn_exp2f(arg);
    ls += e[r];
  }
  int wd = __float_as_int(e[0]);   // any value: both halves are overwritten below
  if constexpr (PVF == PV_INT8) {
    // rint(127 P~) clipped to [0, 127] as bytes (the conversion is exact on the rounded values).  The clip
    // matters: for scores beyond 2^16 the rounding of m - log2(127) lets the row's largest term come out as
    // 127 * 2^(half an ulp of m) > 127.5, and a byte of 128 would be read as -128 by the integer MFMA.
#pragma unroll
    for (int r = 0; r < 4; ++r)
      wd = (int)__builtin_amdgcn_cvt_pk_u8_f32(rintf(fminf(e[r], INT8_PV_MAX)), (unsigned)r, (unsigned)wd);
  } else if constexpr (PVF == PV_E5M2) {
    wd = __builtin_amdgcn_cvt_pk_bf8_f32(e[0], e[1], wd, false);
    wd = __builtin_amdgcn_cvt_pk_bf8_f32(e[2], e[3], wd, true);
  } else {
    wd = __builtin_amdgcn_cvt_pk_fp8_f32(e[0], e[1], wd, false);
    wd = __builtin_amdgcn_cvt_pk_fp8_f32(e[2], e[3], wd, true);
  }
  pb[KT * 4 + G] = wd;
}

// Second half: the two-level accumulation of Sec. 3.4 on gfx950.  One v_mfma_f32_32x32x64_f8f6f4 has
// K = 64 = b_kv: the instruction sums the block's 64 FP8 products in its internal accumulator
// (level 1, confined to this block) and then adds its C operand in full FP32 (level 2: the
// cross-block accumulator O; measured - C passes through bit-exactly and C + product keeps FP32
// precision).  So O is the C/D operand, pre-scaled by alpha = 2^(m_old - m_new) only when some
// query of the wavefront actually moved its running max in this block.
template <int D>
__device__ __forceinline__ void block_rescale(RowState<D>& st, float alpha) {
  if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
#pragma unroll
    for (int ct = 0; ct < D / 32; ++ct) {
#pragma unroll
      for (int v = 0; v < 16; ++v) st.O[ct][v] = __fmul_rn(alpha, st.O[ct][v]);
    }
  }
}
// With INT8 codes the block's product is an integer matrix product (two K = 32 instructions) into a
// fresh int32 accumulator - level 1 of Sec. 3.4 as the paper describes it - which is then converted and
// added to O in FP32 (level 2): 32 more vector instructions per channel tile and block.
template <int D, int CT, int PVF>
__device__ __forceinline__ void pv_step(RowState<D>& st, const v4i (&va)[2 * (D / 32)], const v8i& pb) {
  if constexpr (PVF == PV_INT8) {
    const v4i p0 = {pb[0], pb[1], pb[2], pb[3]}, p1 = {pb[4], pb[5], pb[6], pb[7]};
    v16i r;
#pragma unroll
    for (int v = 0; v < 16; ++v) r[v] = 0;
    r = __builtin_amdgcn_mfma_i32_32x32x32_i8(va[CT * 2 + 0], p0, r, 0, 0, 0);
    r = __builtin_amdgcn_mfma_i32_32x32x32_i8(va[CT * 2 + 1], p1, r, 0, 0, 0);
#pragma unroll
    for (int v = 0; v < 16; ++v) st.O[CT][v] = __fadd_rn(st.O[CT][v], (float)r[v]);
    return;
  }
  v8i a;
  const v4i a0 = va[CT * 2 + 0];
  const v4i a1 = va[CT * 2 + 1];
  a[0] = a0[0]; a[1] = a0[1]; a[2] = a0[2]; a[3] = a0[3];
  a[4] = a1[0]; a[5] = a1[1]; a[6] = a1[2]; a[7] = a1[3];
  // operand formats: 0 = E4M3, 1 = E5M2, for both V^ (A) and P^ (B)
  constexpr int FMT = PVF == PV_E5M2 ? 1 : 0;
  st.O[CT] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, pb, st.O[CT], FMT, FMT, 0, 0, 0, 0);
}

// Wavefronts per SIMD the attention kernel is built for, by variant.  d = 128 with the default key groups: 3 (168
// registers: one block's scores live at a time, no software pipeline inside a wavefront - the other two wavefronts
// of the SIMD fill its waits; measured 8 - 9 % faster than 2 wavefronts with the score product of the next block
// pipelined into the exponentials of the current one).  The variants that hold more per-block state (a key scale
// per quad or per key, the INT8 P~V product) would spill at 168 registers and keep the pipelined form at 2.
// d = 64: half the accumulator, one more wavefront.  d = 256: 2 (the accumulator alone is 128 registers; 254 in all,
// two LDS stages of 29 KB so that two workgroups fit a CU; 2140 TOPS on the causal 8k case against 1254 for the
// pipelined form at one wavefront per SIMD, whose accumulators had to live in the second half of the register file).
#ifndef SAGE_OCC_D128
#define SAGE_OCC_D128 3
#endif
#ifndef SAGE_OCC_D64
#define SAGE_OCC_D64 4
#endif
#ifndef SAGE_OCC_D256
#define SAGE_OCC_D256 2
#endif
template <int D, int GM, int PVF> constexpr int attn_occupancy() {
  if (D == 256) return SAGE_OCC_D256;
  if (D == 128) return (GM == 0 && PVF != PV_INT8) ? SAGE_OCC_D128 : 2;
  return GM == 0 && PVF != PV_INT8 ? SAGE_OCC_D64 : (SAGE_OCC_D64 >= 3 ? 3 : 2);
}

// Global -> LDS copies without a register stop (the LDS-DMA form of the global load: lane l's
// 16 or 4 bytes land at LDS byte m0 + 16*l or m0 + 4*l).  Issued from inline assembly so that
// the wait for them is placed by hand - one vmcnt wait right before the barrier that publishes a
// stage - instead of in front of every later LDS read.  gbase is wavefront-uniform.
__device__ __forceinline__ void dma_b128(const void* gbase, unsigned voff, unsigned lds_byte) {
  unsigned m0_after;    // M0 is declared as a result, so the compiler knows the statement overwrites it
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, %3"
               : "={m0}"(m0_after) : "s"(lds_byte), "v"(voff), "s"(gbase) : "memory");
}
__device__ __forceinline__ void dma_b32(const void* gbase, unsigned voff, unsigned lds_byte) {
  unsigned m0_after;
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, %3"
               : "={m0}"(m0_after) : "s"(lds_byte), "v"(voff), "s"(gbase) : "memory");
}

// An empty use of a register: the compiler must have the value complete (its load waited for) here.
__device__ __forceinline__ void use_now(int x) { asm volatile("" :: "v"(x)); }
__device__ __forceinline__ void use_now(float x) { asm volatile("" :: "v"(x)); }

// where query r of (batch b, head h) goes in the log-sum-exp output: [B, H, N], or [H, total_q] for a
// variable-length batch
__device__ __forceinline__ size_t lse_index(const AttnParams& p, const Seq& sq, int b, int h, int r) {
  if (p.seq.cu_q) return (size_t)h * (size_t)p.seq.cu_q[p.B] + sq.q0 + r;
  return ((size_t)b * p.H + h) * p.N + r;
}

// PACK (with SPLIT; short queries, grouped KV heads): a tile holds ALL queries of the G = H / H_kv query heads that
// share one KV head - column c of the tile is query c % n of head c / n of the group, n the sequence's query count
// (G N <= 128 for the longest sequence, G <= PACK_G) - so
// the KV head's codes are walked once for the whole group instead of once per query head with 128 - N idle columns
// each.  Everything that belongs to a query (its codes, scale, Delta-S row, output row) is then looked up per lane.
template <int D, bool INT4, bool CAUSAL, bool BF16, int GM, int PVF, bool SPLIT = false, bool PACK = false>
__global__ void __launch_bounds__(256, (attn_occupancy<D, GM, PVF>())) k_attn_fwd(const AttnParams p) {
  constexpr bool OCC3 = attn_occupancy<D, GM, PVF>() >= (D == 256 ? 2 : 3);     // the form without a software pipeline
  static_assert(!PACK || (SPLIT && OCC3 && GM == 0), "packed tiles come with the split key range and the default groups");
  constexpr int DSR = PACK && INT4 ? PACK_G : 1;   // Delta-S rows per stage
  constexpr int KSC = GM == 0 ? 4 : (GM == 1 ? 16 : 64);    // key scales per block
  constexpr int QG = GM == 0 ? QGROUP : 1;                  // queries per scale
  constexpr int CT = D / 32;          // 32-channel tiles of the output
  constexpr int KC = D * BKV / 16;    // 16-byte chunks of one V^ block
  constexpr int KCK = (int)(k_block_bytes(D, INT4) / 16);   // 16-byte chunks of one K^ block
  constexpr int CPT = KC / 256;       // V^ chunks per thread per block copy (2 or 1)
  constexpr int CPTK = (KCK + 255) / 256;   // K^ copy rounds (the last one may skip some wavefronts)
  constexpr int MINC = KCK / 256 + CPT;     // copies every wavefront issues per block, at least
  // LDS stages: block j is read while j+1 and j+2 arrive (d = 256 without the software pipeline: two stages of
  // 29 KB, so that two workgroups fit a CU)
  constexpr int NST = (D == 256 && attn_occupancy<D, GM, PVF>() >= 2) ? 2 : 3;
  constexpr int PD = NST - 1;         // copies run this many blocks ahead
  constexpr int XC = 16 * DSR + 16;   // chunks of the small part: DSR rows of 64 Delta-S floats, then up to 64 key scales
  constexpr int STAGE = KCK + KC + XC;   // chunks per stage: K^, V^, small part
  __shared__ v4i lds[NST][STAGE];
  __shared__ __align__(16) float s_vs[2][D];   // delta_V and (smooth-V option) mean(V) of this KV head, for the epilogue

  // XCD-aware tile order: consecutive workgroup ids land on different XCDs (8 of them), so
  // give every XCD a contiguous range of tiles - tiles of one head then share one L2.
  // Under a causal mask a tile's work grows with its position, and workgroups start in index order.  There the
  // heads are taken in groups of 32 and a group's tiles are issued heaviest first ACROSS its heads (all their last
  // tiles, then all their last but one, ...), workgroup i taking the i-th tile of that list: every XCD then gets
  // every eighth tile of each weight - an equal share of the work whatever the head count - and, with 32 heads in a
  // group, the tiles of the same four heads.  Head by head the heavy tiles of an XCD's last head would start late
  // and finish long after the rest (13 % of the kernel's time at N = 8192, 1.5 % at N = 16384), and contiguous
  // ranges that do not hold whole heads (a head count that 8 does not divide) differ in work by up to a factor of
  // three.  More than four heads per XCD at a time no longer share its L2 once a head's codes exceed about 2 MB
  // (16 interleaved heads of 16384 keys ran 13 % slower than four; up to 4096 keys 16 are 4 % faster than four).
  // Sequences beyond 16384 tokens take groups of 8 heads - one head per XCD at a time, heaviest tile first: four
  // interleaved heads no longer share an XCD's L2 there (N = 32768: 1.5 % slower), and the equal shares still
  // count when 8 does not divide the head count (28 heads of 32768 tokens: +4.5 %).
  const int n_wg = SPLIT ? p.total_tiles * p.splits : p.total_tiles;
  const int per_xcd = (n_wg + 7) / 8;
  const int in_xcd = blockIdx.x / 8;
  int tile = (blockIdx.x % 8) * per_xcd + in_xcd;
  int split = 0;
  int bh, qb;
  if (!SPLIT && CAUSAL) {
    tile = blockIdx.x;
    if (tile >= n_wg) return;
    const int BH = p.total_tiles / p.nQb;
    const int GS = p.nQb <= 32 ? 128 : (p.nQb <= 128 ? 32 : 8);  // heads per group
    const int full = BH / GS;                                   // groups of GS heads; the last one may be smaller
    int grp = tile / (GS * p.nQb), g = GS;
    if (grp >= full) { grp = full; g = BH - full * GS; }
    const int within = tile - grp * GS * p.nQb;
    bh = grp * GS + within % g;
    qb = p.nQb - 1 - within / g;
  } else {
    if (tile >= n_wg) return;
    if constexpr (SPLIT) { split = tile % p.splits; tile /= p.splits; }
    bh = tile / p.nQb;
    qb = CAUSAL ? p.nQb - 1 - tile % p.nQb : tile % p.nQb;   // heavy tiles first
  }
  if (tile >= p.total_tiles) return;
  // PACK: tiles count (batch, KV head) pairs; bh is the first query head of the tile's group
  if constexpr (PACK) bh = (tile / p.Hkv) * p.H + (tile % p.Hkv) * (p.H / p.Hkv);
  const int b = bh / p.H, h = bh % p.H;
  const size_t bhkv = (size_t)b * p.Hkv + h / (p.H / p.Hkv);
  // this sequence's lengths (the launch's N, Nk unless the batch is a variable-length one; slab
  // strides below keep the block counts of the longest sequence)
  const Seq sq = seq_of(p.seq, (unsigned)b, p.N, p.Nk);
  if (qb * BQ >= sq.n) return;                 // a tile past the end of a shorter sequence

  const int t = threadIdx.x, lane = t & 63;
  if (sq.nk == 0) {                            // no keys at all: the rows are defined as zeros
    if (SPLIT && split != 0) return;           // (written once; the merge kernel leaves such a tile alone)
    for (int g = 0; g < (PACK ? p.H / p.Hkv : 1); ++g) {        // (PACK: the tile's rows belong to the whole group)
      unsigned short* o = reinterpret_cast<unsigned short*>(p.out) + head_offset(p.om, (unsigned)(bh + g));
      for (int idx = t; idx < BQ * (D / 8); idx += 256) {
        const int row = qb * BQ + idx / (D / 8);
        if (row < sq.n)
          *reinterpret_cast<uint4*>(o + row_offset(p.om, 0, (int)sq.q0 + row) + (idx % (D / 8)) * 8) =
              make_uint4(0u, 0u, 0u, 0u);
      }
      if (p.lse && t < BQ && qb * BQ + t < sq.n) p.lse[lse_index(p, sq, b, h + g, qb * BQ + t)] = -INFINITY;
    }
    return;
  }
  const int w = __builtin_amdgcn_readfirstlane(t >> 6);
  const int n = lane & 31, half = lane >> 5;
  // PACK: column w * 32 + n of the tile is query qi of head bh + hq; columns past the group's G N queries work on
  // query 0 of the first head and write nothing
  int hq = 0, qi = 0;
  bool col_ok = true;
  if constexpr (PACK) {
    const int col = w * WQ + n;
    col_ok = col < (p.H / p.Hkv) * sq.n;      // (sq.n >= 1 here)
    hq = col_ok ? col / sq.n : 0;
    qi = col_ok ? col - hq * sq.n : 0;
  }
  const int q_lo = PACK ? 0 : qb * BQ + w * WQ;          // first query of this wavefront
  const int q_hi = PACK ? sq.n - 1 : q_lo + WQ - 1;      // ... and the last
  const int query = PACK ? qi : q_lo + n;
  const size_t bhq = (size_t)bh + hq;                    // this lane's query head

  const v4i* gk = reinterpret_cast<const v4i*>(p.k_codes + bhkv * (size_t)p.nKb * k_block_bytes(D, INT4));
  const v4i* gv = reinterpret_cast<const v4i*>(p.v_codes + bhkv * (size_t)p.nKb * BKV * D);
  const float* gd = INT4 ? p.delta_s + ((size_t)bh * p.nQb + qb) * p.nKb * BKV : nullptr;
  const float* gs = p.k_scale + bhkv * (size_t)p.nKb * KSC;

  int nblk = (sq.nk + BKV - 1) / BKV;
  if (CAUSAL) nblk = min(nblk, (qb * BQ + BQ - 1 + sq.coff) / BKV + 1);
  int j_begin = 0;                             // this workgroup's key blocks: [j_begin, nblk)
  if constexpr (SPLIT) {
    const int n_vis = CAUSAL ? min(nblk, (qb * BQ + sq.coff) / BKV + 1) : nblk;
    const KeyChunk kc = key_chunk(split, p.splits, nblk, n_vis);
    j_begin = kc.j0;
    nblk = kc.j1;
    if (j_begin >= nblk) {                     // an empty chunk: offset -inf, sum 0 (the merge skips it)
      if (t < BQ) {
        float* el = p.part_el + ((size_t)((PACK ? tile : bh * p.nQb + qb) * p.splits + split) * BQ + t) * 2;
        el[0] = -INFINITY; el[1] = 0.0f;
      }
      return;
    }
  }

  // Block copies: every wavefront moves its quarter of the K^ and V^ chunks (the copy is the
  // identity on chunk indices), wavefront 0 the block's Delta-S row, wavefront 1 the 4 scales.
  const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)&lds[0][0];
  auto issue = [&](int j, int st) {
    const unsigned sb = lds0 + (unsigned)st * (STAGE * 16);
#pragma unroll
    for (int i = 0; i < CPTK; ++i) {
      if (i * 256 + 64 * w < KCK)
        dma_b128(gk + (size_t)j * KCK + i * 256, (unsigned)t * 16, sb + (unsigned)(i * 256 + 64 * w) * 16);
    }
#pragma unroll
    for (int i = 0; i < CPT; ++i)
      dma_b128(gv + (size_t)j * KC + i * 256, (unsigned)t * 16, sb + (unsigned)(KCK + i * 256 + 64 * w) * 16);
    if (w == 0) {
      if constexpr (INT4) {
        if constexpr (PACK) {          // one Delta-S row per query head of the group (consecutive heads, one row each)
          const int G = p.H / p.Hkv;
          for (int g = 0; g < G; ++g)
            dma_b32(gd + (size_t)g * p.nKb * BKV + (size_t)j * BKV, (unsigned)lane * 4, sb + (KCK + KC) * 16 + 256u * g);
        } else {
          dma_b32(gd + (size_t)j * BKV, (unsigned)lane * 4, sb + (KCK + KC) * 16);
        }
      }
    } else if (w == 1) {
      if (lane < KSC) dma_b32(gs + (size_t)j * KSC, (unsigned)lane * 4, sb + (KCK + KC) * 16 + 256 * DSR);
    }
  };
  // Every wavefront issues at least MINC copies per block, in block order, and loads complete in
  // order: "at most MINC outstanding" therefore means every block but the newest has landed.
  auto wait_all_but_newest = [&]() {
    static_assert(MINC >= 1 && MINC <= 8, "copy count per block");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"(MINC) : "memory");
  };
  auto wait_all = [&]() { asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory"); };

  // Without a causal mask the copies of the first two blocks go out before anything else of the tile is
  // requested, so that their round trip and that of the Q^ loads below overlap (1.2 % on N = 4096; copies
  // older than the compiler's own loads are harmless to its wait counts: loads complete in order, so
  // "at most n outstanding" still covers the load it means).  Under a causal mask, where many tiles are
  // short, the same order measured 1 % slower at N = 8192 and 16384, so there the copies follow the loads.
  constexpr bool COPIES_FIRST = !CAUSAL;
  // The epilogue's per-channel constants travel to LDS now (wavefronts 2 and 3, one copy per 64 channels):
  // read from global memory at the end of the tile, their round trip was idle time of the workgroup's share
  // of the CU.  These copies are older than every block copy, so the wait counts below still hold.
  {
    const unsigned vs0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)&s_vs[0][0];
    if (w == 2) {
#pragma unroll
      for (int i = 0; i < D / 64; ++i) dma_b32(p.v_scale + bhkv * D + 64 * i, (unsigned)lane * 4, vs0 + 256u * i);
    } else if (w == 3 && p.v_mean) {
#pragma unroll
      for (int i = 0; i < D / 64; ++i) dma_b32(p.v_mean + bhkv * D + 64 * i, (unsigned)lane * 4, vs0 + 4u * D + 256u * i);
    }
  }
  if constexpr (COPIES_FIRST) {
    issue(j_begin, 0);
    if (PD > 1 && j_begin + 1 < nblk) issue(j_begin + 1, 1);
  }

  // ---- this wavefront's Q^ operands (registers, for the whole kernel) and scale ----
  typedef typename QkOperand<INT4>::type qk_op;
  constexpr int NP = qk_pieces<D, INT4>();
  qk_op qreg[NP];
  {
    // (PACK: the lane's query sits in 32-query slice qi / 32 of its own head's slab, at lane position qi % 32)
    const int slice = PACK ? qi / WQ : w;
    const int pos = PACK ? (qi % WQ) + 32 * half : lane;
    const v4i* gq = reinterpret_cast<const v4i*>(p.q_codes + (bhq * p.nQb + qb) * q_slab_bytes(D, INT4)) +
                    (size_t)slice * (q_slab_bytes(D, INT4) / 16 / (BQ / WQ));
#pragma unroll
    for (int s = 0; s < NP; ++s) qreg[s] = load_qk_operand<INT4>(gq, s, pos);
  }
  const int row_in_block = PACK ? qi : w * WQ + n;       // the query's place in its smoothing block
  const float dq = p.q_scale[(bhq * p.nQb + qb) * (BQ / QG) + row_in_block / QG];
  // the row constant of the log-sum-exp output, fetched now so that the epilogue does not wait for it
  float lse_corr = 0.0f;
  if (p.lse) lse_corr = p.q_corr[(bhq * p.nQb + qb) * BQ + row_in_block];

  RowState<D> st;
#pragma unroll
  for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
    for (int v = 0; v < 16; ++v) st.O[ct][v] = 0.0f;
  }
  st.m_run = -INFINITY;
  st.l_run = 0.0f;

  // The wavefront walks all nblk blocks of the workgroup (copies and barriers are shared):
  // blocks [0, n_act) hold keys visible to some of its queries, of which [0, n_plain) need no
  // mask; past n_act (causal only) it just helps with the copies.
  int n_plain = min(nblk, sq.nk / BKV);                        // blocks without padded keys
  int n_act = nblk;                                            // blocks with any visible key
  if (CAUSAL) {
    n_plain = min(n_plain, (q_lo + sq.coff + 1) / BKV);        // key0 + 63 <= q_lo + coff
    n_act = min(nblk, (q_hi + sq.coff) / BKV + 1);             // key0 <= q_hi + coff
  }
  if constexpr (PACK) {
    // a wavefront whose 32 columns all lie past the group's queries only keeps up the copies and the barriers
    if (w * WQ >= (p.H / p.Hkv) * sq.n) n_plain = n_act = j_begin;
  }
  n_plain = __builtin_amdgcn_readfirstlane(n_plain);
  n_act = __builtin_amdgcn_readfirstlane(n_act);

  // Keys from here on are masked like the padding past the sequence's end.  For a chunk of a split key range that
  // is the chunk's end: the pipeline always forms the scores of one block past the last (from a stale stage), and
  // its running-max update must see them masked, or the exponent offset handed to the merge would not be the one
  // the sums were taken under.
  const int n_keys_end = SPLIT ? min(sq.nk, nblk * BKV) : sq.nk;

  // Software pipeline, one barrier per block, three LDS stages; every MFMA is issued between
  // pieces of vector work that do not depend on it, one at a time (a burst of MFMAs would hold up
  // the wavefront's own vector instructions behind it).  On entry to iteration j the dequantized
  // scores of block j (`sc`), their alpha and exponent offset are in registers, stage j%3 holds
  // block j and the copy of block j+1 is in flight.  The iteration
  //   B. waits for its own share of block j+1 and meets the other wavefronts at the barrier:
  //      block j+1 is visible, and nobody reads block j-1's stage any more,
  //   C. starts the LDS reads of K^_{j+1} and the copy of block j+2 into block j-1's stage,
  //   R. rescales O if a running max moved (covers the latency of C's reads),
  //   X. exponentials, row sum and FP8 codes of block j, four keys at a time, with one score MFMA
  //      of block j+1 issued in front of each piece; half way, the LDS reads of V^_j, of block j+1's scales
  //      and of the first key tile's half of its Delta-S row are started - the latter straight into the score
  //      registers that half of the exponentials has just finished with; the other half follows at the end,
  //   Y. the P~V MFMAs of block j, each followed by a piece of block j+1's dequantization, then
  //      block j+1's running-max update.
  // Past the wavefront's last block C, X and Y work on a stale stage (in bounds, results unused):
  // unconditional, so that no register stays live for the sake of a path not taken.
  qk_op ka[2 * NP];
  v4i va[2 * CT];
  KeyScales<GM> ks;
  v16i raw[2], sc[2];                 // raw scores being produced / dequantized scores of block j
  auto read_k = [&](int stg) {
    read_k_block<D, INT4>(&lds[stg][0], lane, ka);
  };
  auto read_v = [&](int stg) {
#pragma unroll
    for (int i = 0; i < 2 * CT; ++i) va[i] = lds[stg][KCK + i * 64 + lane];
  };
  // With a scale per key in the 8-bit mode the block's 32 factors stay live through the exponentials (they are
  // fused into the exponent's argument), so the next block's 32 key scales are fetched after them, not half way.
  constexpr bool LATE_SCALES = GM == 2 && !INT4;
  // Delta-S of key tile kt of the block in stage stg, into the registers the tile's scores will be formed in
  // (they are free once the previous block's exponentials of that tile are done)
  auto read_ds = [&](int stg, int kt) {
    if constexpr (INT4) {
      const v4f* dsv = reinterpret_cast<const v4f*>(reinterpret_cast<const float*>(&lds[stg][KCK + KC]) + 64 * hq + 32 * kt + 16 * half);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const v4f t4 = dsv[g];
#pragma unroll
        for (int r = 0; r < 4; ++r) sc[kt][4 * g + r] = __float_as_int(t4[r]);
      }
    }
  };
  auto read_scales = [&](int stg) {
    const float* lx = reinterpret_cast<const float*>(&lds[stg][KCK + KC]) + 64 * (DSR - 1);
    if constexpr (GM == 0) {
      ks.s[0] = lx[64 + half];
      ks.s[1] = lx[66 + half];
    } else if constexpr (GM == 1) {
      ks.s[0] = *reinterpret_cast<const v4f*>(lx + 64 + 4 * half);
      ks.s[1] = *reinterpret_cast<const v4f*>(lx + 72 + 4 * half);
    } else {
#pragma unroll
      for (int kt = 0; kt < 2; ++kt) {
        const v4f* kv = reinterpret_cast<const v4f*>(lx + 64 + 32 * kt + 16 * half);
#pragma unroll
        for (int g = 0; g < 4; ++g) ks.s[kt][g] = kv[g];
      }
    }
  };
  // The compiler does not see the copies, and it would otherwise leave its waits for the ordinary
  // loads of Q^ and the scale inside the loop, where they would also wait for the copies then in
  // flight: use those registers here so that the loads are complete before the loop.
#pragma unroll
  for (int s = 0; s < NP; ++s) {
#pragma unroll
    for (int i = 0; i < (int)(sizeof(qk_op) / 4); ++i) use_now(qreg[s][i]);
  }
  use_now(dq);
  use_now(lse_corr);
  if constexpr (COPIES_FIRST) {
    if constexpr (!OCC3) wait_all();
  } else {
    issue(j_begin, 0);
    if (PD > 1 && j_begin + 1 < nblk) { issue(j_begin + 1, 1); if constexpr (!OCC3) wait_all_but_newest(); } else { if constexpr (!OCC3) wait_all(); }
  }
  float alpha, m_sub = -INFINITY;     // of block j (m_sub: nothing summed yet)
  Factors<GM> fj;                     // block j's dequantization factors (used again by the fused exponent)
  constexpr int NQK = qk_steps<D, INT4>();
  constexpr int QPX = NQK > 8 ? 2 : 1;   // score MFMAs issued in front of each of the 8 pieces of the exponentials
  static_assert(NQK <= 16, "score MFMAs per block");
  constexpr int GPC = CT >= 8 ? 1 : 8 / CT;   // dequantization groups per P~V MFMA

#define SAGE_DEQ(MASKED_, GI_, KEY0_)                                                                \
  dequant_group<INT4, CAUSAL, MASKED_, GM, (GI_) / 4, (GI_) % 4>(raw, sc, fn, half, KEY0_,               \
                                                                 query + sq.coff, n_keys_end)
#define SAGE_DEQ_ALL(MASKED_, KEY0_)                                                                 \
  do {                                                                                               \
    SAGE_DEQ(MASKED_, 0, KEY0_); SAGE_DEQ(MASKED_, 1, KEY0_); SAGE_DEQ(MASKED_, 2, KEY0_);           \
    SAGE_DEQ(MASKED_, 3, KEY0_); SAGE_DEQ(MASKED_, 4, KEY0_); SAGE_DEQ(MASKED_, 5, KEY0_);           \
    SAGE_DEQ(MASKED_, 6, KEY0_); SAGE_DEQ(MASKED_, 7, KEY0_);                                        \
  } while (0)
  if constexpr (!OCC3) {
    __syncthreads();
    read_k(0);
    read_ds(0, 0);
    read_ds(0, 1);
    read_scales(0);
    qk_tile<D, INT4>(ka, qreg, raw);    // the first block holds a visible key for every query
    Factors<GM> fn;
    fn.set(dq, p.kappa, ks);
    if (j_begin < n_plain) SAGE_DEQ_ALL(false, j_begin * BKV); else SAGE_DEQ_ALL(true, j_begin * BKV);
    alpha = update_max<D, INT4, GM, PVF>(st, sc, fn, m_sub);
    fj = fn;
  }

  int cur = 0;   // stage of block j
#define SAGE_X(GI_, MASKED_)                                                                         \
  do {                                                                                               \
    if constexpr (QPX == 2) {                                                                        \
      qk_step<D, INT4, 2 * (GI_) < NQK ? 2 * (GI_) : 0>(ka, qreg, raw);                               \
      qk_step<D, INT4, 2 * (GI_) + 1 < NQK ? 2 * (GI_) + 1 : 0>(ka, qreg, raw);                       \
    } else if constexpr ((GI_) < NQK) {                                                              \
      qk_step<D, INT4, (GI_) < NQK ? (GI_) : 0>(ka, qreg, raw);                                      \
    }                                                                                                \
    exp_group<INT4, MASKED_, GM, PVF, (GI_) / 4, (GI_) % 4>(sc, fj, m_sub, pb, ls);                  \
    __builtin_amdgcn_sched_barrier(0);                                                               \
  } while (0)
#define SAGE_Y(CT_, MASKED_)                                                                         \
  do {                                                                                               \
    if constexpr ((CT_) < CT) {                                                                      \
      pv_step<D, (CT_) < CT ? (CT_) : 0, PVF>(st, va, pb);                                           \
      SAGE_DEQ(MASKED_, ((CT_) * GPC) % 8, (j + 1) * BKV);                                           \
      if constexpr (GPC >= 2) SAGE_DEQ(MASKED_, ((CT_) * GPC + 1) % 8, (j + 1) * BKV);               \
      if constexpr (GPC == 4) {                                                                      \
        SAGE_DEQ(MASKED_, ((CT_) * GPC + 2) % 8, (j + 1) * BKV);                                     \
        SAGE_DEQ(MASKED_, ((CT_) * GPC + 3) % 8, (j + 1) * BKV);                                     \
      }                                                                                              \
      __builtin_amdgcn_sched_barrier(0);                                                             \
    }                                                                                                \
  } while (0)
#define SAGE_BODY(MASKED_, MASKED_NEXT_)                                                                    \
  do {                                                                                               \
    const int nx1 = cur == NST - 1 ? 0 : cur + 1;                                                    \
    const int nx2 = nx1 == NST - 1 ? 0 : nx1 + 1;                                                    \
    wait_all();                                                                               /* B */ \
    __syncthreads();                                                                                 \
    read_k(nx1);                                                                              /* C */ \
    if (j + 2 < nblk) issue(j + 2, nx2);                                                             \
    block_rescale<D>(st, alpha);                                                              /* R */ \
    __builtin_amdgcn_sched_barrier(0);                                                               \
    v8i pb;                                                                                          \
    float ls = 0.0f;                                                                                 \
    SAGE_X(0, MASKED_); SAGE_X(1, MASKED_); SAGE_X(2, MASKED_); SAGE_X(3, MASKED_);           /* X */ \
    read_v(cur);                                                                                     \
    read_ds(nx1, 0);                                                                                 \
    if constexpr (!LATE_SCALES) read_scales(nx1);                                                    \
    __builtin_amdgcn_sched_barrier(0);                                                               \
    SAGE_X(4, MASKED_); SAGE_X(5, MASKED_); SAGE_X(6, MASKED_); SAGE_X(7, MASKED_);                  \
    read_ds(nx1, 1);                                                                                 \
    if constexpr (LATE_SCALES) read_scales(nx1);                                                     \
    st.l_run = __fmaf_rn(alpha, st.l_run, ls);                                                       \
    Factors<GM> fn;                                                                                  \
    fn.set(dq, p.kappa, ks);                                                                         \
    SAGE_Y(0, MASKED_NEXT_); SAGE_Y(1, MASKED_NEXT_); SAGE_Y(2, MASKED_NEXT_); SAGE_Y(3, MASKED_NEXT_); /* Y */ \
    SAGE_Y(4, MASKED_NEXT_); SAGE_Y(5, MASKED_NEXT_); SAGE_Y(6, MASKED_NEXT_); SAGE_Y(7, MASKED_NEXT_);         \
    alpha = update_max<D, INT4, GM, PVF>(st, sc, fn, m_sub);                                              \
    fj = fn;                                                                                         \
    cur = nx1;                                                                                       \
  } while (0)
  // Variant for three wavefronts per SIMD (168 registers): no software pipeline inside a wavefront - block j's score
  // product, softmax piece and P~V product run one after the other, and the two other wavefronts of the SIMD fill
  // the waits - so only one block's scores are live at a time.
#define SAGE_E3(GI_, MASKED_) exp_group<INT4, MASKED_, GM, PVF, (GI_) / 4, (GI_) % 4>(sc, fn, m_sub, pb, ls)
#define SAGE_P3(CT_) do { if constexpr ((CT_) < CT) pv_step<D, (CT_) < CT ? (CT_) : 0, PVF>(st, va, pb); } while (0)
#define SAGE_BODY3(MASKED_)                                                                          \
  do {                                                                                               \
    const int nx1 = cur == NST - 1 ? 0 : cur + 1;                                                    \
    const int nxp = PD == 1 ? nx1 : (nx1 == NST - 1 ? 0 : nx1 + 1);      /* stage of block j + PD */  \
    wait_all();                                                                                      \
    __syncthreads();                                                                                 \
    if (j + PD < nblk) issue(j + PD, nxp);                                                           \
    read_k(cur);                                                                                     \
    read_ds(cur, 0);                                                                                 \
    read_ds(cur, 1);                                                                                 \
    read_scales(cur);                                                                                \
    qk_tile<D, INT4>(ka, qreg, raw);                                                                 \
    Factors<GM> fn;                                                                                  \
    fn.set(dq, p.kappa, ks);                                                                         \
    SAGE_DEQ_ALL(MASKED_, j * BKV);                                                                  \
    alpha = update_max<D, INT4, GM, PVF>(st, sc, fn, m_sub);                                         \
    block_rescale<D>(st, alpha);                                                                     \
    v8i pb;                                                                                          \
    float ls = 0.0f;                                                                                 \
    SAGE_E3(0, MASKED_); SAGE_E3(1, MASKED_); SAGE_E3(2, MASKED_); SAGE_E3(3, MASKED_);              \
    read_v(cur);                                                                                     \
    SAGE_E3(4, MASKED_); SAGE_E3(5, MASKED_); SAGE_E3(6, MASKED_); SAGE_E3(7, MASKED_);              \
    st.l_run = __fmaf_rn(alpha, st.l_run, ls);                                                       \
    SAGE_P3(0); SAGE_P3(1); SAGE_P3(2); SAGE_P3(3); SAGE_P3(4); SAGE_P3(5); SAGE_P3(6); SAGE_P3(7);  \
    cur = nx1;                                                                                       \
  } while (0)
  int j = j_begin;
  if constexpr (OCC3) {
    for (; j < n_plain; ++j) SAGE_BODY3(false);
    for (; j < n_act; ++j) SAGE_BODY3(true);
  } else {
    for (; j + 1 < n_plain; ++j) SAGE_BODY(false, false);
    if (j < n_plain) { SAGE_BODY(false, true); ++j; }      // the last unmasked block, a masked (or no) successor
    for (; j < n_act; ++j) SAGE_BODY(true, true);
  }
  // causal only: blocks past this wavefront's last query - keep up the copies and the barriers
  for (; j < nblk; ++j) {
    const int nx1 = cur == NST - 1 ? 0 : cur + 1;
    const int nxp = PD == 1 ? nx1 : (nx1 == NST - 1 ? 0 : nx1 + 1);
    wait_all();
    __syncthreads();
    if (j + PD < nblk) issue(j + PD, nxp);
    cur = nx1;
  }
#undef SAGE_BODY3
#undef SAGE_P3
#undef SAGE_E3
#undef SAGE_BODY
#undef SAGE_Y
#undef SAGE_X
#undef SAGE_DEQ_ALL
#undef SAGE_DEQ

  // ---- epilogue (Algorithm 1 last line): O / l / 448 * delta_V (+ mean(V) with the smooth-V
  // option, Sec. 3.4 last paragraph); l_run already carries the 448
  float l_tot = st.l_run;
  {
    const unsigned u = __float_as_uint(l_tot);
    const auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    l_tot = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
  }
  if constexpr (SPLIT) {
    // a chunk of the keys: the sums stay under the chunk's own exponent offset and go to the merge kernel as they are
    const size_t prow = (size_t)((PACK ? tile : bh * p.nQb + qb) * p.splits + split) * BQ + w * WQ + n;
    if (PACK ? col_ok : query < sq.n) {
      if (half == 0) { p.part_el[prow * 2] = m_sub; p.part_el[prow * 2 + 1] = l_tot; }
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const v4f o4 = {st.O[ct][4 * g], st.O[ct][4 * g + 1], st.O[ct][4 * g + 2], st.O[ct][4 * g + 3]};
          *reinterpret_cast<v4f*>(p.part_o + prow * D + 32 * ct + 8 * g + 4 * half) = o4;
        }
      }
    }
    return;
  }
  if (p.lse && half == 0 && query < sq.n) {
    // ln sum_t exp(sm_scale <q, k_t>) = ln 2 * (e + log2(l) + the row constant smoothing K dropped): l_tot is the
    // sum of 2^(S - e) under the final exponent offset e = m_sub, which survived the pipeline's last update
    // (that one saw a fully masked, stale block and left the running max where it was)
    p.lse[lse_index(p, sq, b, h, query)] =
        LN2 * ((m_sub + __builtin_amdgcn_logf(l_tot)) + lse_corr);
  }
  // One correctly rounded reciprocal per row instead of a division per element (64 of them were 4 % of
  // a tile of 64 blocks): O * fl32(1/l) is within one unit of the last FP32 place of fl32(O / l), far
  // below the rounding to the 16-bit output type that follows.
  const float inv_l = __fdiv_rn(1.0f, l_tot);
  if (query < sq.n) {
    unsigned short* orow = reinterpret_cast<unsigned short*>(p.out) +
                           row_offset(p.om, head_offset(p.om, (unsigned)bh), (int)sq.q0 + query);
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int c0 = 32 * ct + 8 * g + 4 * half;
        const v4f sc = *reinterpret_cast<const v4f*>(&s_vs[0][c0]);
        v4f vm = {0.0f, 0.0f, 0.0f, 0.0f};
        if (p.v_mean) vm = *reinterpret_cast<const v4f*>(&s_vs[1][c0]);
        float o4[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          o4[r] = __fmul_rn(__fmul_rn(st.O[ct][4 * g + r], inv_l), sc[r]);
          if (p.v_mean) o4[r] = __fadd_rn(o4[r], vm[r]);
        }
        *reinterpret_cast<uint2*>(orow + c0) = make_uint2(pack16x2<BF16>(o4[0], o4[1]), pack16x2<BF16>(o4[2], o4[3]));
      }
    }
  }
}

// Merge of the partial results of a tile's key chunks (Eq. 1 applied to disjoint key sets): under the largest of
// the chunks' exponent offsets e* the sums add up with weights 2^(e_s - e*); then the epilogue of Algorithm 1.
// One workgroup per tile; a thread owns four channels of a row, d / 4 threads a row, and the workgroup walks the
// tile's rows 1024 / d at a time - so a tile with few valid rows (a decode step) still spreads over a whole row of
// threads, and a row's chunks are read as contiguous 4 d bytes.
// PACK: the tiles of k_attn_fwd's packed form - row r of a tile is query r % n of head r / n of the KV head's group
// (n: the sequence's query count).
template <int D, bool BF16, bool PACK = false>
__global__ void __launch_bounds__(256) k_merge_splits(const AttnParams p) {
  constexpr int TPR = D / 4, RP = 256 / TPR;      // threads per row, rows per pass
  const int tile = blockIdx.x;
  const int t = threadIdx.x, c_lo = 4 * (t % TPR);
  for (int r = t / TPR; r < BQ; r += RP) {
    int bh = tile / p.nQb, qb = tile % p.nQb, query = qb * BQ + r;
    if constexpr (PACK) bh = (tile / p.Hkv) * p.H + (tile % p.Hkv) * (p.H / p.Hkv);      // the group's first head
    const Seq sq = seq_of(p.seq, (unsigned)(bh / p.H), p.N, p.Nk);
    if constexpr (PACK) {
      if (sq.n <= 0 || r >= (p.H / p.Hkv) * sq.n) return;
      bh += r / sq.n;
      qb = 0;
      query = r % sq.n;
    }
    const int b = bh / p.H, h = bh % p.H;
    const size_t bhkv = (size_t)b * p.Hkv + h / (p.H / p.Hkv);
    if (sq.nk == 0 || query >= sq.n) return;     // (rows ascend; a sequence without keys was written by the attention kernel)
    const size_t row0 = (size_t)tile * p.splits * BQ + r;       // this row in chunk 0; chunk s is s * BQ rows further
    float e_max = -INFINITY;
    for (int s0 = 0; s0 < p.splits; s0 += 8) {
      float e[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) e[i] = p.part_el[(row0 + (size_t)min(s0 + i, p.splits - 1) * BQ) * 2];
#pragma unroll
      for (int i = 0; i < 8; ++i) e_max = fmaxf(e_max, e[i]);
    }
    float l = 0.0f;
    v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
    // eight chunks at a time, all their loads issued before the first use (one round trip per eight chunks, not one
    // per chunk); the chunks are summed in order
    for (int s0 = 0; s0 < p.splits; s0 += 8) {
      float e[8], lc[8];
      v4f o4[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const size_t row = row0 + (size_t)min(s0 + i, p.splits - 1) * BQ;
        e[i] = p.part_el[row * 2];
        lc[i] = p.part_el[row * 2 + 1];
        o4[i] = *reinterpret_cast<const v4f*>(p.part_o + row * D + c_lo);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (s0 + i >= p.splits || e[i] == -INFINITY) continue;     // (an empty chunk left its sums unwritten)
        const float wgt = __builtin_amdgcn_exp2f(e[i] - e_max);
        l = __fmaf_rn(wgt, lc[i], l);
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[k] = __fmaf_rn(wgt, o4[i][k], acc[k]);
      }
    }
    if (p.lse && c_lo == 0)
      p.lse[lse_index(p, sq, b, h, query)] =
          LN2 * ((e_max + __builtin_amdgcn_logf(l)) + p.q_corr[((size_t)bh * p.nQb + qb) * BQ + (query - qb * BQ)]);
    const float inv_l = __fdiv_rn(1.0f, l);
    unsigned short* orow = reinterpret_cast<unsigned short*>(p.out) +
                           row_offset(p.om, head_offset(p.om, (unsigned)bh), (int)sq.q0 + query) + c_lo;
    const v4f vs = *reinterpret_cast<const v4f*>(p.v_scale + bhkv * D + c_lo);
    float o4[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) o4[k] = __fmul_rn(__fmul_rn(acc[k], inv_l), vs[k]);
    if (p.v_mean) {
      const v4f vm = *reinterpret_cast<const v4f*>(p.v_mean + bhkv * D + c_lo);
#pragma unroll
      for (int k = 0; k < 4; ++k) o4[k] = __fadd_rn(o4[k], vm[k]);
    }
    *reinterpret_cast<uint2*>(orow) = make_uint2(pack16x2<BF16>(o4[0], o4[1]), pack16x2<BF16>(o4[2], o4[3]));
  }
}

// Integer score accumulators of one (128-query tile, 64-key block) through qk_tile.
template <int D, bool INT4>
__global__ void __launch_bounds__(256) k_debug_qk(const int8_t* __restrict__ q_codes,
                                                  const int8_t* __restrict__ k_codes, int q_tile,
                                                  int kv_block, int32_t* __restrict__ out) {
  constexpr int KCK = (int)(k_block_bytes(D, INT4) / 16);
  constexpr int NP = qk_pieces<D, INT4>();
  __shared__ v4i lds[KCK];
  const int t = threadIdx.x, lane = t & 63, w = t >> 6, n = lane & 31, half = lane >> 5;
  const v4i* gk = reinterpret_cast<const v4i*>(k_codes) + (size_t)kv_block * KCK;
  for (int i = t; i < KCK; i += 256) lds[i] = gk[i];
  __syncthreads();
  typename QkOperand<INT4>::type qreg[NP], ka[2 * NP];
  const v4i* gq = reinterpret_cast<const v4i*>(q_codes + (size_t)q_tile * q_slab_bytes(D, INT4)) +
                  (size_t)w * (q_slab_bytes(D, INT4) / 16 / (BQ / WQ));
#pragma unroll
  for (int s = 0; s < NP; ++s) qreg[s] = load_qk_operand<INT4>(gq, s, lane);
  // the block's operands come out of LDS through the attention kernel's own fetch code
  read_k_block<D, INT4>(&lds[0], lane, ka);
  v16i acc[2];
  qk_tile<D, INT4>(ka, qreg, acc);
#pragma unroll
  for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
    for (int v = 0; v < 16; ++v)
      out[(w * WQ + n) * BKV + 32 * kt + 16 * half + v] = INT4 ? (int)__int_as_float(acc[kt][v]) : acc[kt][v];
  }
}

// One P~V-type MFMA on caller-provided operands (hardware check of the accumulation path).
__global__ void __launch_bounds__(64) k_debug_mfma_fp8(const v8i* __restrict__ a, const v8i* __restrict__ b,
                                                       const v16f* __restrict__ c, v16f* __restrict__ d) {
  const int l = threadIdx.x;
  d[l] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[l], b[l], c[l], 0, 0, 0, 0, 0, 0);
}

hipError_t launch_debug_mfma_fp8(const void* a, const void* b, const float* c, float* d, hipStream_t s) {
  k_debug_mfma_fp8<<<1, 64, 0, s>>>((const v8i*)a, (const v8i*)b, (const v16f*)c, (v16f*)d);
  return hipGetLastError();
}

template <int D, bool INT4, bool CAUSAL, bool BF16, int GM, int PVF>
static hipError_t launch_attention_g(const Dims& Dm, const Ptrs& P, hipStream_t s) {
  AttnParams p;
  p.q_codes = P.q_codes; p.k_codes = P.k_codes; p.v_codes = P.v_codes;
  p.q_scale = P.q_scale; p.k_scale = P.k_scale; p.v_scale = P.v_scale; p.delta_s = P.delta_s;
  p.v_mean = Dm.smooth_v ? P.v_mean : nullptr;
  p.out = P.out;
  p.H = Dm.H; p.Hkv = Dm.Hkv; p.N = Dm.N; p.Nk = Dm.Nk; p.nQb = Dm.nQb;
  p.om = make_tensor_map(Dm.nhd, Dm.H, Dm.N, Dm.d, Dm.seq.cu_q != nullptr); p.nKb = Dm.nKb;
  p.seq = Dm.seq;
  p.lse = P.lse; p.q_corr = P.q_corr; p.B = Dm.B;
  p.total_tiles = Dm.B * Dm.H * Dm.nQb;
  p.kappa = Dm.kappa;
  p.splits = Dm.splits; p.part_o = P.part_o; p.part_el = P.part_el;
  if constexpr (GM == 0 && PVF == PV_E4M3) {        // (the key split comes with the default groups and data type)
    if (Dm.pack) {                                  // packed tiles: one per (batch, KV head), any number of chunks
      p.total_tiles = Dm.B * Dm.Hkv;
      const int grid = 8 * ((p.total_tiles * Dm.splits + 7) / 8);
      k_attn_fwd<D, INT4, CAUSAL, BF16, GM, PVF, true, true><<<grid, 256, 0, s>>>(p);
      k_merge_splits<D, BF16, true><<<p.total_tiles, 256, 0, s>>>(p);
      return hipGetLastError();
    }
    if (Dm.splits > 1) {
      const int grid = 8 * ((p.total_tiles * Dm.splits + 7) / 8);
      k_attn_fwd<D, INT4, CAUSAL, BF16, GM, PVF, true><<<grid, 256, 0, s>>>(p);
      k_merge_splits<D, BF16><<<p.total_tiles, 256, 0, s>>>(p);
      return hipGetLastError();
    }
  }
  const int grid = 8 * ((p.total_tiles + 7) / 8);
  k_attn_fwd<D, INT4, CAUSAL, BF16, GM, PVF><<<grid, 256, 0, s>>>(p);
  return hipGetLastError();
}
template <int D, bool INT4, bool CAUSAL, bool BF16>
static hipError_t launch_attention_t(const Dims& Dm, const Ptrs& P, hipStream_t s) {
  // the other data types of P~V come with the default key groups only
  if (Dm.pvf == PV_E5M2) return launch_attention_g<D, INT4, CAUSAL, BF16, 0, PV_E5M2>(Dm, P, s);
  if (Dm.pvf == PV_INT8) return launch_attention_g<D, INT4, CAUSAL, BF16, 0, PV_INT8>(Dm, P, s);
  if (Dm.kg == KGROUP) return launch_attention_g<D, INT4, CAUSAL, BF16, 0, PV_E4M3>(Dm, P, s);
  if (Dm.kg == 4) return launch_attention_g<D, INT4, CAUSAL, BF16, 1, PV_E4M3>(Dm, P, s);
  return launch_attention_g<D, INT4, CAUSAL, BF16, 2, PV_E4M3>(Dm, P, s);
}

hipError_t launch_attention(const Dims& D, const Ptrs& P, hipStream_t s) {
#define SAGE_ATT(DD, I4, CA, BF) return launch_attention_t<DD, I4, CA, BF>(D, P, s)
#define SAGE_ATT_BF(DD, I4, CA) do { if (D.bf16) SAGE_ATT(DD, I4, CA, true); else SAGE_ATT(DD, I4, CA, false); } while (0)
#define SAGE_ATT_CA(DD, I4) do { if (D.causal) SAGE_ATT_BF(DD, I4, true); else SAGE_ATT_BF(DD, I4, false); } while (0)
  if (D.d == 256)      { if (D.int4) SAGE_ATT_CA(256, true); else SAGE_ATT_CA(256, false); }
  else if (D.d == 128) { if (D.int4) SAGE_ATT_CA(128, true); else SAGE_ATT_CA(128, false); }
  else                 { if (D.int4) SAGE_ATT_CA(64, true); else SAGE_ATT_CA(64, false); }
#undef SAGE_ATT_CA
#undef SAGE_ATT_BF
#undef SAGE_ATT
}

hipError_t launch_debug_qk(const Dims& D, const Ptrs& P, int b, int h, int q_tile, int kv_block,
                           int32_t* out, hipStream_t s) {
  const size_t bh = (size_t)b * D.H + h;
  const size_t bhkv = (size_t)b * D.Hkv + h / (D.H / D.Hkv);
  const int8_t* qc = P.q_codes + bh * (size_t)D.nQb * q_slab_bytes(D.d, D.int4);
  const int8_t* kc = P.k_codes + bhkv * (size_t)D.nKb * k_block_bytes(D.d, D.int4);
  if (D.d == 256) {
    if (D.int4) k_debug_qk<256, true><<<1, 256, 0, s>>>(qc, kc, q_tile, kv_block, out);
    else k_debug_qk<256, false><<<1, 256, 0, s>>>(qc, kc, q_tile, kv_block, out);
  } else if (D.d == 128) {
    if (D.int4) k_debug_qk<128, true><<<1, 256, 0, s>>>(qc, kc, q_tile, kv_block, out);
    else k_debug_qk<128, false><<<1, 256, 0, s>>>(qc, kc, q_tile, kv_block, out);
  } else {
    if (D.int4) k_debug_qk<64, true><<<1, 256, 0, s>>>(qc, kc, q_tile, kv_block, out);
    else k_debug_qk<64, false><<<1, 256, 0, s>>>(qc, kc, q_tile, kv_block, out);
  }
  return hipGetLastError();
}

}  // namespace sage
