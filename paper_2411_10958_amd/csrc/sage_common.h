// Internal definitions shared by the HIP sources of libsageattn: problem dimensions, the
// workspace map and the packed ("MFMA fragment order") layouts the preprocessing kernels
// write and the attention kernel reads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace sage {

constexpr int BQ = 128;      // queries per workgroup tile = Q smoothing block (Algorithm 1, b_q)
constexpr int BKV = 64;      // keys per block = level-1 accumulation block (b_kv)
constexpr int WQ = 32;       // queries per wavefront (one 32x32 MFMA column tile)
constexpr int QGROUP = 2;    // queries per quantization group (default group map)
constexpr int KGROUP = 16;   // keys per quantization group (default group map)
constexpr int PACK_G = 8;    // query heads per KV head that may share one attention tile (Delta-S rows per LDS stage)
constexpr float E4M3_MAX = 448.0f;
constexpr int MAX_TOKENS = 1 << 24;   // per sequence; keeps token and tile arithmetic inside 32-bit integers
constexpr int STAT_ROWS = 256;  // tokens per workgroup of the column-statistics pass
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LOG2_448 = 8.807354922057604f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float E5M2_MAX = 57344.0f;       // the E5M2 variant of the FP8 stage
constexpr float LOG2_57344 = 15.807354922057604f;
constexpr float INT8_PV_MAX = 127.0f;      // the INT8 variant of the P~V stage
constexpr float LOG2_127 = 6.988684686772166f;
enum { PV_E4M3 = 0, PV_E5M2 = 1, PV_INT8 = 2 };

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

// Where row n of head (b, h) of a user tensor starts, in elements: b * sb + h * sh + n * sn.
struct TensorMap {
  long long sb, sh, sn;
  int heads;
};
// element offset of head bh = b * heads + h (taken once per kernel: it holds the only division),
// and of token n within it
__host__ __device__ inline size_t head_offset(const TensorMap& m, unsigned bh) {
  const unsigned b = bh / (unsigned)m.heads, h = bh - b * (unsigned)m.heads;
  return b * (size_t)m.sb + h * (size_t)m.sh;
}

// Variable-length batches: prefix sums of the sequence lengths (device pointers; both null for a
// fixed-length batch).  seq_of() gives sequence b's lengths, cut to the launch's maxima so that no
// index derived from them can leave the workspace slabs, its first tokens, and the causal offset
// (never negative: a sequence with fewer keys than queries is masked from the first query and key).
struct SeqMap { const int* cu_q; const int* cu_k; };
struct Seq { int n, nk, coff; size_t q0, k0; };
__device__ inline Seq seq_of(const SeqMap& sm, unsigned b, int N, int Nk) {
  Seq s;
  s.n = N; s.nk = Nk; s.q0 = 0; s.k0 = 0;
  if (sm.cu_q) {
    const int* ck = sm.cu_k ? sm.cu_k : sm.cu_q;
    const int q0 = sm.cu_q[b], q1 = sm.cu_q[b + 1], k0 = ck[b], k1 = ck[b + 1];
    s.n = min(max(q1 - q0, 0), N);
    s.nk = min(max(k1 - k0, 0), Nk);
    s.q0 = (size_t)max(q0, 0);
    s.k0 = (size_t)max(k0, 0);
  }
  s.coff = max(s.nk - s.n, 0);
  return s;
}
struct HeadPos { unsigned b; size_t base; };   // batch index and element offset of a head
__host__ __device__ inline HeadPos head_pos(const TensorMap& m, unsigned bh) {
  HeadPos p;
  p.b = bh / (unsigned)m.heads;
  p.base = p.b * (size_t)m.sb + (bh - p.b * (unsigned)m.heads) * (size_t)m.sh;
  return p;
}
__host__ __device__ inline size_t row_offset(const TensorMap& m, size_t head_base, int n) {
  return head_base + (size_t)n * (size_t)m.sn;
}
inline TensorMap make_tensor_map(int nhd, int heads, int tokens, int d, bool varlen = false) {
  TensorMap m;
  m.heads = heads;
  if (varlen) { m.sb = 0; m.sh = d; m.sn = (long long)heads * d; return m; }   // packed [tokens, heads, d]
  if (nhd) { m.sb = (long long)tokens * heads * d; m.sh = d; m.sn = (long long)heads * d; }
  else     { m.sb = (long long)heads * tokens * d; m.sh = (long long)tokens * d; m.sn = d; }
  return m;
}

struct Dims {
  int B, H, Hkv, N, d;
  int Nk;      // keys / values per head (N unless the caller says otherwise)
  int nQb;     // ceil(N / 128) query blocks
  int nKb;     // ceil(Nk / 64) key blocks
  int causal, int4, bf16, smooth_v, block_groups, nhd;
  int smooth_k, smooth_q;   // 0: that mean is taken as zero (the paper's smoothing ablation)
  int ds32;                 // Delta-S accumulated in FP32 instead of FP64 (faster, approximate)
  int ds_mode;              // how Delta-S is formed: 0 digit products on the INT8 matrix unit, 1 FP32, 2 FP64 matrix instructions
  int stats_given;          // mean(K) and delta_V come from the caller: no statistics pass
  int qg, kg;  // queries / keys per stored scale: 2 / 16 (lane and block maps), 1 / 4 (fine), 1 / 1 (token)
  float kappa; // fl32(sm_scale * log2 e)
  SeqMap seq;  // variable-length batch: N, Nk, nQb, nKb then describe the longest sequence
  int want_lse; // the caller asked for the row log-sum-exp
  int pvf;      // data type of P~ and V: PV_E4M3, PV_E5M2 or PV_INT8
  int tensor_groups;  // one scale per (batch, head) tensor of Q and of K (implies block_groups)
  int splits;         // workgroups per query tile in the attention kernel (key range split; 1 = none)
  int pack;           // the query heads of a KV head share one tile (short queries, grouped KV heads; with the split path)
};

// Workspace map (all offsets multiples of 256 bytes).
//
// Packed layouts (one "chunk" = 16 bytes = one lane's operand piece, 64 chunks = one
// wavefront-wide ds_read_b128 / global load):
//  INT8 mode (two's-complement bytes):
//   q_codes: [B*H][N_q32 tiles of 32 queries][d/32 k-steps][64 lanes] chunks.  Lane l of
//            k-step s holds query 32*tile + l%32, channels 32*s + 16*(l/32) + 0..15
//            (the B operand of v_mfma_i32_32x32x32_i8).
//   k_codes: [B*Hkv][nKb blocks][d/32 k-steps][2 key tiles][64 lanes] chunks.  Lane l holds
//            MFMA row rho = l%32 and channels 32*s + 16*(l/32) + 0..15, where row
//            rho = 8g + 4h + r carries key 32*tile + 16h + 4g + r of the block, so that an
//            accumulator lane (half h) ends up with 16 consecutive keys.
//  INT4 mode (6-bit FP6 E2M3 codes of the same integers, see the FP6 note below): one
//  operand of v_mfma_f32_32x32x64_f8f6f4 ("op") covers 32 rows x 64 channels; lane l supplies row
//  l%32 and channels 32*(l/32) + e, element e at bit 6e of a 24-byte payload.  An op is stored
//  as 1536 bytes: a plane of 64 x 16 bytes (payload bytes 0..15 of lanes 0..63) followed by a
//  plane of 64 x 8 bytes (payload bytes 16..23), so that one ds_read_b128 and one ds_read_b64
//  per lane fetch it without bank conflicts.
//   q_codes: [B*H][N_q32 tiles][d/64 ops] x 1536 bytes (row = query 32*tile + l%32).
//   k_codes: [B*Hkv][nKb blocks][d/64 ops][2 key tiles] x 1536 bytes (row rho as above).
//   v_codes: [B*Hkv][nKb blocks][d/32 channel tiles][2 parts][64 lanes] chunks.  Lane l holds
//            channel 32*ct + l%32 and the 16 keys 32*part + 16*(l/32) + 0..15 of the block
//            (the A operand of v_mfma_f32_32x32x64_f8f6f4, key order matching the order in
//            which a lane's P~ registers come out of the score tiles).
//   delta_s: [B*H][nQb][nKb*64] float, zero beyond N.
//   q_scale: [B*H][nQb*128/qg] float;  k_scale: [B*Hkv][nKb*64/kg] float (qg, kg: queries / keys per
//            scale of the chosen group map).
//   k_sum, v_max (and v_sum): [B*Hkv][ceil(Nk/STAT_ROWS)][d] partial results of the statistics pass;
//   v_sum, v_mean only with the smooth-V option (otherwise zero-sized).
struct Workspace {
  size_t k_sum, v_sum, v_max, k_mean, v_mean, v_scale, q_mean, q_scale, k_scale, q_corr, q_head_scale,
      k_head_scale, q_codes, k_codes, v_codes, delta_s, part_o, part_el, q_digits, q_dscale, total;
};

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

constexpr int OP6_BYTES = 1536;   // one FP6 MFMA operand (32 rows x 64 channels x 6 bits)
// bytes of the packed codes of one 128-query slab / one 64-key block
__host__ __device__ constexpr size_t q_slab_bytes(int d, bool int4) {
  return int4 ? (size_t)(BQ / 32) * (d / 64) * OP6_BYTES : (size_t)BQ * d;
}
__host__ __device__ constexpr size_t k_block_bytes(int d, bool int4) {
  return int4 ? (size_t)(d / 64) * 2 * OP6_BYTES : (size_t)BKV * d;
}

inline Workspace make_workspace(const Dims& D) {
  Workspace w;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
  const size_t BH = (size_t)D.B * D.H, BHkv = (size_t)D.B * D.Hkv;
  const size_t nchunk = (size_t)(D.Nk + STAT_ROWS - 1) / STAT_ROWS;   // partial results of the statistics pass
  w.k_sum = take(BHkv * nchunk * D.d * sizeof(double));
  w.v_sum = take(D.smooth_v ? BHkv * nchunk * D.d * sizeof(double) : 0);
  w.v_max = take(BHkv * nchunk * D.d * sizeof(unsigned));
  w.k_mean = take(BHkv * D.d * sizeof(float));
  w.v_mean = take(D.smooth_v ? BHkv * D.d * sizeof(float) : 0);
  w.v_scale = take(BHkv * D.d * sizeof(float));
  w.q_mean = take(BH * D.nQb * D.d * sizeof(float));
  w.q_scale = take(BH * D.nQb * (BQ / D.qg) * sizeof(float));
  w.k_scale = take(BHkv * D.nKb * (BKV / D.kg) * sizeof(float));
  w.q_corr = take(BH * D.nQb * BQ * sizeof(float));      // kappa * <q_r, mean(K)> per query (log-sum-exp output)
  w.q_head_scale = take(BH * sizeof(float));             // per-tensor granularity only
  w.k_head_scale = take(BHkv * sizeof(float));
  w.q_codes = take(BH * D.nQb * q_slab_bytes(D.d, D.int4));
  w.k_codes = take(BHkv * D.nKb * k_block_bytes(D.d, D.int4));
  w.v_codes = take(BHkv * D.nKb * BKV * D.d);
  w.delta_s = take(D.int4 ? BH * D.nQb * D.nKb * BKV * sizeof(float) : 0);
  // partial results of a split key range: per (tile, chunk) 128 rows of d floats, and (offset, sum) per row
  // digits of the block means for the Delta-S product: 6 planes of d bytes per (head, query block), and 2^E per row
  w.q_digits = take(D.int4 ? BH * D.nQb * 6 * D.d : 0);
  w.q_dscale = take(D.int4 ? BH * D.nQb * sizeof(float) : 0);
  const size_t split_tiles = D.pack ? (size_t)D.B * D.Hkv : (D.splits > 1 ? BH * D.nQb : 0);
  w.part_o = take(split_tiles * D.splits * BQ * D.d * sizeof(float));
  w.part_el = take(split_tiles * D.splits * BQ * 2 * sizeof(float));
  w.total = off;
  return w;
}

struct Ptrs {
  const void *q, *k, *v;
  void* out;
  double *k_sum, *v_sum;
  unsigned* v_max;
  float *k_mean, *v_mean, *v_scale, *q_mean, *q_scale, *k_scale, *q_corr, *q_head_scale, *k_head_scale, *delta_s;
  float *part_o, *part_el;
  float* lse;
  int8_t *q_codes, *k_codes;
  uint8_t* v_codes;
  unsigned char* q_digits;   // digits of the block means (Delta-S by digit products)
  float* q_dscale;
};

inline Ptrs make_ptrs(const void* q, const void* k, const void* v, void* out, void* ws,
                      const Workspace& w) {
  char* b = (char*)ws;
  Ptrs p;
  p.q = q; p.k = k; p.v = v; p.out = out;
  p.k_sum = (double*)(b + w.k_sum);
  p.v_sum = (double*)(b + w.v_sum);
  p.v_max = (unsigned*)(b + w.v_max);
  p.k_mean = (float*)(b + w.k_mean);
  p.v_mean = (float*)(b + w.v_mean);
  p.v_scale = (float*)(b + w.v_scale);
  p.q_mean = (float*)(b + w.q_mean);
  p.q_scale = (float*)(b + w.q_scale);
  p.k_scale = (float*)(b + w.k_scale);
  p.q_corr = (float*)(b + w.q_corr);
  p.q_head_scale = (float*)(b + w.q_head_scale);
  p.k_head_scale = (float*)(b + w.k_head_scale);
  p.lse = nullptr;
  p.q_codes = (int8_t*)(b + w.q_codes);
  p.k_codes = (int8_t*)(b + w.k_codes);
  p.v_codes = (uint8_t*)(b + w.v_codes);
  p.delta_s = (float*)(b + w.delta_s);
  p.part_o = (float*)(b + w.part_o);
  p.part_el = (float*)(b + w.part_el);
  p.q_digits = (unsigned char*)(b + w.q_digits);
  p.q_dscale = (float*)(b + w.q_dscale);
  return p;
}

// ---- packed-layout index helpers (byte offsets inside one (batch, head) slab) ----
// q_codes: query n (0..nQb*128), channel c
__host__ __device__ inline size_t q_code_off(int n, int c, int d) {
  const int tile = n >> 5, col = n & 31, s = c >> 5, half = (c >> 4) & 1, byte = c & 15;
  return ((size_t)(tile * (d >> 5) + s) * 64 + col + 32 * half) * 16 + byte;
}
// k_codes: key n, channel c
__host__ __device__ inline size_t k_code_off(int n, int c, int d) {
  const int blk = n >> 6, kt = (n >> 5) & 1, kk = n & 31;
  const int h = kk >> 4, g = (kk >> 2) & 3, r = kk & 3, rho = 8 * g + 4 * h + r;
  const int s = c >> 5, half = (c >> 4) & 1, byte = c & 15;
  return ((size_t)((blk * (d >> 5) + s) * 2 + kt) * 64 + rho + 32 * half) * 16 + byte;
}
// v_codes: key n, channel c
__host__ __device__ inline size_t v_code_off(int n, int c, int d) {
  const int blk = n >> 6, part = (n >> 5) & 1, h = (n >> 4) & 1, byte = n & 15;
  const int ct = c >> 5, ch = c & 31;
  return ((size_t)((blk * (d >> 5) + ct) * 2 + part) * 64 + ch + 32 * h) * 16 + byte;
}

// ---- INT4 codes travel as 6-bit FP6 E2M3 values ----
// gfx950 has no 4-bit integer MFMA, but every integer in [-7, 7] is an E2M3 value (sign, 2 exponent
// bits with bias 1, 3 mantissa bits: 1, 2, 3 = 1.5*2, 4, 5 = 1.25*4, 6 = 1.5*4, 7 = 1.75*4), products
// (<= 49) and their sums over d <= 128 channels (<= 6272) are exact in the FP32 accumulator of
// v_mfma_f32_32x32x64_f8f6f4, and the FP6 operand format runs at twice the rate of the 8-bit
// formats: the gfx950 counterpart of "INT4 matmul is twice as fast as INT8".  The accumulators come
// out as exact integers in float - no int->float conversion afterwards.
// (The quantizers produce the fields with the hardware FP32 -> FP6 conversion; the decoder below serves
// the copy-out of sage_attn_quant.)
__host__ __device__ inline int e2m3_to_int4_code(unsigned b) {
  const int e = (b >> 3) & 3, m = b & 7;
  const int a = e == 0 ? 0 : ((8 + m) << (e - 1)) >> 3;     // (1 + m/8) * 2^(e-1)
  return (b & 0x20) ? -a : a;
}
// byte b (0..23) of lane_m's payload inside an op (16-byte plane, then 8-byte plane)
__host__ __device__ inline int op6_byte(int lane_m, int b) {
  return b < 16 ? lane_m * 16 + b : 1024 + lane_m * 8 + (b - 16);
}
// op base (bytes inside one (batch, head) slab), MFMA lane and element index of query / key n, channel c
__host__ __device__ inline size_t q_op6(int n, int c, int d, int* lane_m, int* e) {
  *lane_m = (n & 31) + 32 * ((c >> 5) & 1);
  *e = c & 31;
  return (size_t)((n >> 5) * (d >> 6) + (c >> 6)) * OP6_BYTES;
}
__host__ __device__ inline size_t k_op6(int n, int c, int d, int* lane_m, int* e) {
  const int blk = n >> 6, kt = (n >> 5) & 1, kk = n & 31;
  const int rho = 8 * ((kk >> 2) & 3) + 4 * (kk >> 4) + (kk & 3);
  *lane_m = rho + 32 * ((c >> 5) & 1);
  *e = c & 31;
  return (size_t)((blk * (d >> 6) + (c >> 6)) * 2 + kt) * OP6_BYTES;
}

// ---- 16-bit input helpers ----
__device__ inline float bf16_to_f32(unsigned short u) { return __uint_as_float((unsigned)u << 16); }
__device__ inline float fp16_to_f32(unsigned short u) {
  return (float)__builtin_bit_cast(_Float16, u);
}
template <bool BF16> __device__ inline float load16(unsigned short u) {
  if constexpr (BF16) return bf16_to_f32(u); else return fp16_to_f32(u);
}
// two values rounded (nearest even) to the 16-bit type and packed, a in the low half: the hardware's
// packed conversions (v_cvt_pk_bf16_f32 on gfx950)
template <bool BF16> __device__ inline unsigned pack16x2(float a, float b) {
  typedef float v2f_ __attribute__((ext_vector_type(2)));
  const v2f_ x = {a, b};
  if constexpr (BF16) {
    typedef __bf16 v2b_ __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(unsigned, __builtin_convertvector(x, v2b_));
  } else {
    typedef _Float16 v2h_ __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(unsigned, __builtin_convertvector(x, v2h_));
  }
}

// launchers (defined in the .hip files)
hipError_t launch_prologue(const Dims& D, const Ptrs& P, hipStream_t s);
hipError_t launch_kv_stats(const Dims& D, const Ptrs& P, hipStream_t s);   // writes P.k_mean, P.v_scale
hipError_t launch_kv_stats_update(const Dims& D, const Ptrs& P, double* state_sum, float* state_max, int fresh,
                                  long long n_total, hipStream_t s);
hipError_t launch_attention(const Dims& D, const Ptrs& P, hipStream_t s);
hipError_t launch_unpack(const Dims& D, const Ptrs& P, const void* quant_out, hipStream_t s);
hipError_t launch_debug_mfma_fp8(const void* a, const void* b, const float* c, float* d, hipStream_t s);
hipError_t launch_debug_qk(const Dims& D, const Ptrs& P, int b, int h, int q_tile, int kv_block,
                           int32_t* out, hipStream_t s);

}  // namespace sage
