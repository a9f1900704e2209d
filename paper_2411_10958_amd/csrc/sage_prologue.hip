// Preprocessing kernels of the quantized attention forward pass (paper Sec. 3.1-3.3 and the
// "Preprocessing" line plus the first line of the outer loop of Algorithm 1): token means,
// smoothing, Delta-S, group quantization of Q and K, per-channel FP8 quantization of V.
// The passes stream Q, K and V once or twice each; after the loads it is the vector ALU work per
// element (and, for Delta-S, the FP64 matrix pipe) that sets their speed, so the quantizers avoid
// per-element divisions and per-element code packing.  Codes are written in the MFMA fragment
// order described in sage_common.h so that the attention kernel can move them with plain 16-byte
// copies.
#include "sage_common.h"
#include "sage_attn.h"

namespace sage {

// ------------------------------------------------------------------------------------------
// small helpers
// 16-byte load marked non-temporal: Q, K and V are streamed once per pass, and keeping them out of the
// way of the caches measured 25 % faster on the statistics pass
__device__ inline uint4 nt_load16(const unsigned short* p) {
  typedef unsigned v4u __attribute__((ext_vector_type(4)));
  const v4u r = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
  return make_uint4(r[0], r[1], r[2], r[3]);
}

template <bool BF16, bool NT = true>
__device__ inline void load8(const unsigned short* p, float (&x)[8]) {
  const uint4 raw = NT ? nt_load16(p) : *reinterpret_cast<const uint4*>(p);
  const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = load16<BF16>((unsigned short)(w[i] & 0xffffu));
    x[2 * i + 1] = load16<BF16>((unsigned short)(w[i] >> 16));
  }
}

template <bool BF16>
__device__ inline void unpack8(const uint4& raw, float* x) {
  const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = load16<BF16>((unsigned short)(w[i] & 0xffffu));
    x[2 * i + 1] = load16<BF16>((unsigned short)(w[i] >> 16));
  }
}

__device__ inline float wave_max(float v) {
#pragma unroll
  for (int m = 32; m >= 1; m >>= 1) v = fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}

// psi of Sec. 2.2: code = clip(round-half-even(x / delta)); delta == 0 gives code 0.
__device__ inline int quant_code(float x, float delta, int qmax) {
  if (!(delta > 0.0f)) return 0;
  const float r = rintf(__fdiv_rn(x, delta));
  const int c = (int)r;
  return c > qmax ? qmax : (c < -qmax ? -qmax : c);
}

// The same psi without a division per element.  With r = 1/delta to within 1 ulp (the hardware
// reciprocal), y = fl32(x * r) differs from the oracle's fl32(x / delta) by at most 2^-22 |y|, so
// whenever y is further than tau = 2^-14 (|y| <= 127.5) or 2^-18 (|y| <= 7.5) from a half-integer the
// two round to the same integer.  QuantScale holds r and the bound 0.5 - tau; the caller takes the
// largest |y - rint(y)| of a group of elements and recomputes the group with quant_code when it
// exceeds the bound (about one element in 2^13 resp. 2^17).  Scales outside [2^-100, 2^100]
// always take the exact path (bound -1); delta == 0 gives r = 0 and codes 0.  No clamp is needed:
// |x| <= the group maximum, and fl32(max / fl32(max / qmax)) rounds to qmax.
struct QuantScale { float r, bound; };
template <int QMAX>
__device__ inline QuantScale quant_scale(float delta) {
  QuantScale q;
  const bool regular = delta >= 0x1p-100f && delta <= 0x1p100f;
  q.r = regular ? __builtin_amdgcn_rcpf(delta) : 0.0f;
  q.bound = (regular || delta == 0.0f) ? 0.5f - (QMAX > 7 ? 0x1p-14f : 0x1p-18f) : -1.0f;
  return q;
}
// NE codes (as integer-valued floats) of x[0..NE) with one scale, handed to put(e, code)
template <int NE, int QMAX, class Put>
__device__ inline void quant_group(const float* x, float delta, const QuantScale& qs, Put&& put) {
  float worst = 0.0f;
#pragma unroll
  for (int e = 0; e < NE; ++e) {
    const float y = x[e] * qs.r;
    const float c = rintf(y);
    worst = fmaxf(worst, fabsf(y - c));
    put(e, c);
  }
  if (!(worst <= qs.bound)) {
#pragma unroll
    for (int e = 0; e < NE; ++e) put(e, (float)quant_code(x[e], delta, QMAX));
  }
}

typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned v6u __attribute__((ext_vector_type(6)));
// 32 INT4 codes held as integer-valued floats (every integer of [-7, 7] is an E2M3 value) become
// consecutive 6-bit E2M3 fields, element e at bit 6e: the conversion instruction takes the even
// elements in its first operand and the odd ones in its second (scale 1.0), so the codes are
// collected in that shape from the start
struct Codes32 {
  v16f ev, od;
  __device__ inline void set(int e, float c) { if (e & 1) od[e >> 1] = c; else ev[e >> 1] = c; }
  // The instruction writes its first result registers before it has read all of its inputs, and
  // the compiler does not know: a result allocated on top of part of an input corrupts the codes.
  // The empty asm statements make both operands opaque 16-register values and then need them and
  // the result at the same time, which keeps the three register ranges apart.  (Vector operands
  // of asm statements do not parse in the host pass, which never calls this.)
  __device__ inline v6u pack() const {
    v6u r = {0u, 0u, 0u, 0u, 0u, 0u};
#if defined(__HIP_DEVICE_COMPILE__)
    v16f a = ev, b = od;
    asm volatile("" : "+v"(a), "+v"(b));
    r = __builtin_amdgcn_cvt_scalef32_2xpk16_fp6_f32(a, b, 1.0f);
    asm volatile("" ::"v"(r), "v"(a), "v"(b));
#endif
    return r;
  }
};

// eight int8 codes as two's-complement bytes
__device__ inline uint2 pack8(const int (&c)[8]) {
  uint2 o;
  o.x = (unsigned)(c[0] & 0xff) | ((unsigned)(c[1] & 0xff) << 8) | ((unsigned)(c[2] & 0xff) << 16) |
        ((unsigned)(c[3] & 0xff) << 24);
  o.y = (unsigned)(c[4] & 0xff) | ((unsigned)(c[5] & 0xff) << 8) | ((unsigned)(c[6] & 0xff) << 16) |
        ((unsigned)(c[7] & 0xff) << 24);
  return o;
}

// ------------------------------------------------------------------------------------------
// Column statistics: exact token sums of K (float64 accumulation of 16-bit values) and
// per-channel max |V| (Algorithm 1, "Preprocessing": mean(K) and the scale of psi_V).  Every
// workgroup writes the partial result of its STAT_ROWS tokens; the finalize kernels reduce the
// partials of a head (no atomics, nothing to clear beforehand).
constexpr int STAT_UNROLL = 4; // rows per thread in flight

// With the smooth-V option the first pass takes the exact token sums of V instead of max|V| (the
// maximum must be taken of the centred values, which needs the mean first: k_v_absmax below).
template <bool BF16, int D, bool SMOOTH_V>
__global__ void __launch_bounds__(256) k_col_stats(const unsigned short* __restrict__ K,
                                                   const unsigned short* __restrict__ V,
                                                   double* __restrict__ k_sum, double* __restrict__ v_sum,
                                                   unsigned* __restrict__ v_max, int Nq, int N, TensorMap km,
                                                   SeqMap sm) {
  constexpr int NCG = D / 8, NRG = 256 / NCG;
  __shared__ double s_sum[NRG][D];
  __shared__ double s_vsum[SMOOTH_V ? NRG : 1][D];
  __shared__ float s_max[SMOOTH_V ? 1 : NRG][D];
  const int t = threadIdx.x, cg = t % NCG, rg = t / NCG;
  const HeadPos hp = head_pos(km, blockIdx.y);
  const Seq sq = seq_of(sm, hp.b, Nq, N);
  const int r0 = blockIdx.x * STAT_ROWS;
  const int r1 = min(r0 + STAT_ROWS, sq.nk);
  const size_t hbase = hp.base + sq.k0 * (size_t)km.sn;
  double acc[8], vacc[8];
  float mx[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { acc[e] = 0.0; vacc[e] = 0.0; mx[e] = 0.0f; }
  // STAT_UNROLL rows of K and of V are requested before the first is consumed: the pass is pure
  // streaming, and the bytes in flight per CU are what sets its bandwidth (rows past the end read
  // as zeros, which change neither a sum nor a maximum of magnitudes)
  for (int r = r0 + rg; r < r1; r += STAT_UNROLL * NRG) {
    uint4 rk[STAT_UNROLL], rv[STAT_UNROLL];
#pragma unroll
    for (int u = 0; u < STAT_UNROLL; ++u) {
      const int rr = r + u * NRG;
      rk[u] = rv[u] = make_uint4(0u, 0u, 0u, 0u);
      if (rr < r1) {
        const size_t row = row_offset(km, hbase, rr) + cg * 8;
        rk[u] = nt_load16(K + row);
        rv[u] = nt_load16(V + row);
      }
    }
#pragma unroll
    for (int u = 0; u < STAT_UNROLL; ++u) {
      float xk[8], xv[8];
      unpack8<BF16>(rk[u], xk);
      unpack8<BF16>(rv[u], xv);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        acc[e] += (double)xk[e];
        if constexpr (SMOOTH_V) vacc[e] += (double)xv[e]; else mx[e] = fmaxf(mx[e], fabsf(xv[e]));
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    s_sum[rg][cg * 8 + e] = acc[e];
    if constexpr (SMOOTH_V) s_vsum[rg][cg * 8 + e] = vacc[e]; else s_max[rg][cg * 8 + e] = mx[e];
  }
  __syncthreads();
  if (t < D) {
    double s = 0.0, sv = 0.0;
    float m = 0.0f;
    for (int g = 0; g < NRG; ++g) {
      s += s_sum[g][t];
      if constexpr (SMOOTH_V) sv += s_vsum[g][t]; else m = fmaxf(m, s_max[g][t]);
    }
    const size_t slot = ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * D + t;
    k_sum[slot] = s;
    if constexpr (SMOOTH_V) v_sum[slot] = sv;
    else v_max[slot] = __float_as_uint(m);
  }
}

// Smooth-V option, second pass over V: per-channel max |fl32(V - mean(V))|.
template <bool BF16, int D>
__global__ void __launch_bounds__(256) k_v_absmax(const unsigned short* __restrict__ V,
                                                  const float* __restrict__ v_mean,
                                                  unsigned* __restrict__ v_max, int Nq, int N, TensorMap km,
                                                  SeqMap sm) {
  constexpr int NCG = D / 8, NRG = 256 / NCG;
  __shared__ float s_max[NRG][D];
  const int t = threadIdx.x, cg = t % NCG, rg = t / NCG;
  const HeadPos hp = head_pos(km, blockIdx.y);
  const Seq sq = seq_of(sm, hp.b, Nq, N);
  const int r0 = blockIdx.x * STAT_ROWS;
  const int r1 = min(r0 + STAT_ROWS, sq.nk);
  const size_t hbase = hp.base + sq.k0 * (size_t)km.sn;
  float mean[8], mx[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { mean[e] = v_mean[(size_t)blockIdx.y * D + cg * 8 + e]; mx[e] = 0.0f; }
  for (int r = r0 + rg; r < r1; r += NRG) {
    float xv[8];
    load8<BF16>(V + row_offset(km, hbase, r) + cg * 8, xv);
#pragma unroll
    for (int e = 0; e < 8; ++e) mx[e] = fmaxf(mx[e], fabsf(__fsub_rn(xv[e], mean[e])));
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) s_max[rg][cg * 8 + e] = mx[e];
  __syncthreads();
  if (t < D) {
    float m = 0.0f;
    for (int g = 0; g < NRG; ++g) m = fmaxf(m, s_max[g][t]);
    v_max[((size_t)blockIdx.y * gridDim.x + blockIdx.x) * D + t] = __float_as_uint(m);
  }
}

// k_mean = fl32(sum / N) (Eq. 2), delta_V = fl32(max|V| / 448) (Sec. 3.3); with the smooth-V option
// this call produces v_mean = fl32(sum / N) instead of delta_V, which k_finalize_vscale adds later.
constexpr int FIN_ENT = 16, FIN_PARTS = 16;     // k_finalize_stats: entries per workgroup, threads per entry (256 threads)
__global__ void k_finalize_stats(const double* __restrict__ k_sum, const double* __restrict__ v_sum,
                                 const unsigned* __restrict__ v_max, float* __restrict__ k_mean,
                                 float* __restrict__ v_mean, float* __restrict__ v_scale, int n, int Nq, int N,
                                 int d, int Hkv, int nchunk, SeqMap sm, float code_max, int smooth_k) {
  // FIN_ENT (head, channel) entries per workgroup, FIN_PARTS threads each: thread part p sums chunks p, p + FIN_PARTS,
  // ... (the sums are exact in float64, so their order does not matter) and the parts meet in LDS.  Many threads per
  // entry because a long key range leaves many chunks (128 at 32 k keys) and a thread's loads are one round trip each.
  __shared__ double s_k[FIN_PARTS][FIN_ENT], s_v[FIN_PARTS][FIN_ENT];
  __shared__ float s_m[FIN_PARTS][FIN_ENT];
  const int e = threadIdx.x % FIN_ENT, part = threadIdx.x / FIN_ENT;
  const int i = blockIdx.x * FIN_ENT + e;
  double ks = 0.0, vs = 0.0;
  float vm = 0.0f;
  if (i < n) {
    const int head = i / d, c = i - head * d;
    const size_t p0 = (size_t)head * nchunk * d + c;
#pragma unroll 4
    for (int ch = part; ch < nchunk; ch += FIN_PARTS) {
      ks += k_sum[p0 + (size_t)ch * d];
      if (v_sum) vs += v_sum[p0 + (size_t)ch * d];
      else vm = fmaxf(vm, __uint_as_float(v_max[p0 + (size_t)ch * d]));
    }
  }
  s_k[part][e] = ks; s_v[part][e] = vs; s_m[part][e] = vm;
  __syncthreads();
  if (part == 0 && i < n) {
    const int head = i / d;
    const int nk = seq_of(sm, (unsigned)(head / Hkv), Nq, N).nk;      // this sequence's key count
    ks = 0.0; vs = 0.0; vm = 0.0f;
#pragma unroll
    for (int q = 0; q < FIN_PARTS; ++q) {
      ks += s_k[q][e];
      vs += s_v[q][e];
      vm = fmaxf(vm, s_m[q][e]);
    }
    k_mean[i] = nk > 0 && smooth_k ? (float)(ks / (double)nk) : 0.0f;   // smoothing of K off: mean 0
    if (v_sum) v_mean[i] = nk > 0 ? (float)(vs / (double)nk) : 0.0f;
    else v_scale[i] = __fdiv_rn(vm, code_max);
  }
}
// Running statistics of a growing K / V (a KV cache that is appended to): the exact column sums of K and the column
// maxima of |V| are kept as state, a new chunk's partial results are added to them, and mean(K), delta_V of the whole
// are written.  Float64 sums of 16-bit values are exact, so the state after any sequence of chunks equals the one
// pass over everything, bit for bit.  fresh != 0: the state is initialised from this chunk.
__global__ void k_accumulate_stats(const double* __restrict__ k_sum, const unsigned* __restrict__ v_max,
                                   double* __restrict__ state_sum, float* __restrict__ state_max,
                                   float* __restrict__ k_mean, float* __restrict__ v_scale, int n, int d, int nchunk,
                                   int fresh, long long n_total, float code_max) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const int head = i / d, c = i - head * d;
    const size_t p0 = (size_t)head * nchunk * d + c;
    double ks = fresh ? 0.0 : state_sum[i];
    float vm = fresh ? 0.0f : state_max[i];
#pragma unroll 8
    for (int ch = 0; ch < nchunk; ++ch) {
      ks += k_sum[p0 + (size_t)ch * d];
      vm = fmaxf(vm, __uint_as_float(v_max[p0 + (size_t)ch * d]));
    }
    state_sum[i] = ks;
    state_max[i] = vm;
    k_mean[i] = n_total > 0 ? (float)(ks / (double)n_total) : 0.0f;
    v_scale[i] = __fdiv_rn(vm, code_max);
  }
}

__global__ void k_finalize_vscale(const unsigned* __restrict__ v_max, float* __restrict__ v_scale, int n, int d,
                                  int nchunk, float code_max) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    const int head = i / d, c = i - head * d;
    float vm = 0.0f;
    for (int ch = 0; ch < nchunk; ++ch) vm = fmaxf(vm, __uint_as_float(v_max[((size_t)head * nchunk + ch) * d + c]));
    v_scale[i] = __fdiv_rn(vm, code_max);
  }
}

// ------------------------------------------------------------------------------------------
// Fixed-point digits for the Delta-S product (the scheme is described at k_quant_k).
constexpr int DS_ND = 6;                         // digits per number
constexpr int DS_MAXPAIR = 7;                    // digit pairs (a, b) with a + b up to this are multiplied: 30 of 36
constexpr float DS_MAGIC = 12582912.0f;          // 1.5 * 2^23: adding it leaves rint() of a small number in the low mantissa bits

// The DS_ND digit bytes of y (|y| < 0.5: a value already divided by its row's 2^E) into byte `pos` of out[0..DS_ND).
// y 2^42 is taken as two integers of 21 bits and a sign, N1 = rint(y 2^21) and N2 = rint((y 2^21 - N1) 2^21) (both
// steps exact in FP32: adding 1.5 * 2^23 leaves the integer in the low mantissa bits), and each is cut into a signed
// top digit (bits 14..21, -64..64) and two digits of 7 bits (0..127): y = sum_a n_a 2^(-7(a+1)) up to 2^-43.
static_assert(DS_ND == 6, "two halves of three digits");
__device__ __forceinline__ void ds_digits(float y, unsigned (&out)[DS_ND], int pos) {
  const float s1 = __fmaf_rn(y, 0x1p21f, DS_MAGIC);           // MAGIC + N1
  const float r = __fmaf_rn(y, 0x1p21f, -(s1 - DS_MAGIC));    // y 2^21 - N1, exact, |r| <= 1/2
  const float s2 = __fmaf_rn(r, 0x1p21f, DS_MAGIC);           // MAGIC + N2
  const unsigned b1 = __float_as_uint(s1), b2 = __float_as_uint(s2);   // low 22 bits: N in two's complement
  out[0] |= ((b1 >> 14) & 0xffu) << (8 * pos);
  out[1] |= ((b1 >> 7) & 0x7fu) << (8 * pos);
  out[2] |= (b1 & 0x7fu) << (8 * pos);
  out[3] |= ((b2 >> 14) & 0xffu) << (8 * pos);
  out[4] |= ((b2 >> 7) & 0x7fu) << (8 * pos);
  out[5] |= (b2 & 0x7fu) << (8 * pos);
}
// 2^-E and 2^E for a row whose largest magnitude is mx: E = exponent(mx) + 2, so that |x| 2^-E < 0.5.  A row of
// zeros, or magnitudes of 2^125 and beyond (whose products overflow FP32 anyway), get 0 and 0: Delta-S = 0.
__device__ __forceinline__ void ds_row_scale(float mx, float* down, float* up) {
  const unsigned eb = __float_as_uint(mx) >> 23;              // biased exponent (mx >= 0)
  const bool ok = mx > 0.0f && eb <= 251u;
  *down = ok ? __uint_as_float((252u - eb) << 23) : 0.0f;
  *up = ok ? __uint_as_float((eb + 2u) << 23) : 0.0f;
}

// Digits of one row of block means (DS_DIGITS), by one wavefront: `row` holds the D means (LDS or global), `digits`
// receives [digit a][channel] bytes, `scale` 2^E.
template <int D>
__device__ __forceinline__ void ds_slice_row(const float* row, unsigned char* __restrict__ digits, float* __restrict__ scale,
                                             int lane) {
  constexpr int PER = D / 64;                  // consecutive channels per lane
  float x[PER];
  float mx = 0.0f;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    x[e] = row[PER * lane + e];
    mx = fmaxf(mx, fabsf(x[e]));
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  float down, up;
  ds_row_scale(mx, &down, &up);
  if (lane == 0) *scale = up;
  unsigned dg[DS_ND];
#pragma unroll
  for (int a = 0; a < DS_ND; ++a) dg[a] = 0u;
#pragma unroll
  for (int e = 0; e < PER; ++e) ds_digits(x[e] * down, dg, e);
#pragma unroll
  for (int a = 0; a < DS_ND; ++a) {
    unsigned char* dst = digits + a * D + PER * lane;
    if constexpr (PER == 4) *reinterpret_cast<unsigned*>(dst) = dg[a];
    else if constexpr (PER == 2) *reinterpret_cast<unsigned short*>(dst) = (unsigned short)dg[a];
    else *dst = (unsigned char)dg[a];
  }
}

// ------------------------------------------------------------------------------------------
// KV head of query head bh (G query heads per KV head)
__device__ inline size_t kv_head(const TensorMap& qm, unsigned bh, int G) {
  const unsigned b = bh / (unsigned)qm.heads, h = bh - b * (unsigned)qm.heads;
  return (size_t)b * (qm.heads / G) + h / G;
}
// kappa * <q_r, mean(K)> for the rows of one thread group (the row constant that smoothing K drops
// from the scores, Sec. 3.1; needed only for the log-sum-exp output): float64 products and sums,
// one rounding.  x: this thread's 8 channels of RPT rows; NCG consecutive lanes share a row.
template <int D, int NCG, int RPT>
__device__ inline void row_constants(const float (&x)[RPT][8], float* out, int n_valid, const float* kbar8,
                                     float kappa, int cg) {
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    double dot = 0.0;
#pragma unroll
    for (int e = 0; e < 8; ++e) dot += (double)x[i][e] * (double)kbar8[e];
#pragma unroll
    for (int m = NCG / 2; m >= 1; m >>= 1) dot += __shfl_xor(dot, m, 64);
    if (cg == 0 && i < n_valid) out[i] = (float)((double)kappa * dot);
  }
}

// Q, 8-bit variant: pair-group quantization psi_Q(Q_i), no smoothing (the 8-bit kernel of the
// paper's "two kernel implementations" leaves Q as it is).  One workgroup per 128 queries of one
// (batch, head).
template <bool BF16, int D>
__global__ void __launch_bounds__(256) k_quant_q8(const unsigned short* __restrict__ Q,
                                                  float* __restrict__ q_scale, int8_t* __restrict__ q_codes,
                                                  int N, int Nk, int nQb, int block_groups, int qg,
                                                  TensorMap qm, SeqMap sm, float* __restrict__ q_corr,
                                                  const float* __restrict__ k_mean, int G, float kappa,
                                                  const float* __restrict__ head_scale, int stats_only) {
  constexpr int NCG = D / 8, NRG = 256 / NCG, RPT = BQ / NRG;  // RPT rows per thread (8 or 4)
  constexpr int QMAX = 127;
  const int t = threadIdx.x, cg = t % NCG, rg = t / NCG;
  const int qb = blockIdx.x;
  const size_t bh = blockIdx.y;
  const int n0 = qb * BQ;
  const HeadPos hp = head_pos(qm, blockIdx.y);
  const Seq sq = seq_of(sm, hp.b, N, Nk);
  const int valid = min(BQ, sq.n - n0);
  if (valid <= 0) return;                     // a block past the end of a shorter sequence
  const size_t hbase = hp.base + sq.q0 * (size_t)qm.sn;
  float x[RPT][8];
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    const int r = rg * RPT + i;
    if (r < valid) {
      load8<BF16>(Q + row_offset(qm, hbase, n0 + r) + cg * 8, x[i]);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[i][e] = 0.0f;
    }
  }
  if (q_corr) row_constants<D, NCG, RPT>(x, q_corr + (bh * nQb + qb) * BQ + rg * RPT, valid - rg * RPT,
                                         k_mean + kv_head(qm, blockIdx.y, G) * D + cg * 8, kappa, cg);
  // codes go to LDS in the packed order of this 128-query slab (contiguous in the workspace) and
  // leave as coalesced 16-byte stores
  __shared__ uint4 s_codes[BQ * D / 16];
  __shared__ float s_bmax[4];
  uint8_t* img = reinterpret_cast<uint8_t*>(s_codes);
  float block_max = 0.0f;
  if (block_groups) {       // per-block granularity: one scale for the whole 128-query block
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
#pragma unroll
      for (int e = 0; e < 8; ++e) block_max = fmaxf(block_max, fabsf(x[i][e]));
    }
    block_max = wave_max(block_max);
    if ((t & 63) == 0) s_bmax[t >> 6] = block_max;
    __syncthreads();
    block_max = fmaxf(fmaxf(s_bmax[0], s_bmax[1]), fmaxf(s_bmax[2], s_bmax[3]));
  }
#pragma unroll
  for (int p = 0; p < RPT / 2; ++p) {
    float mxr[2];                       // per query; the pair shares the larger one unless qg == 1
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      mxr[i] = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) mxr[i] = fmaxf(mxr[i], fabsf(x[2 * p + i][e]));
#pragma unroll
      for (int m = NCG / 2; m >= 1; m >>= 1) mxr[i] = fmaxf(mxr[i], __shfl_xor(mxr[i], m, 64));
    }
    if (qg == 2) mxr[0] = mxr[1] = fmaxf(mxr[0], mxr[1]);
    if (block_groups) mxr[0] = mxr[1] = block_max;
#pragma unroll
    for (int i = 2 * p; i < 2 * p + 2; ++i) {
      const float delta = head_scale ? head_scale[bh] : __fdiv_rn(mxr[i - 2 * p], (float)QMAX);
      if (cg == 0 && (qg == 1 || i == 2 * p))
        q_scale[(bh * nQb + qb) * (BQ >> (qg - 1)) + ((rg * RPT + i) >> (qg - 1))] = delta;   // qg is 1 or 2
      if (stats_only) continue;          // per-tensor scales, first pass: only the block maxima are wanted
      const QuantScale qs = quant_scale<QMAX>(delta);
      int c[8];
      quant_group<8, QMAX>(x[i], delta, qs, [&](int e, float cf) { c[e] = (int)cf; });
      *reinterpret_cast<uint2*>(img + q_code_off(rg * RPT + i, cg * 8, D)) = pack8(c);
    }
  }
  if (stats_only) return;
  __syncthreads();
  constexpr int SLAB16 = (int)(q_slab_bytes(D, false) / 16);
  uint4* dst = reinterpret_cast<uint4*>(q_codes + (bh * nQb + qb) * q_slab_bytes(D, false));
#pragma unroll
  for (int i = t; i < SLAB16; i += 256) dst[i] = s_codes[i];
}

// Q, 4-bit variant: block mean, smoothing, pair-group quantization (Algorithm 1: q_bar_i =
// mean(Q_i), psi_Q(Q_i - q_bar_i)).  Two thread-to-data maps, joined through LDS:
//  - loading and the exact column sums of the block mean use the coalesced map of k_quant_q8 (a
//    thread owns 8 channels of BQ*D/2048 rows), and the raw 16-bit rows are parked in LDS;
//  - quantization uses the map the codes are consumed in: a thread owns D/4 consecutive channels
//    of the two queries of one scale group, i.e. (half of) one MFMA lane's payload per query, so
//    the group maximum is two lane exchanges away and the codes leave through one FP32->FP6
//    conversion per query instead of per-element table look-ups and 6-bit shifts.
// LDS rows are kept as 16-byte chunks with the chunk index XOR-ed by the row's group number, which
// makes both maps conflict-free for d = 128.
// LDS: the raw rows (32 KB at d = 128), which the packed code image takes over once every thread holds its values in
// registers, and one row of column sums per wavefront (the row groups of a wavefront are summed by lane exchanges
// first) - 37 KB, so that four workgroups share a CU and their loads, arithmetic and stores overlap.
template <bool BF16, int D>
__global__ void __launch_bounds__(256, D == 256 ? 2 : 4) k_quant_q4(const unsigned short* __restrict__ Q,
                                                  float* __restrict__ q_mean, float* __restrict__ q_scale,
                                                  int8_t* __restrict__ q_codes, int N, int Nk, int nQb,
                                                  int block_groups, int qg, TensorMap qm, SeqMap sm,
                                                  float* __restrict__ q_corr, const float* __restrict__ k_mean,
                                                  int G, float kappa, const float* __restrict__ head_scale,
                                                  int stats_only, int smooth_q, unsigned char* __restrict__ q_digits,
                                                  float* __restrict__ q_dscale) {
  constexpr int NCG = D / 8, NRG = 256 / NCG, RPT = BQ / NRG;   // load map: RPT rows x 8 channels
  constexpr int CPL = D / 4, CPC = CPL / 8;                      // quantization map: 2 rows x CPL channels
  constexpr int QMAX = 7;
  constexpr int SLAB = (int)q_slab_bytes(D, true);
  __shared__ uint4 s_raw[BQ * NCG];           // the raw rows; later the packed code image of the slab
  static_assert(SLAB <= (int)sizeof(uint4) * BQ * NCG, "the code image fits where the raw rows were");
  __shared__ double s_sum[4][D];              // column sums, one row per wavefront
  __shared__ __align__(16) float s_mean[D];
  __shared__ float s_bmax[4];
  const int t = threadIdx.x;
  const int qb = blockIdx.x;
  const size_t bh = blockIdx.y;
  const int n0 = qb * BQ;
  const HeadPos hp = head_pos(qm, blockIdx.y);
  const Seq sq = seq_of(sm, hp.b, N, Nk);
  const int valid = min(BQ, sq.n - n0);
  if (valid <= 0) return;                     // a block past the end of a shorter sequence
  const size_t hbase = hp.base + sq.q0 * (size_t)qm.sn;
  auto swz = [](int r) { return (r >> 1) & (D >= 128 ? 3 : 1); };
  {
    const int cg = t % NCG, rg = t / NCG;
    double cs[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) cs[e] = 0.0;
    uint4 raw[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
      const int r = rg * RPT + i;
      raw[i] = r < valid ? nt_load16(Q + row_offset(qm, hbase, n0 + r) + cg * 8)
                         : make_uint4(0u, 0u, 0u, 0u);                  // padded rows are zero
    }
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
      const int r = rg * RPT + i;
      s_raw[r * NCG + (cg ^ swz(r))] = raw[i];
      float x8[8];
      unpack8<BF16>(raw[i], x8);
#pragma unroll
      for (int e = 0; e < 8; ++e) cs[e] += (double)x8[e];
    }
    // a wavefront holds 64 / NCG row groups (lane = (rg % (64 / NCG)) * NCG + cg): summed by lane exchanges first
    // (float64 sums of 16-bit values are exact: the order of the additions does not matter)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
#pragma unroll
      for (int o = NCG; o < 64; o <<= 1) cs[e] += __shfl_xor(cs[e], o, 64);
    }
    if ((t & 63) < NCG) {
#pragma unroll
      for (int e = 0; e < 8; ++e) s_sum[t >> 6][cg * 8 + e] = cs[e];
    }
  }
  __syncthreads();
  if (t < D) {
    double sm = 0.0;
    for (int g = 0; g < 4; ++g) sm += s_sum[g][t];
    const float m = smooth_q ? (float)(sm / (double)valid) : 0.0f;   // smoothing of Q off: mean 0
    s_mean[t] = m;
    q_mean[(bh * nQb + qb) * D + t] = m;
  }
  __syncthreads();
  // the block mean cut into digits for the Delta-S product (first wavefront; the others go on)
  if (q_digits && t < 64)
    ds_slice_row<D>(s_mean, q_digits + (bh * nQb + qb) * (size_t)(DS_ND * D), q_dscale + (bh * nQb + qb), t);

  const int pair = t >> 2, c4 = t & 3;
  float x[2][CPL];
  float mxr[2] = {0.0f, 0.0f};          // per query; the pair shares the larger one unless qg == 1
  double dotk[2] = {0.0, 0.0};          // <q_r, mean(K)> over this thread's channels (log-sum-exp output only)
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int r = 2 * pair + i;
#pragma unroll
    for (int j = 0; j < CPC; ++j) {
      unpack8<BF16>(s_raw[r * NCG + ((c4 * CPC + j) ^ swz(r))], &x[i][8 * j]);
      if (q_corr) {
        const float* kb = k_mean + kv_head(qm, blockIdx.y, G) * D + CPL * c4 + 8 * j;
#pragma unroll
        for (int e = 0; e < 8; ++e) dotk[i] += (double)x[i][8 * j + e] * (double)kb[e];
      }
      if (r < valid) {
        const float4 m0 = *reinterpret_cast<const float4*>(&s_mean[CPL * c4 + 8 * j]);
        const float4 m1 = *reinterpret_cast<const float4*>(&s_mean[CPL * c4 + 8 * j + 4]);
        const float mean[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          x[i][8 * j + e] = __fsub_rn(x[i][8 * j + e], mean[e]);
          mxr[i] = fmaxf(mxr[i], fabsf(x[i][8 * j + e]));
        }
      }
    }
    mxr[i] = fmaxf(mxr[i], __shfl_xor(mxr[i], 1, 64));
    mxr[i] = fmaxf(mxr[i], __shfl_xor(mxr[i], 2, 64));
    if (q_corr) {
      dotk[i] += __shfl_xor(dotk[i], 1, 64);
      dotk[i] += __shfl_xor(dotk[i], 2, 64);
      if (c4 == 0 && r < valid) q_corr[(bh * nQb + qb) * BQ + r] = (float)((double)kappa * dotk[i]);
    }
  }
  if (qg == 2) mxr[0] = mxr[1] = fmaxf(mxr[0], mxr[1]);
  if (block_groups) {       // per-block granularity: one scale for the whole 128-query block
    const float bm = wave_max(mxr[0]);
    if ((t & 63) == 0) s_bmax[t >> 6] = bm;
    __syncthreads();
    mxr[0] = mxr[1] = fmaxf(fmaxf(s_bmax[0], s_bmax[1]), fmaxf(s_bmax[2], s_bmax[3]));
  }
  __syncthreads();                       // every thread holds its rows in registers: the image may take their place
  uint8_t* img = reinterpret_cast<uint8_t*>(s_raw);
  // the thread's CPL channels of a query are one MFMA lane payload of 32 codes (d = 128), half of one (d = 64) or
  // two of them (d = 256: both lane halves of one operand)
  constexpr int NPL = CPL > 32 ? CPL / 32 : 1, CPP = CPL / NPL;     // payloads per query and thread, codes in each
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const float delta = head_scale ? head_scale[bh] : __fdiv_rn(mxr[i], (float)QMAX);
    if (c4 == 0 && (qg == 1 || i == 0))   // qg is 1 or 2
      q_scale[(bh * nQb + qb) * (BQ >> (qg - 1)) + ((2 * pair + i) >> (qg - 1))] = delta;
    if (stats_only) continue;            // per-tensor scales, first pass: only the block maxima are wanted
    const QuantScale qs = quant_scale<QMAX>(delta);
#pragma unroll
    for (int pl = 0; pl < NPL; ++pl) {
      Codes32 cd;
#pragma unroll
      for (int e = 0; e < 16; ++e) { cd.ev[e] = 0.0f; cd.od[e] = 0.0f; }
#pragma unroll
      for (int g = 0; g < CPP / 8; ++g)
        quant_group<8, QMAX>(&x[i][CPP * pl + 8 * g], delta, qs, [&](int e, float c) { cd.set(8 * g + e, c); });
      const v6u pw = cd.pack();
      int lane_m, e0;
      const size_t op = q_op6(2 * pair + i, CPL * c4 + CPP * pl, D, &lane_m, &e0);
      const int d0 = (6 * e0) >> 5;
#pragma unroll
      for (int k = 0; k < CPP * 6 / 32; ++k)
        *reinterpret_cast<unsigned*>(img + op + op6_byte(lane_m, 4 * (d0 + k))) = pw[k];
    }
  }
  if (stats_only) return;
  __syncthreads();
  uint4* dst = reinterpret_cast<uint4*>(q_codes + (bh * nQb + qb) * q_slab_bytes(D, true));
  const uint4* src = reinterpret_cast<const uint4*>(img);
#pragma unroll
  for (int i = t; i < SLAB / 16; i += 256) dst[i] = src[i];
}

// ------------------------------------------------------------------------------------------
// K: smoothing by the token mean, group quantization (runs of 16 keys by default) and, in the int4
// mode, Delta-S.
// (Algorithm 1: psi_K(K_j) after K = K - mean(K); Sec. 3.1: Delta-S = q_bar_i . gamma(K)^T.)
//
// One workgroup per 64 keys of one (batch, KV head); wavefront w owns keys 16w..16w+15, which
// is exactly one default quantization group.  Lane l holds key 16w + l%16 and the D/4 consecutive
// channels (D/4)*(l/16) .. +D/4-1, i.e. the wavefront reads 16 whole rows as one contiguous
// piece.  That is also the B-operand shape of the 16x16x4 FP64 MFMA (lane l supplies
// B[k = l/16][column l%16]) once contraction slot (step cs, k = l/16) is assigned channel
// (D/4)*(l/16) + cs - any assignment is valid as long as the A operand uses the same one - so
// the smoothed keys feed the Delta-S product straight from the registers they were quantized in.
//
// Delta-S: D[i, t] = fl32(kappa * <q_bar_i, gamma(K)_t>), the inner product formed exactly (or in float64) so that
// the value does not depend on summation order: a small GEMM [nQb x d] . [d x 64] per query head of the KV group,
// walked 32 query blocks ("a pass") at a time; three forms, template parameter DSM below.  The FP64 form:
// v_mfma_f64_16x16x4_f64 sustains about 70 TFLOP/s on the whole chip and, unlike the low-precision matrix
// instructions, does not run concurrently with other vector work of the SIMD, so it costs its own matrix time
// (2*nQb*N*d flops per head) on top of the quantization.
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int DS_QROWS = 32;    // query-block means staged in LDS per pass: two 16-row MFMA tiles

// How the Delta-S product is formed (template parameter DSM of k_quant_k):
//   DS_DIGITS  both factors cut into 7-bit digits of a fixed-point number and multiplied digit by digit on the INT8
//              matrix instruction: exact integer sums, recombined in float64 (the default),
//   DS_FP32    v_mfma_f32_16x16x4_f32: faster still, approximate (an option of the boundary),
//   DS_FP64    v_mfma_f64_16x16x4_f64: the reference form (an option of the boundary).
//
// DS_DIGITS.  A row x of d numbers (a block mean q_bar_i, or a smoothed key) with largest magnitude below 2^(E-1) is
// written x_c = 2^E sum_a n_a[c] 2^(-7(a+1)) + rest, a = 0..5, with digits that fit a signed byte (ds_digits: n_0 and
// n_3 in -64..64, the others in 0..127); the rest is zero for every x_c whose exponent is within 17 of the row's
// largest (smaller ones lose what lies below 2^(E-42)).  Then
//   <x, y> = 2^(Ex+Ey) sum_{a,b} 2^(-7(a+b+2)) sum_c n_a[c] m_b[c],
// the inner sums are integers below 2^23 that v_mfma_i32_16x16x64_i8 forms exactly, pairs with the same a + b share
// an accumulator (below 2^25), and the pairs with a + b > 7 are left out: together less than 2^-45 of
// |x|_max |y|_max d.  The result agrees with the float64 inner product far below its FP32 rounding, at a quarter of
// the FP64 instruction's time, and - being INT8 matrix work - it runs alongside the vector work of the quantizers.
enum { DS_DIGITS = 0, DS_FP32 = 1, DS_FP64 = 2 };

template <bool BF16, bool INT4, int D, int DSM = DS_DIGITS>
__global__ void __launch_bounds__(256, D == 256 ? 2 : (INT4 && DSM == DS_DIGITS ? 3 : 4)) k_quant_k(const unsigned short* __restrict__ K,
                                                 const float* __restrict__ k_mean,
                                                 float* __restrict__ k_scale, int8_t* __restrict__ k_codes,
                                                 const float* __restrict__ q_mean,
                                                 float* __restrict__ delta_s, int Nq, int Nmax, int nKb,
                                                 int nQb, int G, float kappa, int block_groups, int kg,
                                                 int causal, TensorMap km, SeqMap sm,
                                                 const float* __restrict__ head_scale, int stats_only,
                                                 int zero_ds, const unsigned char* __restrict__ q_digits,
                                                 const float* __restrict__ q_dscale) {
  constexpr bool DS32 = DSM == DS_FP32, DSD = INT4 && DSM == DS_DIGITS;
  constexpr int CPL = D / 4;                       // channels per lane (32 or 16)
  constexpr int QMAX = INT4 ? 7 : 127;
  // LDS row of staged block means: channel c sits at column c + 16*(c / 32) when D = 128, so the
  // 32 lanes of a half-wavefront (16 rows x 2 channel groups) hit 32 different banks (odd stride)
  constexpr int SQW = D + (D >= 128 ? 48 : 0) + 1;
  constexpr int PADSH = D == 256 ? 6 : 5;          // 16 columns of padding after every 32 (d = 128) / 64 (d = 256) channels
  __shared__ uint4 s_codes[BKV * D / 16];          // the block's packed image
  __shared__ float s_q[INT4 && !DSD ? DS_QROWS : 1][SQW];
  // DS_DIGITS: a staged row is its DS_ND digit planes of D bytes; 16 bytes of padding make the 16 rows of an operand read
  // start in 16 different bank groups
  constexpr int ROWB = DS_ND * D + 16;
  __shared__ __align__(16) unsigned char s_qd[DSD ? DS_QROWS : 1][DSD ? ROWB : 16];
  __shared__ float s_qs[DS_QROWS];                 // 2^E of the staged rows
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int r16 = lane & 15, k4 = lane >> 4;
  const int kb = blockIdx.x;
  const size_t bhkv = blockIdx.y;
  const int n0 = kb * BKV;
  const int r = 16 * w + r16, c0 = CPL * k4;
  // this sequence's key count N, query-block count nQs and causal offset (the slabs keep the
  // strides nQb, nKb of the longest sequence)
  const HeadPos hp = head_pos(km, blockIdx.y);
  const Seq sq = seq_of(sm, hp.b, Nq, Nmax);
  const int N = sq.nk, coff = sq.coff;
  const int nQs = (sq.n + BQ - 1) / BQ;
  if (n0 >= N) return;                             // a block past the end of a shorter sequence

  // Delta-S passes: (query head of the group, 32 query blocks); the first pass's block means are
  // requested before the K rows so that both round trips overlap
  constexpr int QPT = DS_QROWS * (D / 4) / 256;    // float4 pieces per thread per pass
  // A sequence with fewer than 32 query blocks (a decode step, a short chunk against a long cache) would leave most
  // rows of a pass empty: there the rows of all the query heads of the group are numbered through, head-major,
  // and share passes ("flat").  Which pass a row sits in changes nothing in its value.
  const bool flat = nQs < DS_QROWS;
  const int npass_h = flat ? 1 : (nQs + DS_QROWS - 1) / DS_QROWS;
  const int nrow = flat ? G * max(nQs, 0) : 0;
  const int npass = INT4 ? (flat ? (nrow + DS_QROWS - 1) / DS_QROWS : G * npass_h) : 0;
  // under a causal mask (query r sees keys t <= r + coff) query block i sees this key block only
  // if 128 i + 127 + coff >= its first key: the passes of a head start with the one that holds
  // block (first key - coff) / 128
  const int p_first = causal && !flat ? (max(kb * BKV - coff, 0) / BQ) / DS_QROWS : 0;
  // A pass is named by (head of the group, pass within the head), or by (0, pass) when flat; carried as a pair so
  // that nothing in the pass loop divides.
  struct PassId { int g, ph; };
  const PassId pass_first = {0, p_first};
  auto pass_ok = [&](PassId q) { return INT4 && (flat ? q.ph < npass : q.g < G); };
  auto pass_next = [&](PassId q) {
    PassId n = q;
    if (flat || q.ph + 1 < npass_h) n.ph = q.ph + 1;
    else { n.g = q.g + 1; n.ph = p_first; }
    return n;
  };
  const float inv_nqs = 1.0f / (float)max(nQs, 1);
  // row rr of a pass: its index (head, query block) in the [B H][nQb] arrays, or -1 for an empty row
  const int bh0 = (int)bhkv * G;
  auto pass_row = [&](PassId q, int rr) {
    if (flat) {
      // (R + 1/2) / nQs never comes within rounding distance of an integer for the few thousand rows there can be
      const int R = q.ph * DS_QROWS + rr, g = (int)(((float)R + 0.5f) * inv_nqs);
      return R < nrow ? (bh0 + g) * nQb + (R - g * nQs) : -1;
    }
    const int i = q.ph * DS_QROWS + rr;
    return i < nQs ? (bh0 + q.g) * nQb + i : -1;
  };
  constexpr int NCH = DS_ND * D / 16;              // 16-byte pieces of a row of digits
  constexpr int QPD = DS_QROWS * NCH / 256;        // ... per thread per pass
  float4 qpre[DSD ? 1 : QPT];
  uint4 dpre[DSD ? QPD : 1];
  float spre = 0.0f;
  auto load_q = [&](PassId p) {
    if constexpr (DSD) {
      if (!flat) {
        // the pass's rows are consecutive query blocks of one head: one contiguous piece of the digit array
        const int row0 = (bh0 + p.g) * nQb + p.ph * DS_QROWS, rows = min(DS_QROWS, nQs - p.ph * DS_QROWS);
        const uint4* src = reinterpret_cast<const uint4*>(q_digits + (size_t)row0 * (DS_ND * D));
#pragma unroll
        for (int k = 0; k < QPD; ++k) {
          const int idx = t + k * 256;
          dpre[k] = idx < rows * NCH ? src[idx] : make_uint4(0u, 0u, 0u, 0u);
        }
        if (t < DS_QROWS) spre = t < rows ? q_dscale[row0 + t] : 0.0f;
        return;
      }
#pragma unroll
      for (int k = 0; k < QPD; ++k) {
        const int idx = t + k * 256, rr = idx / NCH, ch = idx % NCH;
        const int row = pass_row(p, rr);
        dpre[k] = row >= 0 ? *reinterpret_cast<const uint4*>(q_digits + (size_t)row * (DS_ND * D) + 16 * ch)
                           : make_uint4(0u, 0u, 0u, 0u);
      }
      if (t < DS_QROWS) {
        const int row = pass_row(p, t);
        spre = row >= 0 ? q_dscale[row] : 0.0f;
      }
      return;
    }
#pragma unroll
    for (int k = 0; k < (DSD ? 0 : QPT); ++k) {
      const int idx = t + k * 256, rr = idx / (D / 4), c4 = idx % (D / 4);
      const int row = pass_row(p, rr);
      qpre[k] = row >= 0 ? *reinterpret_cast<const float4*>(q_mean + (size_t)row * D + 4 * c4)
                         : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  auto store_q = [&]() {
    if constexpr (DSD) {
#pragma unroll
      for (int k = 0; k < QPD; ++k) {
        const int idx = t + k * 256, rr = idx / NCH, ch = idx % NCH;
        *reinterpret_cast<uint4*>(&s_qd[rr][16 * ch]) = dpre[k];
      }
      if (t < DS_QROWS) s_qs[t] = spre;
      return;
    }
#pragma unroll
    for (int k = 0; k < (DSD ? 0 : QPT); ++k) {
      const int idx = t + k * 256, rr = idx / (D / 4), c4 = idx % (D / 4);
      const int col = 4 * c4 + (D >= 128 ? 16 * ((4 * c4) >> PADSH) : 0);
      s_q[rr][col + 0] = qpre[k].x; s_q[rr][col + 1] = qpre[k].y;
      s_q[rr][col + 2] = qpre[k].z; s_q[rr][col + 3] = qpre[k].w;
    }
  };
  if constexpr (INT4) load_q(pass_first);

  float x[CPL];
  float mx = 0.0f;
  const size_t hbase = hp.base + sq.k0 * (size_t)km.sn;
  if (n0 + r < N) {
#pragma unroll
    for (int p = 0; p < CPL / 8; ++p) {
      float x8[8];
      load8<BF16, false>(K + row_offset(km, hbase, n0 + r) + c0 + 8 * p, x8);
      const float4 m0 = *reinterpret_cast<const float4*>(k_mean + bhkv * D + c0 + 8 * p);
      const float4 m1 = *reinterpret_cast<const float4*>(k_mean + bhkv * D + c0 + 8 * p + 4);
      const float mean[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        x[8 * p + e] = __fsub_rn(x8[e], mean[e]);
        mx = fmaxf(mx, fabsf(x[8 * p + e]));
      }
    }
  } else {
#pragma unroll
    for (int e = 0; e < CPL; ++e) x[e] = 0.0f;      // padded keys: codes 0, Delta-S 0
  }
  // lanes l, l^16, l^32, l^48 hold one key: its maximum first, then (unless every key has its own
  // scale) the run of 4 keys, then (default) the wavefront's run of 16
  mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  const float mx_key = mx;                         // this key's largest magnitude (DS_DIGITS: its fixed-point exponent)
  if (kg >= 4) {
    mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 2, 64));
  }
  if (kg == 16) {
    mx = fmaxf(mx, __shfl_xor(mx, 4, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 8, 64));
  }
  __shared__ float s_bmax[4];
  if (block_groups) {       // per-block granularity: one scale for the whole 64-key block
    if (lane == 0) s_bmax[w] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(s_bmax[0], s_bmax[1]), fmaxf(s_bmax[2], s_bmax[3]));
  }
  const float delta = head_scale ? head_scale[bhkv] : __fdiv_rn(mx, (float)QMAX);
  const int ksh = kg == 16 ? 4 : (kg == 4 ? 2 : 0);
  if (k4 == 0 && (r16 & (kg - 1)) == 0) k_scale[(bhkv * nKb + kb) * (BKV >> ksh) + ((16 * w + r16) >> ksh)] = delta;
  if (stats_only) return;                // per-tensor scales, first pass: only the block maxima are wanted
  uint8_t* img = reinterpret_cast<uint8_t*>(s_codes);
  const QuantScale qs = quant_scale<QMAX>(delta);
  if constexpr (INT4) {
    // the lane's CPL codes are CPL*6/32 consecutive dwords of one MFMA lane's payload (all 6 of
    // them when d = 128; dwords 0..2 or 3..5 when d = 64), or two whole payloads (d = 256)
    constexpr int NPL = CPL > 32 ? CPL / 32 : 1, CPP = CPL / NPL;
#pragma unroll
    for (int pl = 0; pl < NPL; ++pl) {
      Codes32 cd;
#pragma unroll
      for (int e = 0; e < 16; ++e) { cd.ev[e] = 0.0f; cd.od[e] = 0.0f; }
#pragma unroll
      for (int g = 0; g < CPP / 8; ++g)
        quant_group<8, QMAX>(x + CPP * pl + 8 * g, delta, qs, [&](int e, float c) { cd.set(8 * g + e, c); });
      const v6u pw = cd.pack();
      int lane_m, e0;
      const size_t op = k_op6(r, c0 + CPP * pl, D, &lane_m, &e0);
      const int d0 = (6 * e0) >> 5;
#pragma unroll
      for (int i = 0; i < CPP * 6 / 32; ++i)
        *reinterpret_cast<unsigned*>(img + op + op6_byte(lane_m, 4 * (d0 + i))) = pw[i];
    }
  } else {
#pragma unroll
    for (int p = 0; p < CPL / 8; ++p) {
      int c[8];
      quant_group<8, QMAX>(x + 8 * p, delta, qs, [&](int e, float cf) { c[e] = (int)cf; });
      *reinterpret_cast<uint2*>(img + k_code_off(r, c0 + 8 * p, D)) = pack8(c);
    }
  }
  __syncthreads();
  constexpr int BLK16 = (int)(k_block_bytes(D, INT4) / 16);
  uint4* dst = reinterpret_cast<uint4*>(k_codes + (bhkv * nKb + kb) * k_block_bytes(D, INT4));
#pragma unroll
  for (int i = t; i < BLK16; i += 256) dst[i] = s_codes[i];

  if constexpr (INT4) {
    // FP64 MFMA lane map: lane l supplies A[l%16][l/16] and B[l/16][l%16]; result element v of
    // lane l is row 4*v + l/16, column l%16
    // the smoothed keys stay in FP32 registers and are widened per use: CPL more conversions per
    // pass (a few percent of the pass's MFMA time) instead of 2 CPL more live registers, which is
    // what lets four workgroups share a CU
    const double kap = (double)kappa;
    const int qcol = c0 + (D >= 128 ? 16 * k4 : 0);
    // DS_DIGITS: the digits of this lane's CPL smoothed values as B operands of v_mfma_i32_16x16x64_i8.  An operand is
    // 16 bytes per lane; contraction slot (step st, lane group k4, byte j) is given channel CPL k4 + 16 st + j - any
    // assignment is valid as long as the A operand uses the same one.
    constexpr int NST = CPL / 16;
    v4i bd[DSD ? DS_ND : 1][DSD ? NST : 1];
    double key_up = 0.0;
    if constexpr (DSD) {
      float down, up;
      ds_row_scale(mx_key, &down, &up);
      key_up = (double)up * kap;                   // 2^E of the key, times kappa
#pragma unroll
      for (int st = 0; st < NST; ++st) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          unsigned dg[DS_ND];
#pragma unroll
          for (int a = 0; a < DS_ND; ++a) dg[a] = 0u;
#pragma unroll
          for (int j = 0; j < 4; ++j) ds_digits(x[16 * st + 4 * q4 + j] * down, dg, j);
#pragma unroll
          for (int a = 0; a < DS_ND; ++a) bd[a][st][q4] = (int)dg[a];
        }
      }
      // (opaque to the compiler from here on: it would otherwise form the digits anew in every pass)
#pragma unroll
      for (int a = 0; a < DS_ND; ++a) {
#pragma unroll
        for (int st = 0; st < NST; ++st) asm volatile("" : "+v"(bd[a][st]));
      }
    }
    bool first_pass = true;
    for (PassId p = pass_first; pass_ok(p); p = pass_next(p)) {
      if (!first_pass) __syncthreads();            // everyone is done with the previous pass's rows
      first_pass = false;
      store_q();
      __syncthreads();
      if (pass_ok(pass_next(p))) load_q(pass_next(p));   // next pass, in flight under the MFMAs
      // rows 16..31 of the pass all empty (a short last pass): their chain of matrix instructions is left out
      const bool upper = p.ph * DS_QROWS + 16 < (flat ? nrow : nQs);
      // (not flat: the pass's rows are consecutive rows of the Delta-S array of one head)
      const unsigned rowstride = (unsigned)nKb * BKV;
      float* const out0 = delta_s + (size_t)((bh0 + p.g) * nQb + p.ph * DS_QROWS) * rowstride + (size_t)(n0 + r);
      const int rows_here = nQs - p.ph * DS_QROWS;
      const bool full = rows_here >= DS_QROWS;        // (all but a head's last pass)
      auto put = [&](int rr, float val) {
        if (!flat) {
          if (full || rr < rows_here) out0[(size_t)((unsigned)rr * rowstride)] = val;
          return;
        }
        const int row = pass_row(p, rr);
        if (row >= 0) delta_s[(size_t)row * rowstride + (size_t)(n0 + r)] = val;
      };
      if constexpr (DSD) {
        // accumulators by digit-pair weight: acc[k][rt] collects the pairs with a + b = k for row tile rt; result
        // element v of lane l is row 4 (l / 16) + v, column l % 16
        // one 16-row tile at a time (its seven accumulators are live only until its results are out)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) {
          if (rt == 1 && !upper) break;
          if (zero_ds) {     // (Q not smoothed: the block means are zero and so is Delta-S)
#pragma unroll
            for (int v = 0; v < 4; ++v) put(16 * rt + 4 * k4 + v, 0.0f);
            continue;
          }
          v4i acc[DS_MAXPAIR + 1];
#pragma unroll
          for (int a = 0; a < DS_ND; ++a) {
#pragma unroll
            for (int st = 0; st < NST; ++st) {
              const v4i qa = *reinterpret_cast<const v4i*>(&s_qd[16 * rt + r16][a * D + CPL * k4 + 16 * st]);
#pragma unroll
              for (int b = 0; b < DS_ND && a + b <= DS_MAXPAIR; ++b) {
                // the first pair of a weight starts from zero (a constant operand of the instruction)
                const bool first = st == 0 && a == (a + b >= DS_ND ? a + b - (DS_ND - 1) : 0);
                acc[a + b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(qa, bd[b][st], first ? v4i{0, 0, 0, 0} : acc[a + b], 0, 0, 0);
              }
            }
          }
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const int rr = 16 * rt + 4 * k4 + v;
            // sum_k acc_k 2^(-7 (k + 2)): neighbours joined as integers first (128 acc_k + acc_{k+1} < 2^31: with the
            // digit ranges of ds_digits the largest is 128 acc_6 + acc_7 < 2^30.1 at d = 128; at d = 256 that one would
            // not fit and stays apart), then float64, smallest weights first
            static_assert(DS_ND == 6 && DS_MAXPAIR == 7, "eight accumulators");
            const int u0 = acc[0][v] * 128 + acc[1][v], u1 = acc[2][v] * 128 + acc[3][v],
                      u2 = acc[4][v] * 128 + acc[5][v];
            double sum;
            if constexpr (D <= 128) {
              sum = (double)(acc[6][v] * 128 + acc[7][v]) * 0x1p-63;
            } else {
              sum = (double)acc[7][v] * 0x1p-63;
              sum = __fma_rn((double)acc[6][v], 0x1p-56, sum);
            }
            sum = __fma_rn((double)u2, 0x1p-49, sum);
            sum = __fma_rn((double)u1, 0x1p-35, sum);
            sum = __fma_rn((double)u0, 0x1p-21, sum);
            put(rr, (float)(sum * ((double)s_qs[rr] * key_up)));
          }
        }
      } else if constexpr (DS32) {
        // Faster, approximate form (an option of the boundary): the same product on the FP32 form of the
        // instruction (result element v of lane l is row 4*(l/16) + v, column l%16).  FP32 accumulation:
        // within (d + 2) 2^-24 kappa sum_c |q_bar_c gamma(K)_c| of the exact value, about half a unit of 2^-24 of
        // that magnitude on average.  It runs at twice the rate and under the vector work of the workgroups
        // that share the CU, so the product costs next to nothing on top of the quantization.
        v4f acc0 = {0.0f, 0.0f, 0.0f, 0.0f}, acc1 = {0.0f, 0.0f, 0.0f, 0.0f};
        if (!zero_ds) {
#pragma unroll
          for (int cs = 0; cs < CPL; ++cs) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x4f32(s_q[r16][qcol + cs], x[cs], acc0, 0, 0, 0);
            if (upper) acc1 = __builtin_amdgcn_mfma_f32_16x16x4f32(s_q[16 + r16][qcol + cs], x[cs], acc1, 0, 0, 0);
          }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          put(4 * k4 + v, __fmul_rn(kappa, acc0[v]));
          if (upper) put(16 + 4 * k4 + v, __fmul_rn(kappa, acc1[v]));
        }
      } else {
        v4d acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};
        if (!zero_ds) {      // (Q not smoothed: the block means are zero and so is Delta-S)
#pragma unroll
          for (int cs = 0; cs < CPL; ++cs) {
            asm volatile("" : "+v"(x[cs]));            // keeps the widening inside the pass loop
            const double bk = (double)x[cs];
            acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64((double)s_q[r16][qcol + cs], bk, acc0, 0, 0, 0);
            if (upper) acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64((double)s_q[16 + r16][qcol + cs], bk, acc1, 0, 0, 0);
          }
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          put(4 * v + k4, (float)(kap * acc0[v]));
          if (upper) put(16 + 4 * v + k4, (float)(kap * acc1[v]));
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// V: per-channel FP8 codes (E4M3, or E5M2 with the E5M2 template flag), transposed into the A-operand
// order of the P~V product
// (Sec. 3.3; Algorithm 1 "Preprocessing": (delta_V, V^) = psi_V(V)).  v_mean is null, or the token
// mean to subtract first (smooth-V option, SMOOTH_V).
template <bool BF16, int D, bool SMOOTH_V, int PVF>
__global__ void __launch_bounds__(256) k_quant_v(const unsigned short* __restrict__ V,
                                                 const float* __restrict__ v_scale,
                                                 const float* __restrict__ v_mean,
                                                 uint8_t* __restrict__ v_codes, int Nq, int Nmax, int nKb,
                                                 TensorMap km, SeqMap sm) {
  constexpr int NCG = D / 8, NRG = 256 / NCG, RPT = BKV / NRG;
  __shared__ uint8_t tile[BKV][D + 16];
  const int t = threadIdx.x, cg = t % NCG, rg = t / NCG;
  const int kb = blockIdx.x;
  const size_t bh = blockIdx.y;
  const int n0 = kb * BKV;
  const HeadPos hp = head_pos(km, blockIdx.y);
  const Seq sq = seq_of(sm, hp.b, Nq, Nmax);
  const int N = sq.nk;
  if (n0 >= N) return;                             // a block past the end of a shorter sequence
  const size_t hbase = hp.base + sq.k0 * (size_t)km.sn;
  float sc[8], mean[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    sc[e] = v_scale[bh * D + cg * 8 + e];
    mean[e] = SMOOTH_V ? v_mean[bh * D + cg * 8 + e] : 0.0f;
  }
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    const int r = rg * RPT + i;
    float x[8];
    if (n0 + r < N) {
      load8<BF16>(V + row_offset(km, hbase, n0 + r) + cg * 8, x);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if constexpr (SMOOTH_V) x[e] = __fsub_rn(x[e], mean[e]);
        x[e] = sc[e] > 0.0f ? __fdiv_rn(x[e], sc[e]) : 0.0f;
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = 0.0f;
    }
    int w0 = 0, w1 = 0;
    if constexpr (PVF == PV_INT8) {
      // psi of Sec. 2.2 with qmax 127: |x / delta_V| <= 127 (1 + 2^-23), round-half-even, two's-complement bytes
      int c[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) c[e] = (int)rintf(x[e]);
      const uint2 pk = pack8(c);
      w0 = (int)pk.x; w1 = (int)pk.y;
    } else if constexpr (PVF == PV_E5M2) {
      w0 = __builtin_amdgcn_cvt_pk_bf8_f32(x[0], x[1], w0, false);
      w0 = __builtin_amdgcn_cvt_pk_bf8_f32(x[2], x[3], w0, true);
      w1 = __builtin_amdgcn_cvt_pk_bf8_f32(x[4], x[5], w1, false);
      w1 = __builtin_amdgcn_cvt_pk_bf8_f32(x[6], x[7], w1, true);
    } else {
      w0 = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], w0, false);
      w0 = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], w0, true);
      w1 = __builtin_amdgcn_cvt_pk_fp8_f32(x[4], x[5], w1, false);
      w1 = __builtin_amdgcn_cvt_pk_fp8_f32(x[6], x[7], w1, true);
    }
    *reinterpret_cast<uint2*>(&tile[r][cg * 8]) = make_uint2((unsigned)w0, (unsigned)w1);
  }
  __syncthreads();
  uint8_t* dst = v_codes + (bh * nKb + kb) * (size_t)BKV * D;
  constexpr int NCHUNK = (D / 32) * 2 * 64;
  for (int ch = t; ch < NCHUNK; ch += 256) {
    const int lane = ch & 63, part = (ch >> 6) & 1, ct = ch >> 7;
    const int c = 32 * ct + (lane & 31), key0 = 32 * part + 16 * (lane >> 5);
    unsigned w[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
      w[q] = (unsigned)tile[key0 + 4 * q][c] | ((unsigned)tile[key0 + 4 * q + 1][c] << 8) |
             ((unsigned)tile[key0 + 4 * q + 2][c] << 16) | ((unsigned)tile[key0 + 4 * q + 3][c] << 24);
    *reinterpret_cast<uint4*>(dst + (size_t)ch * 16) = make_uint4(w[0], w[1], w[2], w[3]);
  }
}

// ------------------------------------------------------------------------------------------
// Per-tensor scales (the coarsest granularity of the paper's comparison, Sec. 2.2): the quantizers run
// once in per-block mode just to leave every block's scale, this kernel takes the largest scale of a
// head (delta = fl32(max / qmax) is monotone in the maximum, so the largest block scale is the
// head's), and the quantizers run again with that scale.  One workgroup per head; `per_block` scale
// entries per block, `stride` entries per head, blocks counted from the sequence's own length.
__global__ void __launch_bounds__(256) k_head_scale(const float* __restrict__ scale, float* __restrict__ head_scale,
                                                    int per_block, int stride, int tokens_per_block, int heads,
                                                    int which_k, int Nq, int Nk, SeqMap sm) {
  __shared__ float s_m[4];
  const unsigned head = blockIdx.x;
  const Seq sq = seq_of(sm, head / (unsigned)heads, Nq, Nk);
  const int n = which_k ? sq.nk : sq.n;
  const int entries = ((n + tokens_per_block - 1) / tokens_per_block) * per_block;
  float m = 0.0f;
  for (int i = threadIdx.x; i < entries; i += 256) m = fmaxf(m, scale[(size_t)head * stride + i]);
  m = wave_max(m);
  if ((threadIdx.x & 63) == 0) s_m[threadIdx.x >> 6] = m;
  __syncthreads();
  if (threadIdx.x == 0) head_scale[head] = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
}

// ------------------------------------------------------------------------------------------
// Copies from the packed workspace to plain layouts (used only by sage_attn_quant).
__global__ void k_unpack_codes(const int8_t* __restrict__ packed, int8_t* __restrict__ plain, int N,
                               int d, size_t slab, int which, int fp6) {
  // grid: (ceil(N*d/256), heads); which: 0 = q, 1 = k, 2 = v; fp6: q/k hold 6-bit E2M3 codes
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)N * d) return;
  const int n = (int)(i / d), c = (int)(i % d);
  const uint8_t* src = reinterpret_cast<const uint8_t*>(packed) + (size_t)blockIdx.y * slab;
  int8_t b;
  if (fp6 && which != 2) {
    int lane_m, e;
    const size_t op = which == 0 ? q_op6(n, c, d, &lane_m, &e) : k_op6(n, c, d, &lane_m, &e);
    const int bit = 6 * e, by = bit >> 3;
    unsigned v = src[op + op6_byte(lane_m, by)];
    if (by + 1 < 24) v |= (unsigned)src[op + op6_byte(lane_m, by + 1)] << 8;
    b = (int8_t)e2m3_to_int4_code((v >> (bit & 7)) & 63u);
  } else {
    const size_t off = which == 0 ? q_code_off(n, c, d) : (which == 1 ? k_code_off(n, c, d) : v_code_off(n, c, d));
    b = (int8_t)src[off];
  }
  plain[(size_t)blockIdx.y * N * d + i] = b;
}

__global__ void k_unpack_rows(const float* __restrict__ src, float* __restrict__ dst, int n_valid,
                              int src_stride) {
  // grid: (ceil(n_valid/256), rows): dst[row][0..n_valid) = src[row][0..n_valid)
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_valid) dst[(size_t)blockIdx.y * n_valid + i] = src[(size_t)blockIdx.y * src_stride + i];
}

// ------------------------------------------------------------------------------------------
// The statistics pass: mean(K) and delta_V (and mean(V) with the smooth-V option) into P.k_mean, P.v_scale, P.v_mean.
template <bool BF16, int D>
static void launch_stats_t(const Dims& Dm, const Ptrs& P, hipStream_t s) {
  const int BHkv = Dm.B * Dm.Hkv;
  const unsigned short* k = (const unsigned short*)P.k;
  const unsigned short* v = (const unsigned short*)P.v;
  const int nstat = BHkv * Dm.d;
  const dim3 gstat((Dm.Nk + STAT_ROWS - 1) / STAT_ROWS, BHkv);
  const TensorMap km = make_tensor_map(Dm.nhd, Dm.Hkv, Dm.Nk, Dm.d, Dm.seq.cu_q != nullptr);
  const SeqMap sm = Dm.seq;
  const int nchunk = (int)gstat.x;
  const float code_max = Dm.pvf == PV_INT8 ? INT8_PV_MAX : (Dm.pvf == PV_E5M2 ? E5M2_MAX : E4M3_MAX);
  if (Dm.smooth_v) {
    k_col_stats<BF16, D, true><<<gstat, 256, 0, s>>>(k, v, P.k_sum, P.v_sum, P.v_max, Dm.N, Dm.Nk, km, sm);
    k_finalize_stats<<<(nstat + FIN_ENT - 1) / FIN_ENT, FIN_ENT * FIN_PARTS, 0, s>>>(P.k_sum, P.v_sum, P.v_max, P.k_mean, P.v_mean, P.v_scale,
                                                        nstat, Dm.N, Dm.Nk, Dm.d, Dm.Hkv, nchunk, sm, code_max, Dm.smooth_k);
    k_v_absmax<BF16, D><<<gstat, 256, 0, s>>>(v, P.v_mean, P.v_max, Dm.N, Dm.Nk, km, sm);
    k_finalize_vscale<<<(nstat + 255) / 256, 256, 0, s>>>(P.v_max, P.v_scale, nstat, Dm.d, nchunk, code_max);
  } else {
    k_col_stats<BF16, D, false><<<gstat, 256, 0, s>>>(k, v, P.k_sum, nullptr, P.v_max, Dm.N, Dm.Nk, km, sm);
    k_finalize_stats<<<(nstat + FIN_ENT - 1) / FIN_ENT, FIN_ENT * FIN_PARTS, 0, s>>>(P.k_sum, nullptr, P.v_max, P.k_mean, nullptr, P.v_scale,
                                                        nstat, Dm.N, Dm.Nk, Dm.d, Dm.Hkv, nchunk, sm, code_max, Dm.smooth_k);
  }
}

template <bool BF16, bool INT4, int D>
static hipError_t launch_prologue_t(const Dims& Dm, const Ptrs& P, hipStream_t s) {
  const int BH = Dm.B * Dm.H, BHkv = Dm.B * Dm.Hkv;
  const unsigned short* q = (const unsigned short*)P.q;
  const unsigned short* k = (const unsigned short*)P.k;
  const unsigned short* v = (const unsigned short*)P.v;
  const bool varlen = Dm.seq.cu_q != nullptr;
  const TensorMap qm = make_tensor_map(Dm.nhd, Dm.H, Dm.N, Dm.d, varlen),
                  km = make_tensor_map(Dm.nhd, Dm.Hkv, Dm.Nk, Dm.d, varlen);
  const SeqMap sm = Dm.seq;
  const float* v_mean = Dm.smooth_v ? P.v_mean : nullptr;
  // Q goes first: it depends on nothing, and with the statistics pass next to the K and V quantizers
  // those re-read K and V while the chip's memory-side cache still holds most of them.  Only when
  // the log-sum-exp output is wanted does Q wait for mean(K) (its row constants need it).
  auto quant_q_pass = [&](float* corr, const float* head_scale, int stats_only) {
    if constexpr (INT4)
      k_quant_q4<BF16, D><<<dim3(Dm.nQb, BH), 256, 0, s>>>(q, P.q_mean, P.q_scale, P.q_codes, Dm.N, Dm.Nk, Dm.nQb,
                                                       Dm.block_groups, Dm.qg, qm, sm, corr, P.k_mean,
                                                       Dm.H / Dm.Hkv, Dm.kappa, head_scale, stats_only, Dm.smooth_q,
                                                       Dm.ds_mode == DS_DIGITS && Dm.smooth_q ? P.q_digits : nullptr, P.q_dscale);
    else
      k_quant_q8<BF16, D><<<dim3(Dm.nQb, BH), 256, 0, s>>>(q, P.q_scale, P.q_codes, Dm.N, Dm.Nk, Dm.nQb,
                                                       Dm.block_groups, Dm.qg, qm, sm, corr, P.k_mean,
                                                       Dm.H / Dm.Hkv, Dm.kappa, head_scale, stats_only);
  };
  auto quant_q = [&]() {
    float* corr = Dm.want_lse ? P.q_corr : nullptr;
    if (Dm.tensor_groups) {     // block scales, their maximum per head, then the codes with that one scale
      quant_q_pass(nullptr, nullptr, 1);
      k_head_scale<<<BH, 256, 0, s>>>(P.q_scale, P.q_head_scale, BQ / Dm.qg, Dm.nQb * (BQ / Dm.qg), BQ, Dm.H, 0, Dm.N,
                                     Dm.Nk, sm);
      quant_q_pass(corr, P.q_head_scale, 0);
    } else {
      quant_q_pass(corr, nullptr, 0);
    }
  };
  auto quant_k_pass = [&](const float* head_scale, int stats_only) {
#define SAGE_QK(DSM_)                                                                                                  \
  k_quant_k<BF16, INT4, D, DSM_><<<dim3(Dm.nKb, BHkv), 256, 0, s>>>(k, P.k_mean, P.k_scale, P.k_codes, P.q_mean, P.delta_s, \
                                                                    Dm.N, Dm.Nk, Dm.nKb, Dm.nQb, Dm.H / Dm.Hkv, Dm.kappa,  \
                                                                    Dm.block_groups, Dm.kg, Dm.causal, km, sm, head_scale, \
                                                                    stats_only, !Dm.smooth_q, P.q_digits, P.q_dscale)
    // (the 8-bit build has no Delta-S: one instantiation, named by the default mode)
    if (INT4 && Dm.ds_mode == DS_FP32) SAGE_QK(INT4 ? DS_FP32 : DS_DIGITS);
    else if (INT4 && Dm.ds_mode == DS_FP64) SAGE_QK(INT4 ? DS_FP64 : DS_DIGITS);
    else {
      SAGE_QK(DS_DIGITS);
    }
#undef SAGE_QK
  };
  if (!Dm.want_lse) quant_q();
  if (!Dm.stats_given) launch_stats_t<BF16, D>(Dm, P, s);     // else P.k_mean and P.v_scale are the caller's arrays
  if (Dm.want_lse) quant_q();
  if (Dm.tensor_groups) {
    quant_k_pass(nullptr, 1);
    k_head_scale<<<BHkv, 256, 0, s>>>(P.k_scale, P.k_head_scale, BKV / Dm.kg, Dm.nKb * (BKV / Dm.kg), BKV, Dm.Hkv, 1,
                                     Dm.N, Dm.Nk, sm);
    quant_k_pass(P.k_head_scale, 0);
  } else {
    quant_k_pass(nullptr, 0);
  }
  const dim3 gv(Dm.nKb, BHkv);
#define SAGE_QV(SV, PF, VM) k_quant_v<BF16, D, SV, PF><<<gv, 256, 0, s>>>(v, P.v_scale, VM, P.v_codes, Dm.N, Dm.Nk, Dm.nKb, km, sm)
  if (Dm.smooth_v) {
    if (Dm.pvf == PV_INT8) SAGE_QV(true, PV_INT8, v_mean);
    else if (Dm.pvf == PV_E5M2) SAGE_QV(true, PV_E5M2, v_mean);
    else SAGE_QV(true, PV_E4M3, v_mean);
  } else {
    if (Dm.pvf == PV_INT8) SAGE_QV(false, PV_INT8, nullptr);
    else if (Dm.pvf == PV_E5M2) SAGE_QV(false, PV_E5M2, nullptr);
    else SAGE_QV(false, PV_E4M3, nullptr);
  }
#undef SAGE_QV
  return hipGetLastError();
}

hipError_t launch_prologue(const Dims& D, const Ptrs& P, hipStream_t s) {
#define SAGE_PRO(BF, I4, DD) return launch_prologue_t<BF, I4, DD>(D, P, s)
  if (D.d == 256) {
    if (D.bf16) { if (D.int4) SAGE_PRO(true, true, 256); else SAGE_PRO(true, false, 256); }
    else        { if (D.int4) SAGE_PRO(false, true, 256); else SAGE_PRO(false, false, 256); }
  } else if (D.d == 128) {
    if (D.bf16) { if (D.int4) SAGE_PRO(true, true, 128); else SAGE_PRO(true, false, 128); }
    else        { if (D.int4) SAGE_PRO(false, true, 128); else SAGE_PRO(false, false, 128); }
  } else {
    if (D.bf16) { if (D.int4) SAGE_PRO(true, true, 64); else SAGE_PRO(true, false, 64); }
    else        { if (D.int4) SAGE_PRO(false, true, 64); else SAGE_PRO(false, false, 64); }
  }
#undef SAGE_PRO
}

hipError_t launch_kv_stats(const Dims& D, const Ptrs& P, hipStream_t s) {
  if (D.d == 256)      { if (D.bf16) launch_stats_t<true, 256>(D, P, s); else launch_stats_t<false, 256>(D, P, s); }
  else if (D.d == 128) { if (D.bf16) launch_stats_t<true, 128>(D, P, s); else launch_stats_t<false, 128>(D, P, s); }
  else                 { if (D.bf16) launch_stats_t<true, 64>(D, P, s); else launch_stats_t<false, 64>(D, P, s); }
  return hipGetLastError();
}

template <bool BF16, int D>
static void launch_stats_update_t(const Dims& Dm, const Ptrs& P, double* state_sum, float* state_max, int fresh,
                                  long long n_total, hipStream_t s) {
  const int BHkv = Dm.B * Dm.Hkv, nstat = BHkv * Dm.d;
  const dim3 gstat((Dm.Nk + STAT_ROWS - 1) / STAT_ROWS, BHkv);
  const TensorMap km = make_tensor_map(Dm.nhd, Dm.Hkv, Dm.Nk, Dm.d, false);
  const float code_max = Dm.pvf == PV_INT8 ? INT8_PV_MAX : (Dm.pvf == PV_E5M2 ? E5M2_MAX : E4M3_MAX);
  k_col_stats<BF16, D, false><<<gstat, 256, 0, s>>>((const unsigned short*)P.k, (const unsigned short*)P.v, P.k_sum, nullptr,
                                                    P.v_max, Dm.N, Dm.Nk, km, Dm.seq);
  k_accumulate_stats<<<(nstat + 255) / 256, 256, 0, s>>>(P.k_sum, P.v_max, state_sum, state_max, P.k_mean, P.v_scale, nstat,
                                                         Dm.d, (int)gstat.x, fresh, n_total, code_max);
}

hipError_t launch_kv_stats_update(const Dims& D, const Ptrs& P, double* state_sum, float* state_max, int fresh,
                                  long long n_total, hipStream_t s) {
#define SAGE_SU(BF, DD) launch_stats_update_t<BF, DD>(D, P, state_sum, state_max, fresh, n_total, s)
  if (D.d == 256)      { if (D.bf16) SAGE_SU(true, 256); else SAGE_SU(false, 256); }
  else if (D.d == 128) { if (D.bf16) SAGE_SU(true, 128); else SAGE_SU(false, 128); }
  else                 { if (D.bf16) SAGE_SU(true, 64); else SAGE_SU(false, 64); }
#undef SAGE_SU
  return hipGetLastError();
}

hipError_t launch_unpack(const Dims& D, const Ptrs& P, const void* quant_out, hipStream_t s) {
  const sage_quant_out& qo = *(const sage_quant_out*)quant_out;
  struct { int8_t *qc, *kc; uint8_t* vc; float *qs, *ks, *vs, *km, *qm, *ds, *vm; } o = {
      qo.q_codes, qo.k_codes, qo.v_codes, qo.q_scale, qo.k_scale, qo.v_scale, qo.k_mean, qo.q_mean, qo.delta_s,
      qo.v_mean};
  const int BH = D.B * D.H, BHkv = D.B * D.Hkv;
  const unsigned gx = (unsigned)(((size_t)D.N * D.d + 255) / 256), gxk = (unsigned)(((size_t)D.Nk * D.d + 255) / 256);
  if (o.qc) k_unpack_codes<<<dim3(gx, BH), 256, 0, s>>>(P.q_codes, o.qc, D.N, D.d, D.nQb * q_slab_bytes(D.d, D.int4), 0, D.int4);
  if (o.kc) k_unpack_codes<<<dim3(gxk, BHkv), 256, 0, s>>>(P.k_codes, o.kc, D.Nk, D.d, D.nKb * k_block_bytes(D.d, D.int4), 1, D.int4);
  if (o.vc) k_unpack_codes<<<dim3(gxk, BHkv), 256, 0, s>>>((const int8_t*)P.v_codes, (int8_t*)o.vc, D.Nk, D.d, (size_t)D.nKb * BKV * D.d, 2, 0);
  const int nqg = (D.N + D.qg - 1) / D.qg, nkg = (D.Nk + D.kg - 1) / D.kg;
  if (o.qs) k_unpack_rows<<<dim3((nqg + 255) / 256, BH), 256, 0, s>>>(P.q_scale, o.qs, nqg, D.nQb * (BQ / D.qg));
  if (o.ks) k_unpack_rows<<<dim3((nkg + 255) / 256, BHkv), 256, 0, s>>>(P.k_scale, o.ks, nkg, D.nKb * (BKV / D.kg));
  if (o.vs) k_unpack_rows<<<dim3(1, BHkv), 256, 0, s>>>(P.v_scale, o.vs, D.d, D.d);
  if (o.km) k_unpack_rows<<<dim3(1, BHkv), 256, 0, s>>>(P.k_mean, o.km, D.d, D.d);
  if (o.vm && D.smooth_v) k_unpack_rows<<<dim3(1, BHkv), 256, 0, s>>>(P.v_mean, o.vm, D.d, D.d);
  if (D.int4) {
    if (o.qm) k_unpack_rows<<<dim3(1, BH * D.nQb), 256, 0, s>>>(P.q_mean, o.qm, D.d, D.d);
    if (o.ds) k_unpack_rows<<<dim3((D.Nk + 255) / 256, BH * D.nQb), 256, 0, s>>>(P.delta_s, o.ds, D.Nk, D.nKb * BKV);
  }
  return hipGetLastError();
}

}  // namespace sage
