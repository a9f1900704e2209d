// Preprocessing kernels of the quantized attention forward pass (paper Sec. 3.1-3.3 and the
// "Preprocessing" line plus the first line of the outer loop of Algorithm 1): token means,
// smoothing, Delta-S, group quantization of Q and K, per-channel FP8 quantization of V.
// Everything here is bandwidth-bound; codes are written in the MFMA fragment order described
// in sage_common.h so that the attention kernel can move them with plain 16-byte copies.
#include "sage_common.h"
#include "sage_attn.h"

namespace sage {

// ------------------------------------------------------------------------------------------
// small helpers
template <bool BF16>
__device__ inline void load8(const unsigned short* p, float (&x)[8]) {
  const uint4 raw = *reinterpret_cast<const uint4*>(p);
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

template <bool AS_E4M3>
__device__ inline uint2 pack8(const int (&cc)[8]) {
  int c[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) c[e] = AS_E4M3 ? (int)int4_code_to_e4m3(cc[e]) : cc[e];
  uint2 o;
  o.x = (unsigned)(c[0] & 0xff) | ((unsigned)(c[1] & 0xff) << 8) | ((unsigned)(c[2] & 0xff) << 16) |
        ((unsigned)(c[3] & 0xff) << 24);
  o.y = (unsigned)(c[4] & 0xff) | ((unsigned)(c[5] & 0xff) << 8) | ((unsigned)(c[6] & 0xff) << 16) |
        ((unsigned)(c[7] & 0xff) << 24);
  return o;
}

// ------------------------------------------------------------------------------------------
// Column statistics: exact token sums of K (float64 accumulation of 16-bit values) and
// per-channel max |V| (Algorithm 1, "Preprocessing": mean(K) and the scale of psi_V).
__global__ void k_zero_stats(double* k_sum, unsigned* v_max, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) { k_sum[i] = 0.0; v_max[i] = 0u; }
}

constexpr int STAT_ROWS = 512;  // tokens per workgroup of k_col_stats

template <bool BF16, int D>
__global__ void __launch_bounds__(256) k_col_stats(const unsigned short* __restrict__ K,
                                                   const unsigned short* __restrict__ V,
                                                   double* __restrict__ k_sum,
                                                   unsigned* __restrict__ v_max, int N) {
  constexpr int NCG = D / 8, NRG = 256 / NCG;
  __shared__ double s_sum[NRG][D];
  __shared__ float s_max[NRG][D];
  const int t = threadIdx.x, cg = t % NCG, rg = t / NCG;
  const size_t head = (size_t)blockIdx.y * N * D;
  const int r0 = blockIdx.x * STAT_ROWS;
  const int r1 = min(r0 + STAT_ROWS, N);
  double acc[8];
  float mx[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { acc[e] = 0.0; mx[e] = 0.0f; }
  for (int r = r0 + rg; r < r1; r += NRG) {
    float xk[8], xv[8];
    load8<BF16>(K + head + (size_t)r * D + cg * 8, xk);
    load8<BF16>(V + head + (size_t)r * D + cg * 8, xv);
#pragma unroll
    for (int e = 0; e < 8; ++e) { acc[e] += (double)xk[e]; mx[e] = fmaxf(mx[e], fabsf(xv[e])); }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) { s_sum[rg][cg * 8 + e] = acc[e]; s_max[rg][cg * 8 + e] = mx[e]; }
  __syncthreads();
  if (t < D) {
    double s = 0.0;
    float m = 0.0f;
    for (int g = 0; g < NRG; ++g) { s += s_sum[g][t]; m = fmaxf(m, s_max[g][t]); }
    atomicAdd(&k_sum[(size_t)blockIdx.y * D + t], s);
    atomicMax(&v_max[(size_t)blockIdx.y * D + t], __float_as_uint(m));  // m >= 0: uint order = float order
  }
}

// k_mean = fl32(sum / N) (Eq. 2), delta_V = fl32(max|V| / 448) (Sec. 3.3)
__global__ void k_finalize_stats(const double* __restrict__ k_sum, const unsigned* __restrict__ v_max,
                                 float* __restrict__ k_mean, float* __restrict__ v_scale, int n, int N) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    k_mean[i] = (float)(k_sum[i] / (double)N);
    v_scale[i] = __fdiv_rn(__uint_as_float(v_max[i]), E4M3_MAX);
  }
}

// ------------------------------------------------------------------------------------------
// Q: block mean, smoothing (int4 mode), pair-group quantization.  One workgroup per 128
// queries of one (batch, head)  (Algorithm 1: q_bar_i = mean(Q_i), psi_Q(Q_i - q_bar_i)).
template <bool BF16, bool INT4, int D>
__global__ void __launch_bounds__(256) k_quant_q(const unsigned short* __restrict__ Q,
                                                 float* __restrict__ q_mean, float* __restrict__ q_scale,
                                                 int8_t* __restrict__ q_codes, int N, int nQb) {
  constexpr int NCG = D / 8, NRG = 256 / NCG, RPT = BQ / NRG;  // RPT rows per thread (8 or 4)
  constexpr int QMAX = INT4 ? 7 : 127;
  __shared__ double s_sum[NRG][D];
  __shared__ float s_mean[D];
  const int t = threadIdx.x, cg = t % NCG, rg = t / NCG;
  const int qb = blockIdx.x;
  const size_t bh = blockIdx.y;
  const int n0 = qb * BQ;
  const int valid = min(BQ, N - n0);
  float x[RPT][8];
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    const int r = rg * RPT + i;
    if (r < valid) {
      load8<BF16>(Q + (bh * N + n0 + r) * D + cg * 8, x[i]);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[i][e] = 0.0f;
    }
  }
  if constexpr (INT4) {
    double cs[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      cs[e] = 0.0;
#pragma unroll
      for (int i = 0; i < RPT; ++i) cs[e] += (double)x[i][e];   // padded rows are zero
      s_sum[rg][cg * 8 + e] = cs[e];
    }
    __syncthreads();
    if (t < D) {
      double s = 0.0;
      for (int g = 0; g < NRG; ++g) s += s_sum[g][t];
      const float m = (float)(s / (double)valid);
      s_mean[t] = m;
      q_mean[(bh * nQb + qb) * D + t] = m;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
      if (rg * RPT + i < valid) {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[i][e] = __fsub_rn(x[i][e], s_mean[cg * 8 + e]);
      }
    }
  }
  // codes go to LDS in the packed order of this 128-query slab (4 tiles x d/32 steps x 64 lanes
  // chunks, contiguous in the workspace) and leave as coalesced 16-byte stores
  __shared__ uint4 s_codes[BQ * D / 16];
  uint8_t* img = reinterpret_cast<uint8_t*>(s_codes);
#pragma unroll
  for (int p = 0; p < RPT / 2; ++p) {
    float mx = 0.0f;
#pragma unroll
    for (int e = 0; e < 8; ++e) mx = fmaxf(mx, fmaxf(fabsf(x[2 * p][e]), fabsf(x[2 * p + 1][e])));
#pragma unroll
    for (int m = NCG / 2; m >= 1; m >>= 1) mx = fmaxf(mx, __shfl_xor(mx, m, 64));
    const float delta = __fdiv_rn(mx, (float)QMAX);
    if (cg == 0) q_scale[(bh * nQb + qb) * (BQ / QGROUP) + (rg * RPT) / 2 + p] = delta;
#pragma unroll
    for (int i = 2 * p; i < 2 * p + 2; ++i) {
      int c[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) c[e] = quant_code(x[i][e], delta, QMAX);
      *reinterpret_cast<uint2*>(img + q_code_off(rg * RPT + i, cg * 8, D)) = pack8<INT4>(c);
    }
  }
  __syncthreads();
  uint4* dst = reinterpret_cast<uint4*>(q_codes + (bh * nQb + qb) * (size_t)BQ * D);
#pragma unroll
  for (int i = t; i < BQ * D / 16; i += 256) dst[i] = s_codes[i];
}

// ------------------------------------------------------------------------------------------
// K: smoothing by the token mean, 16-key-group quantization.  One workgroup per 64 keys;
// a 16-key group is exactly one wavefront's rows.  (Algorithm 1: psi_K(K_j) after
// K = K - mean(K).)
template <bool BF16, bool INT4, int D>
__global__ void __launch_bounds__(256) k_quant_k(const unsigned short* __restrict__ K,
                                                 const float* __restrict__ k_mean,
                                                 float* __restrict__ k_scale, int8_t* __restrict__ k_codes,
                                                 int N, int nKb) {
  constexpr int NCG = D / 8, NRG = 256 / NCG, RPT = BKV / NRG;  // 4 or 2 rows per thread
  constexpr int QMAX = INT4 ? 7 : 127;
  const int t = threadIdx.x, cg = t % NCG, rg = t / NCG;
  const int kb = blockIdx.x;
  const size_t bh = blockIdx.y;
  const int n0 = kb * BKV;
  float mean[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) mean[e] = k_mean[bh * D + cg * 8 + e];
  float x[RPT][8];
  float mx = 0.0f;
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    const int n = n0 + rg * RPT + i;
    if (n < N) {
      load8<BF16>(K + (bh * N + n) * D + cg * 8, x[i]);
#pragma unroll
      for (int e = 0; e < 8; ++e) { x[i][e] = __fsub_rn(x[i][e], mean[e]); mx = fmaxf(mx, fabsf(x[i][e])); }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[i][e] = 0.0f;
    }
  }
  mx = wave_max(mx);  // the wavefront's rows are keys 16*wave .. 16*wave+15 of the block
  const float delta = __fdiv_rn(mx, (float)QMAX);
  if ((t & 63) == 0) k_scale[(bh * nKb + kb) * (BKV / KGROUP) + (t >> 6)] = delta;
  __shared__ uint4 s_codes[BKV * D / 16];   // the block's packed image, then coalesced 16-byte stores
  uint8_t* img = reinterpret_cast<uint8_t*>(s_codes);
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    int c[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) c[e] = quant_code(x[i][e], delta, QMAX);
    *reinterpret_cast<uint2*>(img + k_code_off(rg * RPT + i, cg * 8, D)) = pack8<INT4>(c);
  }
  __syncthreads();
  uint4* dst = reinterpret_cast<uint4*>(k_codes + (bh * nKb + kb) * (size_t)BKV * D);
#pragma unroll
  for (int i = t; i < BKV * D / 16; i += 256) dst[i] = s_codes[i];
}

// ------------------------------------------------------------------------------------------
// V: per-channel FP8 E4M3 codes, transposed into the A-operand order of the P~V product
// (Sec. 3.3; Algorithm 1 "Preprocessing": (delta_V, V^) = psi_V(V)).
template <bool BF16, int D>
__global__ void __launch_bounds__(256) k_quant_v(const unsigned short* __restrict__ V,
                                                 const float* __restrict__ v_scale,
                                                 uint8_t* __restrict__ v_codes, int N, int nKb) {
  constexpr int NCG = D / 8, NRG = 256 / NCG, RPT = BKV / NRG;
  __shared__ uint8_t tile[BKV][D + 16];
  const int t = threadIdx.x, cg = t % NCG, rg = t / NCG;
  const int kb = blockIdx.x;
  const size_t bh = blockIdx.y;
  const int n0 = kb * BKV;
  float sc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) sc[e] = v_scale[bh * D + cg * 8 + e];
#pragma unroll
  for (int i = 0; i < RPT; ++i) {
    const int r = rg * RPT + i;
    float x[8];
    if (n0 + r < N) {
      load8<BF16>(V + (bh * N + n0 + r) * D + cg * 8, x);
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = sc[e] > 0.0f ? __fdiv_rn(x[e], sc[e]) : 0.0f;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x[e] = 0.0f;
    }
    int w0 = 0, w1 = 0;
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(x[0], x[1], w0, false);
    w0 = __builtin_amdgcn_cvt_pk_fp8_f32(x[2], x[3], w0, true);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(x[4], x[5], w1, false);
    w1 = __builtin_amdgcn_cvt_pk_fp8_f32(x[6], x[7], w1, true);
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
// Delta-S (Sec. 3.1): D[i, t] = fl32(kappa * <q_bar_i, gamma(K)_t>), inner product in float64
// so that the value does not depend on summation order.  A small GEMM per (batch, query head):
// [nQb x d] . [d x N], run on the FP64 matrix pipe (v_mfma_f64_16x16x4f64).  One workgroup per
// 64 keys; wavefront w owns keys 16w..16w+15 and keeps their gamma(K) (as float64 B operands)
// in registers while it walks the query blocks 16 at a time.
typedef double v4d __attribute__((ext_vector_type(4)));

constexpr int DS_QROWS = 32;    // query-block means staged in LDS per pass: two 16-row MFMA tiles

template <bool BF16, int D>
__global__ void __launch_bounds__(256) k_delta_s(const unsigned short* __restrict__ K,
                                                 const float* __restrict__ k_mean,
                                                 const float* __restrict__ q_mean,
                                                 float* __restrict__ delta_s, int N, int nQb, int nKb,
                                                 int H, int Hkv, float kappa) {
  __shared__ float s_gk[BKV][D + 1];
  __shared__ float s_q[DS_QROWS][D + 1];
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int kb = blockIdx.x;
  const size_t bh = blockIdx.y;
  const int b = (int)(bh / H), h = (int)(bh % H);
  const size_t bhkv = (size_t)b * Hkv + h / (H / Hkv);
  const int n0 = kb * BKV;
  // the first pass of block means is requested before the K tile so both round trips overlap
  constexpr int QPT = DS_QROWS * (D / 4) / 256;   // float4 pieces per thread per pass
  float4 qpre[QPT];
  auto load_q = [&](int i0) {
#pragma unroll
    for (int k = 0; k < QPT; ++k) {
      const int idx = t + k * 256, r = idx / (D / 4), c4 = idx % (D / 4);
      qpre[k] = (i0 + r < nQb) ? *reinterpret_cast<const float4*>(q_mean + (bh * nQb + i0 + r) * D + 4 * c4)
                               : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  };
  auto store_q = [&]() {
#pragma unroll
    for (int k = 0; k < QPT; ++k) {
      const int idx = t + k * 256, r = idx / (D / 4), c4 = idx % (D / 4);
      s_q[r][4 * c4 + 0] = qpre[k].x; s_q[r][4 * c4 + 1] = qpre[k].y;
      s_q[r][4 * c4 + 2] = qpre[k].z; s_q[r][4 * c4 + 3] = qpre[k].w;
    }
  };
  load_q(0);
  {
    constexpr int NCG = D / 8, NRG = 256 / NCG, RPT = BKV / NRG;
    const int cg = t % NCG, rg = t / NCG;
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
      const int r = rg * RPT + i;
      float x[8];
      if (n0 + r < N) {
        load8<BF16>(K + (bhkv * N + n0 + r) * D + cg * 8, x);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = __fsub_rn(x[e], k_mean[bhkv * D + cg * 8 + e]);
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = 0.0f;
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) s_gk[r][cg * 8 + e] = x[e];
    }
  }
  // operand lane map of the 16x16x4 FP64 MFMA: lane l supplies A[l%16][l/16] and B[l/16][l%16];
  // result: lane l, element v holds row 4*v + l/16, column l%16
  const int r16 = lane & 15, k4 = lane >> 4;
  const double kap = (double)kappa;
  bool have_b = false;
  double bk[D / 4];
  for (int i0 = 0; i0 < nQb; i0 += DS_QROWS) {
    if (i0 > 0) __syncthreads();       // everyone is done with the previous pass's rows
    store_q();
    __syncthreads();
    if (i0 + DS_QROWS < nQb) load_q(i0 + DS_QROWS);   // next pass, in flight under the MFMAs
    if (!have_b) {   // this wavefront's 16 keys as float64 B operands, kept for the whole kernel
#pragma unroll
      for (int cs = 0; cs < D / 4; ++cs) bk[cs] = (double)s_gk[16 * w + r16][4 * cs + k4];
      have_b = true;
    }
    // two independent accumulator chains (rows 0..15 and 16..31 of the pass) keep the pipe busy
    v4d acc0 = {0.0, 0.0, 0.0, 0.0}, acc1 = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int cs = 0; cs < D / 4; ++cs) {
      acc0 = __builtin_amdgcn_mfma_f64_16x16x4f64((double)s_q[r16][4 * cs + k4], bk[cs], acc0, 0, 0, 0);
      acc1 = __builtin_amdgcn_mfma_f64_16x16x4f64((double)s_q[16 + r16][4 * cs + k4], bk[cs], acc1, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int i = i0 + 4 * v + k4;
      float* dst = delta_s + (bh * nQb + i) * (size_t)nKb * BKV + n0 + 16 * w + r16;
      if (i < nQb) dst[0] = (float)(kap * acc0[v]);
      if (i + 16 < nQb) dst[(size_t)16 * nKb * BKV] = (float)(kap * acc1[v]);
    }
  }
}

// ------------------------------------------------------------------------------------------
// Copies from the packed workspace to plain layouts (used only by sage_attn_quant).
__global__ void k_unpack_codes(const int8_t* __restrict__ packed, int8_t* __restrict__ plain, int N,
                               int d, size_t slab, int which, int e4m3_ints) {
  // grid: (ceil(N*d/256), heads); which: 0 = q, 1 = k, 2 = v; e4m3_ints: q/k bytes hold integers as E4M3
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)N * d) return;
  const int n = (int)(i / d), c = (int)(i % d);
  const size_t off = which == 0 ? q_code_off(n, c, d) : (which == 1 ? k_code_off(n, c, d) : v_code_off(n, c, d));
  int8_t b = packed[(size_t)blockIdx.y * slab + off];
  if (e4m3_ints && which != 2) b = (int8_t)e4m3_to_int4_code((unsigned char)b);
  plain[(size_t)blockIdx.y * N * d + i] = b;
}

__global__ void k_unpack_rows(const float* __restrict__ src, float* __restrict__ dst, int n_valid,
                              int src_stride) {
  // grid: (ceil(n_valid/256), rows): dst[row][0..n_valid) = src[row][0..n_valid)
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_valid) dst[(size_t)blockIdx.y * n_valid + i] = src[(size_t)blockIdx.y * src_stride + i];
}

// ------------------------------------------------------------------------------------------
template <bool BF16, bool INT4, int D>
static hipError_t launch_prologue_t(const Dims& Dm, const Ptrs& P, hipStream_t s) {
  const int BH = Dm.B * Dm.H, BHkv = Dm.B * Dm.Hkv;
  const unsigned short* q = (const unsigned short*)P.q;
  const unsigned short* k = (const unsigned short*)P.k;
  const unsigned short* v = (const unsigned short*)P.v;
  const int nstat = BHkv * Dm.d;
  k_zero_stats<<<(nstat + 255) / 256, 256, 0, s>>>(P.k_sum, P.v_max, nstat);
  k_col_stats<BF16, D><<<dim3((Dm.N + STAT_ROWS - 1) / STAT_ROWS, BHkv), 256, 0, s>>>(k, v, P.k_sum, P.v_max, Dm.N);
  k_finalize_stats<<<(nstat + 255) / 256, 256, 0, s>>>(P.k_sum, P.v_max, P.k_mean, P.v_scale, nstat, Dm.N);
  k_quant_q<BF16, INT4, D><<<dim3(Dm.nQb, BH), 256, 0, s>>>(q, P.q_mean, P.q_scale, P.q_codes, Dm.N, Dm.nQb);
  k_quant_k<BF16, INT4, D><<<dim3(Dm.nKb, BHkv), 256, 0, s>>>(k, P.k_mean, P.k_scale, P.k_codes, Dm.N, Dm.nKb);
  k_quant_v<BF16, D><<<dim3(Dm.nKb, BHkv), 256, 0, s>>>(v, P.v_scale, P.v_codes, Dm.N, Dm.nKb);
  if constexpr (INT4)
    k_delta_s<BF16, D><<<dim3(Dm.nKb, BH), 256, 0, s>>>(k, P.k_mean, P.q_mean, P.delta_s, Dm.N, Dm.nQb,
                                                        Dm.nKb, Dm.H, Dm.Hkv, Dm.kappa);
  return hipGetLastError();
}

hipError_t launch_prologue(const Dims& D, const Ptrs& P, hipStream_t s) {
#define SAGE_PRO(BF, I4, DD) return launch_prologue_t<BF, I4, DD>(D, P, s)
  if (D.d == 128) {
    if (D.bf16) { if (D.int4) SAGE_PRO(true, true, 128); else SAGE_PRO(true, false, 128); }
    else        { if (D.int4) SAGE_PRO(false, true, 128); else SAGE_PRO(false, false, 128); }
  } else {
    if (D.bf16) { if (D.int4) SAGE_PRO(true, true, 64); else SAGE_PRO(true, false, 64); }
    else        { if (D.int4) SAGE_PRO(false, true, 64); else SAGE_PRO(false, false, 64); }
  }
#undef SAGE_PRO
}

hipError_t launch_unpack(const Dims& D, const Ptrs& P, const void* quant_out, hipStream_t s) {
  const sage_quant_out& qo = *(const sage_quant_out*)quant_out;
  struct { int8_t *qc, *kc; uint8_t* vc; float *qs, *ks, *vs, *km, *qm, *ds; } o = {
      qo.q_codes, qo.k_codes, qo.v_codes, qo.q_scale, qo.k_scale, qo.v_scale, qo.k_mean, qo.q_mean, qo.delta_s};
  const int BH = D.B * D.H, BHkv = D.B * D.Hkv;
  const unsigned gx = (unsigned)(((size_t)D.N * D.d + 255) / 256);
  if (o.qc) k_unpack_codes<<<dim3(gx, BH), 256, 0, s>>>(P.q_codes, o.qc, D.N, D.d, (size_t)D.nQb * BQ * D.d, 0, D.int4);
  if (o.kc) k_unpack_codes<<<dim3(gx, BHkv), 256, 0, s>>>(P.k_codes, o.kc, D.N, D.d, (size_t)D.nKb * BKV * D.d, 1, D.int4);
  if (o.vc) k_unpack_codes<<<dim3(gx, BHkv), 256, 0, s>>>((const int8_t*)P.v_codes, (int8_t*)o.vc, D.N, D.d, (size_t)D.nKb * BKV * D.d, 2, 0);
  const int nqg = (D.N + QGROUP - 1) / QGROUP, nkg = (D.N + KGROUP - 1) / KGROUP;
  if (o.qs) k_unpack_rows<<<dim3((nqg + 255) / 256, BH), 256, 0, s>>>(P.q_scale, o.qs, nqg, D.nQb * (BQ / QGROUP));
  if (o.ks) k_unpack_rows<<<dim3((nkg + 255) / 256, BHkv), 256, 0, s>>>(P.k_scale, o.ks, nkg, D.nKb * (BKV / KGROUP));
  if (o.vs) k_unpack_rows<<<dim3(1, BHkv), 256, 0, s>>>(P.v_scale, o.vs, D.d, D.d);
  if (o.km) k_unpack_rows<<<dim3(1, BHkv), 256, 0, s>>>(P.k_mean, o.km, D.d, D.d);
  if (D.int4) {
    if (o.qm) k_unpack_rows<<<dim3(1, BH * D.nQb), 256, 0, s>>>(P.q_mean, o.qm, D.d, D.d);
    if (o.ds) k_unpack_rows<<<dim3((D.N + 255) / 256, BH * D.nQb), 256, 0, s>>>(P.delta_s, o.ds, D.N, D.nKb * BKV);
  }
  return hipGetLastError();
}

}  // namespace sage
