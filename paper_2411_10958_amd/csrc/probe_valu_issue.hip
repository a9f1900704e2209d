// Hardware probe behind the vector-ALU ceiling of the attention kernel (not part of the library): how many core
// cycles a SIMD of gfx950 needs per wavefront instruction of the classes Algorithm 1's inner loop is made of, with
// 1, 2, 3 and 4 wavefronts resident per SIMD, each class alone and in the loop's own mix.
//
// One workgroup per CU (256 workgroups of 256 .. 1024 threads); every wavefront runs `iters` rounds of 16 independent
// instructions of one class (or the ten-instruction mix for two scores: 2 multiply-adds, 1 three-input maximum,
// 2 subtractions, 2 exponentials, 2 additions, 1 packed FP8 conversion).  The workgroup's time is taken between two
// barriers with the shader clock (s_memtime) by wavefront 0, so it covers the slowest wavefront; cycles per SIMD
// instruction = time / (instructions per wavefront * wavefronts per SIMD).  The figures are medians over the
// workgroups.  Every loop has a fixed trip count and touches no memory: nothing here can hang or fault.
#include <hip/hip_runtime.h>
#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

enum { ADD, SUB, MUL, FMA, FMAC, MAX3, EXP, CVT_FP8, MIX, NKIND };
static const char* NAMES[NKIND] = {"v_add_f32", "v_sub_f32", "v_mul_f32", "v_fma_f32", "v_fmac_f32", "v_max3_f32", "v_exp_f32",
                                   "v_cvt_pk_fp8_f32", "softmax mix (10 per 2 scores)"};

template <int KIND>
__global__ void __launch_bounds__(1024) k_issue(float* out, long long* ticks, int iters, float seed) {
  float x[16], y[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) { x[i] = seed + i + threadIdx.x * 0.001f; y[i] = 0.5f; }
  __syncthreads();
  const long long t0 = __builtin_amdgcn_s_memtime();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int j = (i + 1) & 15;
      if (KIND == ADD) asm volatile("v_add_f32 %0, %1, %0" : "+v"(y[i]) : "v"(x[i]));
      if (KIND == SUB) asm volatile("v_sub_f32 %0, %1, %2" : "=v"(y[i]) : "v"(x[i]), "v"(x[j]));
      if (KIND == MUL) asm volatile("v_mul_f32 %0, %1, %0" : "+v"(y[i]) : "v"(x[i]));
      if (KIND == FMA) asm volatile("v_fma_f32 %0, %1, %2, %0" : "+v"(y[i]) : "v"(x[i]), "v"(x[j]));
      if (KIND == FMAC) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(y[i]) : "v"(x[i]), "v"(x[j]));
      if (KIND == MAX3) asm volatile("v_max3_f32 %0, %1, %2, %0" : "+v"(y[i]) : "v"(x[i]), "v"(x[j]));
      if (KIND == EXP) asm volatile("v_exp_f32 %0, %1" : "=v"(y[i]) : "v"(x[i]));
      if (KIND == CVT_FP8) asm volatile("v_cvt_pk_fp8_f32 %0, %1, %2" : "+v"(y[i]) : "v"(x[i]), "v"(x[j]));
      if (KIND == MIX && i < 10) {
        if (i == 0 || i == 1) asm volatile("v_fmac_f32 %0, %1, %2" : "+v"(y[i]) : "v"(x[i]), "v"(x[j]));
        if (i == 2) asm volatile("v_max3_f32 %0, %1, %2, %0" : "+v"(y[i]) : "v"(x[i]), "v"(x[j]));
        if (i == 3 || i == 4) asm volatile("v_sub_f32 %0, %1, %2" : "=v"(y[i]) : "v"(x[i]), "v"(x[j]));
        if (i == 5 || i == 6) asm volatile("v_exp_f32 %0, %1" : "=v"(y[i]) : "v"(x[i]));
        if (i == 7 || i == 8) asm volatile("v_add_f32 %0, %1, %0" : "+v"(y[i]) : "v"(x[i]));
        if (i == 9) asm volatile("v_cvt_pk_fp8_f32 %0, %1, %2" : "+v"(y[i]) : "v"(x[i]), "v"(x[j]));
      }
    }
  }
  __syncthreads();
  const long long t1 = __builtin_amdgcn_s_memtime();
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) s += y[i] + x[i];
  out[(blockIdx.x * blockDim.x + threadIdx.x) & 0xffff] = s;
  if (threadIdx.x == 0) ticks[blockIdx.x] = t1 - t0;
}

static float* g_out;
static long long* g_ticks;

template <int KIND> double cycles(int threads) {
  const int iters = 20000, blocks = 256;
  k_issue<KIND><<<blocks, threads>>>(g_out, g_ticks, iters, 1.0f);     // clocks and caches
  k_issue<KIND><<<blocks, threads>>>(g_out, g_ticks, iters, 1.0f);
  CK(hipDeviceSynchronize());
  std::vector<long long> h(blocks);
  CK(hipMemcpy(h.data(), g_ticks, blocks * sizeof(long long), hipMemcpyDeviceToHost));
  std::sort(h.begin(), h.end());
  const double per_wave = iters * (KIND == MIX ? 10.0 : 16.0);
  return (double)h[blocks / 2] / (per_wave * (threads / 256));
}

int main() {
  CK(hipMalloc(&g_out, 65536 * sizeof(float)));
  CK(hipMalloc(&g_ticks, 256 * sizeof(long long)));
  printf("core cycles per wavefront instruction issued by one SIMD (median of 256 workgroups, one per CU)\n");
  printf("%-32s %10s %10s %10s %10s\n", "wavefronts per SIMD:", "1", "2", "3", "4");
  double mix[4] = {0, 0, 0, 0};
  for (int kind = 0; kind < NKIND; ++kind) {
    double c[4];
    for (int w = 1; w <= 4; ++w) {
      const int threads = 256 * w;
      switch (kind) {
        case ADD: c[w - 1] = cycles<ADD>(threads); break;
        case SUB: c[w - 1] = cycles<SUB>(threads); break;
        case MUL: c[w - 1] = cycles<MUL>(threads); break;
        case FMA: c[w - 1] = cycles<FMA>(threads); break;
        case FMAC: c[w - 1] = cycles<FMAC>(threads); break;
        case MAX3: c[w - 1] = cycles<MAX3>(threads); break;
        case EXP: c[w - 1] = cycles<EXP>(threads); break;
        case CVT_FP8: c[w - 1] = cycles<CVT_FP8>(threads); break;
        default: c[w - 1] = cycles<MIX>(threads); break;
      }
    }
    if (kind == MIX) for (int w = 0; w < 4; ++w) mix[w] = c[w];
    printf("%-32s %10.2f %10.2f %10.2f %10.2f\n", NAMES[kind], c[0], c[1], c[2], c[3]);
  }
  printf("ceiling of the loop's vector work (a wavefront instruction covers 64 lanes; 4 d operations per score; 1024 SIMDs, "
         "2.4 GHz):\n");
  for (int w = 1; w < 4; ++w)
    printf("  %d wavefronts per SIMD: %.1f cycles per 2 scores of 64 lanes -> %.0f TOP/s at d = 128\n", w + 1, 10.0 * mix[w],
           1024 * 2.4e9 * 128.0 / (10.0 * mix[w]) * 512.0 / 1e12);
  return 0;
}
