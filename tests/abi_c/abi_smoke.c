/* A caller of the C ABI that knows nothing of Python or torch: plain C, device memory from the HIP
 * runtime, the convenience entry point sage_attn_fwd (bf16, H_kv = H) and the explicit-workspace form
 * sage_attn_fwd_ex.  The outputs are checked against softmax(Q K^T / sqrt(d)) V evaluated in double on
 * the host (the definition of Sec. 2.1; quantized attention is close to it, not equal: the bar here is a
 * cosine of 0.99 in the 8-bit mode and 0.9 in the 4-bit mode on these well-conditioned inputs), and the two
 * entry points against each other bit for bit.  Built by paper_2411_10958_amd/build.py, run by
 * tests/test_gpu_c_abi.py.  Exit status 0 = passed. */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sage_attn.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
  fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, hipGetErrorString(e_)); return 2; } } while (0)

static uint16_t f32_to_bf16(float x) {
  uint32_t u; memcpy(&u, &x, 4);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
static float bf16_to_f32(uint16_t h) { uint32_t u = (uint32_t)h << 16; float x; memcpy(&x, &u, 4); return x; }

/* a small deterministic generator: roughly normal values from sums of uniforms */
static uint32_t lcg_state = 12345u;
static float next_value(void) {
  float s = 0.0f;
  for (int i = 0; i < 4; ++i) { lcg_state = lcg_state * 1664525u + 1013904223u; s += (float)(lcg_state >> 8) / 16777216.0f; }
  return (s - 2.0f) * 1.7320508f;
}

int main(void) {
  const int B = 1, H = 2, N = 200, d = 64;           /* a ragged last tile on purpose */
  const size_t n = (size_t)B * H * N * d;
  uint16_t *hq = malloc(n * 2), *hk = malloc(n * 2), *hv = malloc(n * 2), *ho = malloc(n * 2), *ho2 = malloc(n * 2);
  if (!hq || !hk || !hv || !ho || !ho2) return 2;
  for (size_t i = 0; i < n; ++i) {
    hq[i] = f32_to_bf16(next_value());
    hk[i] = f32_to_bf16(next_value() + 0.5f * (float)((i % d) % 7));   /* a per-channel offset in K */
    hv[i] = f32_to_bf16(next_value());
  }
  void *dq, *dk, *dv, *dout;
  CHECK_HIP(hipMalloc(&dq, n * 2)); CHECK_HIP(hipMalloc(&dk, n * 2));
  CHECK_HIP(hipMalloc(&dv, n * 2)); CHECK_HIP(hipMalloc(&dout, n * 2));
  CHECK_HIP(hipMemcpy(dq, hq, n * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dk, hk, n * 2, hipMemcpyHostToDevice));
  CHECK_HIP(hipMemcpy(dv, hv, n * 2, hipMemcpyHostToDevice));

  int failures = 0;
  for (int mode = 0; mode < 2; ++mode) {
    for (int causal = 0; causal < 2; ++causal) {
      CHECK_HIP(hipMemset(dout, 0xff, n * 2));
      int st = sage_attn_fwd(dq, dk, dv, dout, B, H, N, d, causal, 0.0f, mode);
      if (st != SAGE_OK) { fprintf(stderr, "sage_attn_fwd: %s\n", sage_status_string(st)); return 1; }
      CHECK_HIP(hipDeviceSynchronize());
      CHECK_HIP(hipMemcpy(ho, dout, n * 2, hipMemcpyDeviceToHost));

      /* the same call through the explicit form with a workspace of the caller */
      sage_attn_args a;
      memset(&a, 0, sizeof a);
      a.q = dq; a.k = dk; a.v = dv; a.out = dout;
      a.B = B; a.H = H; a.H_kv = H; a.N = N; a.d = d;
      a.causal = causal; a.mode = mode; a.dtype = SAGE_DT_BF16;
      a.workspace_bytes = sage_attn_workspace_bytes(&a);
      if (a.workspace_bytes == 0) { fprintf(stderr, "workspace size 0\n"); return 1; }
      CHECK_HIP(hipMalloc(&a.workspace, a.workspace_bytes));
      CHECK_HIP(hipMemset(dout, 0xff, n * 2));
      st = sage_attn_fwd_ex(&a);
      if (st != SAGE_OK) { fprintf(stderr, "sage_attn_fwd_ex: %s\n", sage_status_string(st)); return 1; }
      CHECK_HIP(hipDeviceSynchronize());
      CHECK_HIP(hipMemcpy(ho2, dout, n * 2, hipMemcpyDeviceToHost));
      CHECK_HIP(hipFree(a.workspace));
      if (memcmp(ho, ho2, n * 2) != 0) { fprintf(stderr, "the two entry points disagree\n"); ++failures; }

      /* the definition, in double */
      double dot = 0.0, nn = 0.0, mm = 0.0;
      int finite = 1;
      double* p = malloc((size_t)N * sizeof(double));
      for (int h = 0; h < H; ++h) {
        for (int r = 0; r < N; ++r) {
          const int last = causal ? r : N - 1;
          double mx = -1e300, sum = 0.0;
          for (int t = 0; t <= last; ++t) {
            double s = 0.0;
            for (int c = 0; c < d; ++c)
              s += (double)bf16_to_f32(hq[((size_t)h * N + r) * d + c]) * (double)bf16_to_f32(hk[((size_t)h * N + t) * d + c]);
            p[t] = s / sqrt((double)d);
            if (p[t] > mx) mx = p[t];
          }
          for (int t = 0; t <= last; ++t) { p[t] = exp(p[t] - mx); sum += p[t]; }
          for (int c = 0; c < d; ++c) {
            double o = 0.0;
            for (int t = 0; t <= last; ++t) o += p[t] * (double)bf16_to_f32(hv[((size_t)h * N + t) * d + c]);
            o /= sum;
            const double g = (double)bf16_to_f32(ho[((size_t)h * N + r) * d + c]);
            if (!isfinite(g)) finite = 0;
            dot += o * g; nn += o * o; mm += g * g;
          }
        }
      }
      free(p);
      const double cosv = dot / sqrt(nn * mm);
      const double bar = mode == SAGE_MODE_INT8_FP8 ? 0.99 : 0.9;
      printf("mode %d causal %d: cosine against the definition %.5f (bar %.2f)\n", mode, causal, cosv, bar);
      if (!finite || !(cosv >= bar)) ++failures;
    }
  }
  /* argument errors come back as status codes, not as faults */
  if (sage_attn_fwd(dq, dk, dv, dout, B, H, N, 96, 0, 0.0f, 0) != SAGE_ERR_UNSUPPORTED) { fprintf(stderr, "d = 96 accepted\n"); ++failures; }
  if (sage_attn_fwd(NULL, dk, dv, dout, B, H, N, d, 0, 0.0f, 0) != SAGE_ERR_INVALID_ARG) { fprintf(stderr, "null q accepted\n"); ++failures; }
  sage_attn_release();
  CHECK_HIP(hipFree(dq)); CHECK_HIP(hipFree(dk)); CHECK_HIP(hipFree(dv)); CHECK_HIP(hipFree(dout));
  free(hq); free(hk); free(hv); free(ho); free(ho2);
  printf(failures ? "FAILED\n" : "abi smoke ok\n");
  return failures ? 1 : 0;
}
