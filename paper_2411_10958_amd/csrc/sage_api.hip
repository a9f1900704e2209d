// C ABI of libsageattn (declared in include/sage_attn.h): argument validation, workspace map,
// kernel sequencing.  Host code only; no torch types.
#include "sage_attn.h"
#include "sage_common.h"

#include <cmath>

namespace {

using namespace sage;

int validate(const sage_attn_args* a, Dims* D, bool need_io) {
  if (!a) return SAGE_ERR_INVALID_ARG;
  if (a->B <= 0 || a->H <= 0 || a->H_kv <= 0 || a->N <= 0 || a->d <= 0) return SAGE_ERR_INVALID_ARG;
  if (a->H % a->H_kv != 0 || a->N_kv < 0) return SAGE_ERR_INVALID_ARG;
  // token indices and their tile arithmetic stay in 32-bit integers inside the kernels
  if (a->N > MAX_TOKENS || a->N_kv > MAX_TOKENS) return SAGE_ERR_UNSUPPORTED;
  const int Nk = a->N_kv > 0 ? a->N_kv : a->N;
  if (a->causal && Nk < a->N) return SAGE_ERR_UNSUPPORTED;
  if (a->d != 64 && a->d != 128 && a->d != 256) return SAGE_ERR_UNSUPPORTED;
  if (a->mode != SAGE_MODE_INT4_FP8 && a->mode != SAGE_MODE_INT8_FP8) return SAGE_ERR_UNSUPPORTED;
  if (a->dtype != SAGE_DT_FP16 && a->dtype != SAGE_DT_BF16) return SAGE_ERR_UNSUPPORTED;
  if ((a->flags & ~(SAGE_FLAG_SMOOTH_V | SAGE_FLAG_NO_SMOOTH_K | SAGE_FLAG_NO_SMOOTH_Q | SAGE_FLAG_FP32_DELTA_S | SAGE_FLAG_FP64_DELTA_S | SAGE_FLAG_DIGIT_DELTA_S)) != 0) return SAGE_ERR_UNSUPPORTED;
  if (a->group_map < SAGE_GROUPS_LANE || a->group_map > SAGE_GROUPS_TENSOR) return SAGE_ERR_UNSUPPORTED;
  if (a->layout != SAGE_LAYOUT_HND && a->layout != SAGE_LAYOUT_NHD) return SAGE_ERR_UNSUPPORTED;
  if (a->pv_format < SAGE_PV_E4M3 || a->pv_format > SAGE_PV_INT8) return SAGE_ERR_UNSUPPORTED;
  if (a->pv_format != SAGE_PV_E4M3 && (a->group_map == SAGE_GROUPS_FINE || a->group_map == SAGE_GROUPS_TOKEN))
    return SAGE_ERR_UNSUPPORTED;
  if (a->cu_seqlens_k && !a->cu_seqlens_q) return SAGE_ERR_INVALID_ARG;
  if (a->cu_seqlens_q && a->layout != SAGE_LAYOUT_NHD) return SAGE_ERR_UNSUPPORTED;
  if (need_io && (!a->q || !a->k || !a->v || !a->out)) return SAGE_ERR_INVALID_ARG;
  // statistics supplied by the producer of K and V: both arrays or neither, and only where mean(K) and
  // delta_V are all the statistics pass would have produced
  if ((a->k_mean_in != nullptr) != (a->v_scale_in != nullptr)) return SAGE_ERR_INVALID_ARG;
  if (a->k_mean_in && (a->flags & (SAGE_FLAG_SMOOTH_V | SAGE_FLAG_NO_SMOOTH_K)) != 0) return SAGE_ERR_UNSUPPORTED;
  if ((((uintptr_t)a->k_mean_in | (uintptr_t)a->v_scale_in) & 15u) != 0) return SAGE_ERR_INVALID_ARG;
  // the kernels move rows with 16-byte accesses (rows are multiples of 128 bytes, so the base decides)
  if ((((uintptr_t)a->q | (uintptr_t)a->k | (uintptr_t)a->v | (uintptr_t)a->out) & 15u) != 0) return SAGE_ERR_INVALID_ARG;
  if ((((uintptr_t)a->lse | (uintptr_t)a->cu_seqlens_q | (uintptr_t)a->cu_seqlens_k) & 3u) != 0) return SAGE_ERR_INVALID_ARG;
  // grid limits of the launches below (y dimension <= 65535, tile count fits an int)
  if ((long long)a->B * a->H > 65535) return SAGE_ERR_UNSUPPORTED;
  const long long nQb = (a->N + BQ - 1) / BQ, nKb = (Nk + BKV - 1) / BKV;
  if ((long long)a->B * a->H * nQb > (1LL << 30)) return SAGE_ERR_UNSUPPORTED;
  D->B = a->B; D->H = a->H; D->Hkv = a->H_kv; D->N = a->N; D->d = a->d;
  D->Nk = Nk;
  D->nQb = (int)nQb; D->nKb = (int)nKb;
  D->causal = a->causal != 0;
  D->int4 = a->mode == SAGE_MODE_INT4_FP8;
  D->bf16 = a->dtype == SAGE_DT_BF16;
  D->smooth_v = (a->flags & SAGE_FLAG_SMOOTH_V) != 0;
  D->smooth_k = (a->flags & SAGE_FLAG_NO_SMOOTH_K) == 0;
  D->smooth_q = (a->flags & SAGE_FLAG_NO_SMOOTH_Q) == 0;
  D->ds32 = (a->flags & SAGE_FLAG_FP32_DELTA_S) != 0;
  // Delta-S: digit products on the INT8 matrix unit, unless a key block meets at most 16 rows of block means (a decode
  // step, a short chunk): one chain of FP64 matrix instructions is then cheaper than cutting the keys into digits
  D->ds_mode = D->ds32 ? 1
             : (a->flags & SAGE_FLAG_FP64_DELTA_S) != 0 ? 2
             : (a->flags & SAGE_FLAG_DIGIT_DELTA_S) != 0 ? 0
             : ((long long)(D->H / D->Hkv) * D->nQb <= 16 ? 2 : 0);

  D->stats_given = a->k_mean_in != nullptr;
  D->tensor_groups = a->group_map == SAGE_GROUPS_TENSOR;
  D->block_groups = a->group_map == SAGE_GROUPS_BLOCK || D->tensor_groups;
  D->qg = (a->group_map == SAGE_GROUPS_FINE || a->group_map == SAGE_GROUPS_TOKEN) ? 1 : QGROUP;
  D->kg = a->group_map == SAGE_GROUPS_TOKEN ? 1 : (a->group_map == SAGE_GROUPS_FINE ? 4 : KGROUP);
  D->nhd = a->layout == SAGE_LAYOUT_NHD;
  D->seq.cu_q = a->cu_seqlens_q; D->seq.cu_k = a->cu_seqlens_k;
  D->want_lse = a->lse != nullptr;
  D->pvf = a->pv_format;        // SAGE_PV_* and PV_* share their values
  // key range split (kv_splits): only where few tiles would leave the chip idle, at least 8 key blocks per chunk
  if (a->kv_splits < 0 || a->kv_splits > 64) return SAGE_ERR_INVALID_ARG;
  D->splits = 1;
  D->pack = 0;
  if (D->kg == KGROUP && D->pvf == PV_E4M3 && a->kv_splits != 1) {
    // short queries on grouped KV heads: the 2..8 query heads of a KV head share one tile when all their queries fit it
    const int G = a->H / a->H_kv;
    D->pack = G >= 2 && G <= PACK_G && (long long)G * a->N <= BQ;     // (a->N: the longest sequence's queries)
    const long long tiles = D->pack ? (long long)a->B * a->H_kv : (long long)a->B * a->H * nQb;
    long long S = a->kv_splits > 1 ? a->kv_splits : (tiles < 256 ? (512 + tiles - 1) / tiles : 1);
    if (S > nKb / 8) S = nKb / 8;
    if (S > 64) S = 64;
    if (S >= 2) D->splits = (int)S;
  }
  const float sm = a->sm_scale > 0.0f ? a->sm_scale : (float)(1.0 / std::sqrt((double)a->d));
  D->kappa = sm * LOG2E;   // one FP32 rounding of the product of two FP32 values
  return SAGE_OK;
}

int check_workspace(const sage_attn_args* a, const Workspace& w) {
  if (!a->workspace || a->workspace_bytes < w.total) return SAGE_ERR_WORKSPACE;
  if (((uintptr_t)a->workspace & 255u) != 0) return SAGE_ERR_WORKSPACE;
  return SAGE_OK;
}

// Workspace pointers for `a`; mean(K) and delta_V point at the caller's arrays when it supplies them (the kernels
// only read them then).
Ptrs ptrs_for(const sage_attn_args* a, const Workspace& w) {
  Ptrs P = make_ptrs(a->q, a->k, a->v, a->out, a->workspace, w);
  if (a->k_mean_in) {
    P.k_mean = const_cast<float*>(a->k_mean_in);
    P.v_scale = const_cast<float*>(a->v_scale_in);
  }
  return P;
}

int hip_status(hipError_t e) {
  if (e == hipSuccess) return SAGE_OK;
  (void)hipGetLastError();
  return SAGE_ERR_HIP;
}

// Workspace of sage_attn_fwd_static: device memory that exists from the moment the library is loaded on a GPU, so
// the call itself allocates nothing.  Every GPU holds its own copy of the array at its own address; in host code the
// array's name is only a handle for hipGetSymbolAddress, the address kernels can use is what that call returns, taken
// once per device (with that device current) and kept in g_static_ws.
static __device__ __align__(256) unsigned char scratch[SAGE_STATIC_WORKSPACE_BYTES];
constexpr int MAX_DEVICES = 64;
void* g_static_ws[MAX_DEVICES] = {};

void* g_ws = nullptr;      // workspace of the convenience entry point
size_t g_ws_bytes = 0;
int g_ws_device = -1;      // the device it was allocated on

// Frees the convenience workspace on the device that owns it (after that device's work is done).
hipError_t release_ws() {
  if (!g_ws) return hipSuccess;
  int cur = -1;
  hipError_t e = hipGetDevice(&cur);
  if (e == hipSuccess && cur != g_ws_device) e = hipSetDevice(g_ws_device);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e == hipSuccess) e = hipFree(g_ws);
  if (cur >= 0 && cur != g_ws_device) (void)hipSetDevice(cur);
  g_ws = nullptr; g_ws_bytes = 0; g_ws_device = -1;
  return e;
}

}  // namespace

extern "C" {

size_t sage_attn_workspace_bytes(const sage_attn_args* args) {
  Dims D;
  if (validate(args, &D, false) != SAGE_OK) return 0;
  return make_workspace(D).total;
}

int sage_attn_kv_splits(const sage_attn_args* args) {
  Dims D;
  if (validate(args, &D, false) != SAGE_OK) return 0;
  return D.splits;
}

int sage_attn_prologue(const sage_attn_args* args) {
  Dims D;
  int st = validate(args, &D, true);
  if (st != SAGE_OK) return st;
  const Workspace w = make_workspace(D);
  if ((st = check_workspace(args, w)) != SAGE_OK) return st;
  const Ptrs P = ptrs_for(args, w);
  return hip_status(launch_prologue(D, P, (hipStream_t)args->stream));
}

int sage_attn_core(const sage_attn_args* args) {
  Dims D;
  int st = validate(args, &D, true);
  if (st != SAGE_OK) return st;
  const Workspace w = make_workspace(D);
  if ((st = check_workspace(args, w)) != SAGE_OK) return st;
  Ptrs P = ptrs_for(args, w);
  P.lse = args->lse;
  return hip_status(launch_attention(D, P, (hipStream_t)args->stream));
}

int sage_attn_fwd_ex(const sage_attn_args* args) {
  const int st = sage_attn_prologue(args);
  if (st != SAGE_OK) return st;
  return sage_attn_core(args);
}

int sage_attn_fwd(const void* q, const void* k, const void* v, void* out, int B, int H, int N, int d,
                  int causal, float sm_scale, int mode) {
  sage_attn_args a;
  a.q = q; a.k = k; a.v = v; a.out = out;
  a.B = B; a.H = H; a.H_kv = H; a.N = N; a.d = d;
  a.causal = causal; a.sm_scale = sm_scale; a.mode = mode; a.dtype = SAGE_DT_BF16; a.flags = 0; a.group_map = SAGE_GROUPS_LANE; a.N_kv = 0; a.layout = SAGE_LAYOUT_HND;
  a.cu_seqlens_q = nullptr; a.cu_seqlens_k = nullptr; a.lse = nullptr; a.pv_format = SAGE_PV_E4M3;
  a.k_mean_in = nullptr; a.v_scale_in = nullptr; a.kv_splits = 0;
  a.workspace = nullptr; a.workspace_bytes = 0; a.stream = nullptr;
  const size_t need = sage_attn_workspace_bytes(&a);
  if (need == 0) {
    Dims D;
    return validate(&a, &D, true);
  }
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return hip_status(hipErrorUnknown);
  if (need > g_ws_bytes || dev != g_ws_device) {     // grow, or follow the caller to another device
    if (release_ws() != hipSuccess) return hip_status(hipErrorUnknown);
    if (hipMalloc(&g_ws, need) != hipSuccess) { g_ws = nullptr; return hip_status(hipErrorOutOfMemory); }
    g_ws_bytes = need;
    g_ws_device = dev;
  }
  a.workspace = g_ws; a.workspace_bytes = g_ws_bytes;
  return sage_attn_fwd_ex(&a);
}

void sage_attn_release(void) { (void)release_ws(); }

int sage_attn_fwd_static(const sage_attn_args* args) {
  Dims D;
  int st = validate(args, &D, true);
  if (st != SAGE_OK) return st;
  const Workspace w = make_workspace(D);
  if (w.total > (size_t)SAGE_STATIC_WORKSPACE_BYTES) return SAGE_ERR_WORKSPACE;   // beyond the built-in workspace
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return hip_status(hipErrorUnknown);
  if (dev < 0 || dev >= MAX_DEVICES) return SAGE_ERR_UNSUPPORTED;
  if (!g_static_ws[dev]) {                  // first call on this device: where does its copy of the array live?
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return hip_status(hipErrorUnknown);
    g_static_ws[dev] = ptr;
  }
  // Nothing in the workspace has to start at zero (every kernel writes what a later one reads), so the contents
  // the previous call left behind need no clearing.
  sage_attn_args a = *args;
  a.workspace = g_static_ws[dev];
  a.workspace_bytes = (size_t)SAGE_STATIC_WORKSPACE_BYTES;
  Ptrs P = ptrs_for(&a, w);
  if ((st = hip_status(launch_prologue(D, P, (hipStream_t)a.stream))) != SAGE_OK) return st;
  P.lse = a.lse;
  return hip_status(launch_attention(D, P, (hipStream_t)a.stream));
}

int sage_attn_kv_stats(const sage_attn_args* args, float* k_mean_out, float* v_scale_out) {
  if (!k_mean_out || !v_scale_out) return SAGE_ERR_INVALID_ARG;
  if ((((uintptr_t)k_mean_out | (uintptr_t)v_scale_out) & 15u) != 0) return SAGE_ERR_INVALID_ARG;
  Dims D;
  int st = validate(args, &D, false);
  if (st != SAGE_OK) return st;
  if (!args->k || !args->v) return SAGE_ERR_INVALID_ARG;
  if (args->k_mean_in || (args->flags & (SAGE_FLAG_SMOOTH_V | SAGE_FLAG_NO_SMOOTH_K)) != 0) return SAGE_ERR_UNSUPPORTED;
  const Workspace w = make_workspace(D);
  if ((st = check_workspace(args, w)) != SAGE_OK) return st;
  Ptrs P = make_ptrs(args->q, args->k, args->v, args->out, args->workspace, w);
  P.k_mean = k_mean_out;
  P.v_scale = v_scale_out;
  return hip_status(launch_kv_stats(D, P, (hipStream_t)args->stream));
}

int sage_attn_kv_stats_update(const sage_attn_args* args, double* k_sum_state, float* v_absmax_state, long long n_before,
                              float* k_mean_out, float* v_scale_out) {
  if (!k_sum_state || !v_absmax_state || !k_mean_out || !v_scale_out || n_before < 0) return SAGE_ERR_INVALID_ARG;
  if ((((uintptr_t)k_mean_out | (uintptr_t)v_scale_out | (uintptr_t)v_absmax_state) & 15u) != 0 || ((uintptr_t)k_sum_state & 7u) != 0)
    return SAGE_ERR_INVALID_ARG;
  Dims D;
  int st = validate(args, &D, false);
  if (st != SAGE_OK) return st;
  if (!args->k || !args->v) return SAGE_ERR_INVALID_ARG;
  if (args->cu_seqlens_q || args->k_mean_in || (args->flags & (SAGE_FLAG_SMOOTH_V | SAGE_FLAG_NO_SMOOTH_K)) != 0)
    return SAGE_ERR_UNSUPPORTED;
  if (n_before + (long long)D.Nk > MAX_TOKENS) return SAGE_ERR_UNSUPPORTED;
  const Workspace w = make_workspace(D);
  if ((st = check_workspace(args, w)) != SAGE_OK) return st;
  Ptrs P = make_ptrs(args->q, args->k, args->v, args->out, args->workspace, w);
  P.k_mean = k_mean_out;
  P.v_scale = v_scale_out;
  return hip_status(launch_kv_stats_update(D, P, k_sum_state, v_absmax_state, n_before == 0, n_before + (long long)D.Nk,
                                           (hipStream_t)args->stream));
}

int sage_attn_quant(const sage_attn_args* args, const sage_quant_out* out) {
  if (!out) return SAGE_ERR_INVALID_ARG;
  Dims D;
  int st = validate(args, &D, false);
  if (st != SAGE_OK) return st;
  if (!args->q || !args->k || !args->v) return SAGE_ERR_INVALID_ARG;
  if (args->cu_seqlens_q) return SAGE_ERR_UNSUPPORTED;   // the plain copy-out layouts are fixed-length
  if ((long long)D.B * D.H * D.nQb > 65535) return SAGE_ERR_UNSUPPORTED;  // grid limit of the copy-out kernels
  const Workspace w = make_workspace(D);
  if ((st = check_workspace(args, w)) != SAGE_OK) return st;
  const Ptrs P = ptrs_for(args, w);
  if ((st = hip_status(launch_prologue(D, P, (hipStream_t)args->stream))) != SAGE_OK) return st;
  return hip_status(launch_unpack(D, P, out, (hipStream_t)args->stream));
}

int sage_attn_debug_qk(const sage_attn_args* args, int b, int h, int q_tile, int kv_block,
                       int32_t* out_acc) {
  Dims D;
  int st = validate(args, &D, false);
  if (st != SAGE_OK) return st;
  if (args->cu_seqlens_q) return SAGE_ERR_UNSUPPORTED;
  if (!out_acc || b < 0 || b >= D.B || h < 0 || h >= D.H || q_tile < 0 || q_tile >= D.nQb ||
      kv_block < 0 || kv_block >= D.nKb)
    return SAGE_ERR_INVALID_ARG;
  const Workspace w = make_workspace(D);
  if ((st = check_workspace(args, w)) != SAGE_OK) return st;
  const Ptrs P = ptrs_for(args, w);
  return hip_status(launch_debug_qk(D, P, b, h, q_tile, kv_block, out_acc, (hipStream_t)args->stream));
}

int sage_attn_debug_mfma_fp8(const uint8_t* a_codes, const uint8_t* b_codes, const float* c_in,
                             float* d_out, void* stream) {
  if (!a_codes || !b_codes || !c_in || !d_out) return SAGE_ERR_INVALID_ARG;
  return hip_status(launch_debug_mfma_fp8(a_codes, b_codes, c_in, d_out, (hipStream_t)stream));
}

const char* sage_status_string(int status) {
  switch (status) {
    case SAGE_OK: return "ok";
    case SAGE_ERR_INVALID_ARG: return "invalid argument";
    case SAGE_ERR_UNSUPPORTED: return "unsupported head dimension, mode, dtype or size";
    case SAGE_ERR_WORKSPACE: return "workspace missing, too small or misaligned";
    case SAGE_ERR_HIP: return "HIP call or kernel launch failed";
    default: return "unknown status";
  }
}

}  // extern "C"
