/*
 * sage_attn.h - C ABI of the gfx950 (MI355X) quantized attention forward pass.
 *
 * The library computes O = softmax(Q K^T * sm_scale) V per (batch, head) the way
 * SageAttention2 (arXiv 2411.10958) does: K is smoothed by its per-channel token mean and Q
 * by its per-block mean with the Delta-S bias added back (Sec. 3.1, Eq. 2), Q and K are
 * quantized to INT4 (or INT8) codes with one scale per fine-grained token group (Sec. 3.2),
 * P~ and V are quantized to FP8 E4M3 (Sec. 3.3) and P~V is accumulated in two levels
 * (Sec. 3.4); the whole loop is Algorithm 1.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers owned by the caller, 16-byte aligned; the library never
 *     frees or keeps them.  q and out are contiguous [B, H, N, d] (or [B, N, H, d], see layout); k and v are contiguous
 *     [B, H_kv, N_kv, d]; elements are 16-bit (fp16 or bf16, see dtype).  Query head h reads KV
 *     head h / (H / H_kv).  N_kv = N unless sage_attn_args.N_kv says otherwise; a causal mask is
 *     aligned to the last query and key (key t visible to query r iff t <= r + N_kv - N) and
 *     needs N_kv >= N.
 *   - Variable-length batches: with cu_seqlens_q set, the B sequences are packed along the token
 *     axis, q and out are [total_q, H, d], k and v [total_k, H_kv, d] (layout must be
 *     SAGE_LAYOUT_NHD), sequence b owns query tokens cu_seqlens_q[b] .. cu_seqlens_q[b+1]-1 and
 *     key tokens cu_seqlens_k[b] .. cu_seqlens_k[b+1]-1, and N / N_kv are the LONGEST query / key
 *     length (they size the launch and the workspace; a longer sequence is cut to them).  Every
 *     sequence is smoothed, quantized and attended on its own, exactly as a batch of one (bit for bit when
 *     kv_splits is the same in both calls: left to the library it depends on the call's tile count).  The
 *     prefix sums live on the device and are not checked on the host: under a causal mask a
 *     sequence with fewer keys than queries is masked as if aligned to the first query and key,
 *     and a sequence without keys gets zeros.
 *   - d is 64, 128 or 256; mode and dtype take the enum values below; H must be a multiple of H_kv.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream)
 *     and the call returns without synchronising.  Kernels of one call are ordered on that
 *     stream; two calls that share a workspace must be ordered by the caller.
 *   - Every function returns a status (0 = SAGE_OK).  Argument errors are found on the host
 *     before anything is launched; nothing throws or aborts.
 *   - Numerical edge cases are defined, not errors: an all-zero quantization group has scale 0
 *     and codes 0; N need not be a multiple of any tile (padded keys are masked, padded
 *     queries are not written); N >= 1.
 */
#ifndef SAGE_ATTN_H
#define SAGE_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  SAGE_OK = 0,
  SAGE_ERR_INVALID_ARG = -1,  /* null or misaligned pointer, non-positive size, H % H_kv != 0 */
  SAGE_ERR_UNSUPPORTED = -2,  /* d not in {64,128,256}, unknown mode, dtype, flag, group map or layout, causal with N_kv < N,
                                 cu_seqlens without SAGE_LAYOUT_NHD, sage_attn_quant / sage_attn_debug_qk with cu_seqlens */
  SAGE_ERR_WORKSPACE = -3,    /* workspace missing or smaller than sage_attn_workspace_bytes() */
  SAGE_ERR_HIP = -4           /* a HIP call or launch failed (the HIP error is cleared) */
};

/* SageAttn2-4b: INT4 Q,K (Q and K smoothed); SageAttn2-8b: INT8 Q,K (only K smoothed).
   Both use FP8 E4M3 P~ and V (paper, table "Two kernel implementations"). */
enum { SAGE_MODE_INT4_FP8 = 0, SAGE_MODE_INT8_FP8 = 1 };
enum { SAGE_DT_FP16 = 0, SAGE_DT_BF16 = 1 };
/* Optional techniques, or-ed into sage_attn_args.flags.
   SAGE_FLAG_SMOOTH_V: the optional "smooth V" of Sec. 3.4 (last paragraph; Appendix "Smoothing V"):
   the per-channel token mean of V is subtracted before the FP8 quantizer and added back, in FP32, to
   the output (rows of the softmax sum to 1).  Costs one more pass over V in the preprocessing.
   SAGE_FLAG_NO_SMOOTH_K / SAGE_FLAG_NO_SMOOTH_Q switch off the smoothing of K (Eq. 2) or of Q (Sec. 3.1)
   for the rows "none" and "only K" of the paper's smoothing ablation: the corresponding mean is taken
   as zero (k_mean, q_mean and, without Q smoothing, delta_s hold zeros; no Delta-S product is computed).
   They change accuracy only, not the kernels.  The 8-bit mode never smooths Q, so NO_SMOOTH_Q changes
   nothing there.
   SAGE_FLAG_FP32_DELTA_S: Delta-S (Sec. 3.1) accumulated in FP32 on the matrix unit instead of FP64.  The
   preprocessing gets faster (the FP64 product is a quarter of it at N = 4096 and most of it at long
   sequences); Delta-S is then within (d + 2) 2^-24 kappa sum_c |q_bar_c gamma(K)_c| of the exact value
   instead of correctly rounded.  That is far below the quantization noise of the method, but it moves
   the last bits of the scores, so once in about 10^5 scores the FP8 code of P~ comes out one step away
   from what the exact Delta-S gives.  Off by default; ignored by the 8-bit mode.
   SAGE_FLAG_FP64_DELTA_S / SAGE_FLAG_DIGIT_DELTA_S: which exact form of the Delta-S product runs.  "Digit": both
   factors are cut into 7-bit fixed-point digits (42 bits below each row's largest magnitude) and multiplied exactly on
   the INT8 matrix unit (30 of the 36 digit pairs); "FP64": the FP64 matrix instruction.  Both agree with the float64
   inner product to the last bit of the FP32 result (the tests allow one value in 10^3 to differ by that bit).  With neither flag the library picks: digits, except when a key
   block meets at most 16 block means ((H / H_kv) ceil(N / 128) <= 16), where one chain of FP64 instructions is cheaper.
   Ignored by the 8-bit mode; FP32 wins over both, FP64 over digit. */
enum { SAGE_FLAG_SMOOTH_V = 1, SAGE_FLAG_NO_SMOOTH_K = 2, SAGE_FLAG_NO_SMOOTH_Q = 4, SAGE_FLAG_FP32_DELTA_S = 8,
       SAGE_FLAG_FP64_DELTA_S = 16, SAGE_FLAG_DIGIT_DELTA_S = 32 };
/* Quantization granularity of Q and K (Sec. 3.2; the ablation of the paper's granularity table).
   SAGE_GROUPS_LANE: the default, the gfx950 counterpart of per-thread quantization (SAGE_Q_GROUP /
   SAGE_K_GROUP below).  SAGE_GROUPS_BLOCK: one scale per 128-query block and per 64-key block
   (per-block quantization, the granularity of SageAttention-1, Sec. 2.3); same kernels, same speed,
   lower accuracy.  q_scale / k_scale keep their shapes (values repeat inside a block).
   SAGE_GROUPS_FINE: one scale per query and per run of 4 keys - the finest groups that still cost
   one dequantization factor per accumulator quad on gfx950 (a lane of the score MFMA owns one query,
   and its 16 accumulators are 4 runs of 4 consecutive keys): nearly free.  SAGE_GROUPS_TOKEN: one
   scale per query and per key (per-token quantization, Sec. 3.2): a factor per score, not free.
   SAGE_GROUPS_TENSOR: one scale for all queries and one for all keys of a (batch, head) (per-tensor
   quantization, Sec. 2.2): the quantizers run twice (block maxima, then codes), the attention kernel is
   that of LANE; the coarsest and least accurate map of the comparison.
   Queries / keys per entry of q_scale / k_scale: 2 / 16 (LANE, BLOCK, TENSOR), 1 / 4 (FINE), 1 / 1 (TOKEN). */
enum { SAGE_GROUPS_LANE = 0, SAGE_GROUPS_BLOCK = 1, SAGE_GROUPS_FINE = 2, SAGE_GROUPS_TOKEN = 3,
       SAGE_GROUPS_TENSOR = 4 };
/* 8-bit data type of P~ and V (Sec. 3.3; the paper's data-type comparison): E4M3 (the paper's choice,
   static scale 1/448 for P~), E5M2 (static scale 1/57344; one mantissa bit less) or INT8 (static scale
   1/127, V per channel with max|V|/127, integer product converted and added to O in FP32 per block:
   slower and, for long rows, less accurate).  The last two are kept for the comparison; not with
   SAGE_GROUPS_FINE / _TOKEN. */
enum { SAGE_PV_E4M3 = 0, SAGE_PV_E5M2 = 1, SAGE_PV_INT8 = 2 };
/* Memory order of the four tensors (all contiguous): heads outside tokens, [B, H, N, d], or tokens
   outside heads, [B, N, H, d] (k, v: H_kv and N_kv).  The workspace layouts do not depend on it. */
enum { SAGE_LAYOUT_HND = 0, SAGE_LAYOUT_NHD = 1 };

/* Numerical block sizes of Algorithm 1 as this library fixes them. */
#define SAGE_BQ_SMOOTH 128 /* tokens per Q smoothing block (b_q) */
#define SAGE_BKV_ACC 64    /* keys per level-1 accumulation block (b_kv, Sec. 3.4) */
/* Quantization groups (Sec. 3.2 redefined for the gfx950 MFMA accumulator layout: the
   tokens whose products land in one lane): queries {2n, 2n+1}; keys in runs of 16. */
#define SAGE_Q_GROUP 2
#define SAGE_K_GROUP 16

typedef struct sage_attn_args {
  const void* q;          /* device, [B, H, N, d] */
  const void* k;          /* device, [B, H_kv, N_kv, d] */
  const void* v;          /* device, [B, H_kv, N_kv, d] */
  void* out;              /* device, [B, H, N, d], written */
  int B, H, H_kv, N, d;   /* d = 64, 128 or 256; H a multiple of H_kv; N and N_kv <= 2^24; B * H <= 65535 */
  int causal;             /* 0: every key visible; 1: key t visible to query r iff t <= r + N_kv - N */
  float sm_scale;         /* <= 0 means 1/sqrt(d) */
  int mode;               /* SAGE_MODE_* */
  int dtype;              /* SAGE_DT_* : type of q, k, v and out */
  int flags;              /* SAGE_FLAG_* or-ed together; 0 = the paper's default configuration */
  int group_map;          /* SAGE_GROUPS_*; 0 = the default */
  int N_kv;               /* keys / values per head (cross attention, chunked prefill); 0 = N */
  int layout;             /* SAGE_LAYOUT_*: memory order of q, k, v and out; 0 = [B, H, N, d] */
  void* workspace;        /* device scratch of >= sage_attn_workspace_bytes(); 256-byte aligned */
  size_t workspace_bytes;
  void* stream;           /* hipStream_t, NULL = default stream */
  const int* cu_seqlens_q; /* device, [B + 1] prefix sums of the query lengths, or NULL: fixed length N */
  const int* cu_seqlens_k; /* device, [B + 1] prefix sums of the key lengths; NULL = cu_seqlens_q */
  float* lse;             /* device, written if not NULL: [B, H, N] f32 (whatever the layout of q), or [H, total_q]
                             for a variable-length batch.  Natural-log-sum-exp over the visible keys of
                             sm_scale * <q_r, k_t> as the quantized path evaluates these scores: the final
                             running maximum and sum of Algorithm 1 plus the row constant <q_r, mean(K)> that
                             smoothing K removes from every score of a row (Sec. 3.1).  It is the weight needed
                             to merge results computed over disjoint key sets: out = sum_i exp(lse_i - lse) out_i,
                             lse = ln sum_i exp(lse_i).  -inf for a sequence without keys. */
  int pv_format;          /* SAGE_PV_*; 0 = E4M3 */
  const float* k_mean_in;  /* device, [B, H_kv, d] f32, or NULL.  With k_mean_in and v_scale_in the statistics pass over K
                              and V is skipped (K and V are then read once by the preprocessing instead of twice): the
                              producer of K and V - a projection or rotary-embedding kernel, or the keeper of a KV cache -
                              supplies them.  k_mean_in[c] = fl32(sum over the N_kv tokens of K[., c] / N_kv), the sum
                              exact (Eq. 2); 16-byte aligned.  Both or neither; not with SAGE_FLAG_SMOOTH_V or
                              SAGE_FLAG_NO_SMOOTH_K.  sage_attn_kv_stats computes exactly these two arrays. */
  const float* v_scale_in; /* device, [B, H_kv, d] f32, or NULL: fl32(max over tokens |V[., c]| / 448) (Sec. 3.3; / 57344 for
                              SAGE_PV_E5M2, / 127 for SAGE_PV_INT8) */
  int kv_splits;           /* Workgroups per 128-query tile in the attention kernel, each walking its own chunk of the key
                              blocks and leaving (m, l, O) under its own running maximum; a second kernel merges the
                              chunks by the rule that combines consecutive blocks in Eq. 1 (Sec. 2.1).  For calls with
                              few query tiles and many keys - a decode step, a short chunk of queries against a long
                              cache - where one workgroup per tile would leave most of the chip idle.  0: the library
                              decides (it splits when there are fewer than 256 tiles; sage_attn_kv_splits tells);
                              1: never; 2..64: this many (cut to one chunk per 8 key blocks at most).  Default groups
                              (SAGE_GROUPS_LANE, _BLOCK, _TENSOR) and SAGE_PV_E4M3 only, else 1.
                              With 2..8 query heads per KV head whose queries all fit one tile (N * H / H_kv <= 128,
                              N the longest sequence's) and kv_splits != 1, a tile is a KV head: its query heads share the tile's 128
                              columns, so the KV head's codes are walked once for the group (tiles = B * H_kv; also when
                              the chunk count comes out as 1).  Same arithmetic per query, same chunk rule.
                              Chunks of a tile: with nblk its key blocks (those up to its last query's last visible key
                              under a causal mask), n_vis the leading ones in which its FIRST query sees a key (all of
                              them without a mask) and C = ceil(n_vis / S), chunk s covers blocks [s C, (s + 1) C), the
                              last non-empty one runs on to nblk.  The result is Algorithm 1 on every chunk, merged; it
                              differs from the unsplit result where the 8-bit codes of P~ depend on the running
                              maximum, not beyond the accuracy of either. */
} sage_attn_args;

/* Bytes of device scratch one call needs for these shapes (codes, scales, means, Delta-S, partial results of a
   split key range).  Depends on the shapes, mode, options and kv_splits, not on pointers.  Returns 0 if those are invalid. */
size_t sage_attn_workspace_bytes(const sage_attn_args* args);

/* The number of key chunks per query tile sage_attn_fwd_ex / sage_attn_core will use for these arguments (see
   kv_splits); 0 if the arguments are invalid. */
int sage_attn_kv_splits(const sage_attn_args* args);

/* The whole forward pass of Algorithm 1: preprocessing (smoothing, Delta-S, quantization;
   Sec. 3.1-3.3) followed by the fused attention kernel (inner loop and epilogue). */
int sage_attn_fwd_ex(const sage_attn_args* args);

/* The two halves of sage_attn_fwd_ex, for timing them apart the way the paper's kernel
   benchmark does (Appendix "Kernel Benchmark Setup" times the attention kernel on already
   quantized operands).  sage_attn_core reads what sage_attn_prologue left in the workspace
   for the same args; q, k, v are not touched by it. */
int sage_attn_prologue(const sage_attn_args* args);
int sage_attn_core(const sage_attn_args* args);

/* Convenience form named by the problem statement (Sec. 2.1: O = softmax(QK^T/sqrt(d))V):
   bf16 tensors, H_kv = H, default stream, and a workspace the library allocates lazily with
   hipMalloc on the current device, grows when needed (or when the current device changed) and keeps until
   sage_attn_release().  Not thread-safe. */
int sage_attn_fwd(const void* q, const void* k, const void* v, void* out, int B, int H, int N,
                  int d, int causal, float sm_scale, int mode);
void sage_attn_release(void);

/* For callers that cannot allocate device memory or have it allocated on their behalf: code running under HIP
   graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same forward pass as
   sage_attn_fwd_ex, with the workspace taken from a fixed array of SAGE_STATIC_WORKSPACE_BYTES that is part of
   the library's device image (every GPU the library is used on holds its own copy from the first call on it
   until the process ends): the call makes no hipMalloc / hipFree and no other allocating call, and ignores
   args->workspace / workspace_bytes.  q, k, v, out (and lse, cu_seqlens_*, k_mean_in, v_scale_in) are the
   caller's, as everywhere.  Shapes whose sage_attn_workspace_bytes() exceeds SAGE_STATIC_WORKSPACE_BYTES are
   refused with SAGE_ERR_WORKSPACE before anything is launched; more than 64 devices: SAGE_ERR_UNSUPPORTED.
   All calls on one GPU share that GPU's array: calls that overlap there (two streams, two threads) race, and
   the caller must order them; nothing in it has to be cleared between calls. */
#define SAGE_STATIC_WORKSPACE_BYTES (64u << 20)
int sage_attn_fwd_static(const sage_attn_args* args);

/* Output of the preprocessing stage in plain ("logical") layouts, for checking it bit by bit.
   All pointers are device buffers the caller allocates; a NULL member is skipped.
     q_codes [B,H,N,d] int8       codes of gamma(Q) (int4 mode) or Q (int8 mode), Sec. 3.2
     k_codes [B,H_kv,N_kv,d] int8    codes of gamma(K)
     v_codes [B,H_kv,N_kv,d] uint8   E4M3 (or E5M2 / two's-complement INT8, see pv_format) codes of V / delta_V, Sec. 3.3
     q_scale [B,H,ceil(N/2)] f32  delta_Q per query group ([B,H,N] with SAGE_GROUPS_FINE / _TOKEN)
     k_scale [B,H_kv,ceil(N_kv/16)] f32   (ceil(N_kv/4) with SAGE_GROUPS_FINE, N_kv with SAGE_GROUPS_TOKEN)
     v_scale [B,H_kv,d] f32       delta_V per channel
     k_mean  [B,H_kv,d] f32       mean(K) over tokens (Eq. 2)
     q_mean  [B,H,ceil(N/128),d] f32   block means of Q (int4 mode only, else untouched)
     delta_s [B,H,ceil(N/128),N_kv] f32   kappa * <q_mean_i, gamma(K)_t>, kappa = sm_scale*log2(e)
                                       (int4 mode only, else untouched).  With causal = 1 the
                                       entries no query can use are skipped in groups: row i is
                                       defined for keys t < 4096 * (floor(i/32) + 1) + N_kv - N, the rest of the
                                       row is left as it was
     v_mean  [B,H_kv,d] f32       mean(V) over tokens (SAGE_FLAG_SMOOTH_V only, else untouched); with
                                  that flag v_codes and v_scale describe V - v_mean */
typedef struct sage_quant_out {
  int8_t* q_codes;
  int8_t* k_codes;
  uint8_t* v_codes;
  float* q_scale;
  float* k_scale;
  float* v_scale;
  float* k_mean;
  float* q_mean;
  float* delta_s;
  float* v_mean;
} sage_quant_out;

/* The statistics pass of the preprocessing alone (Algorithm 1, "Preprocessing": mean(K) and the scale of
   psi_V): writes k_mean_out and v_scale_out, device [B, H_kv, d] f32 each, in the form k_mean_in / v_scale_in
   take.  Reads k and v only (q and out may be NULL); needs the workspace of sage_attn_workspace_bytes(args). */
int sage_attn_kv_stats(const sage_attn_args* args, float* k_mean_out, float* v_scale_out);

/* The same statistics kept as running state of a K / V that grows (a KV cache): args->k, args->v hold only the NEW
   tokens, [B, H_kv, N_kv, d] (N_kv = the chunk's length; q, out may be NULL), n_before is the number of tokens already
   accumulated (0: the state is initialised from this chunk).  k_sum_state [B, H_kv, d] f64 (exact column sums of
   K, Eq. 2) and v_absmax_state [B, H_kv, d] f32 (column maxima of |V|, Sec. 3.3) are read and updated; k_mean_out and
   v_scale_out, [B, H_kv, d] f32, receive mean(K) and delta_V of all n_before + N_kv tokens in the form k_mean_in /
   v_scale_in take.  The sums are exact, so any split into chunks gives bit for bit what sage_attn_kv_stats gives on
   the whole.  With it the keeper of a cache reads old keys and values once per attention call (in the quantizers)
   instead of twice.  Fixed-length batches only; not with SAGE_FLAG_SMOOTH_V / SAGE_FLAG_NO_SMOOTH_K; needs the
   workspace of sage_attn_workspace_bytes(args); n_before + N_kv <= 2^24. */
int sage_attn_kv_stats_update(const sage_attn_args* args, double* k_sum_state, float* v_absmax_state, long long n_before,
                              float* k_mean_out, float* v_scale_out);

/* Runs the preprocessing of Algorithm 1 (as sage_attn_prologue) and then copies its results
   out of the kernel-private packed workspace layout into `out`. */
int sage_attn_quant(const sage_attn_args* args, const sage_quant_out* out);

/* Integer accumulators of the score product (Algorithm 1, Matmul(Q^_i, K^_j^T)) for one
   128-query tile and one 64-key block, through the same MFMA device code as the attention
   kernel.  Needs a workspace filled by sage_attn_prologue / sage_attn_quant for `args`.
   out_acc: device, [128][64] int32, row = query 128*q_tile + r, column = key 64*kv_block + t
   (positions beyond N hold products of zero codes). */
int sage_attn_debug_qk(const sage_attn_args* args, int b, int h, int q_tile, int kv_block,
                       int32_t* out_acc);

/* Hardware check behind the accumulation design (the probe of Sec. 3.4, "FP32 MMA Buffer for FP22
   Accumulator", run on gfx950): executes ONE v_mfma_f32_32x32x64_f8f6f4, D = A*B + C, the
   instruction the P~V product uses (K = 64 = one accumulation block).
     a_codes, b_codes: device, [64 lanes][32] E4M3 bytes; lane l of A holds row l%32, k = 32*(l/32) + byte;
                       lane l of B holds column l%32, same k.
     c_in, d_out:      device, [64 lanes][16] float; element v of lane l is row 8*(v/4) + 4*(l/32) + v%4,
                       column l%32. */
int sage_attn_debug_mfma_fp8(const uint8_t* a_codes, const uint8_t* b_codes, const float* c_in,
                             float* d_out, void* stream);

const char* sage_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* SAGE_ATTN_H */
