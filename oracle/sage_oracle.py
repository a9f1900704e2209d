"""CPU oracle for the SageAttention2 quantized attention forward pass.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference the GPU kernels are
checked against.  It is imported by tests/, by the smoke check and by the benchmark's
CPU-baseline leg and by nothing else; the product path never calls it and it shares no
code with the HIP sources.

It follows the paper's Algorithm 1 ("Implementation of SageAttention2") step by step,
with the smoothing of Sec. 3.1 (Eq. 2 and the Delta-S decomposition), the group quantizer
of Sec. 2.2 / Sec. 3.2 / Appendix "Per-Thread Quantization Formulation", the FP8 E4M3
quantization of Sec. 3.3 and the two-level accumulation of Sec. 3.4.  The plain
definition of attention (Sec. 2.1, first formula) is `ref_attn_fp64`.

Precision rules (the readings this repository takes where the paper is silent):
  * inputs are fp16/bf16 values widened exactly; all "FP32" quantities are rounded once
    from a float64 evaluation of the stated real-valued expression;
  * means use an exact token sum (float64), one division, one rounding to FP32;
  * scales are delta = fl32(max|x| / qmax); codes = clip(rint(fl32(x / delta)));
    an all-zero group has delta = 0 and codes 0;
  * softmax is evaluated in base 2: scores are multiplied by kappa = fl32(sm_scale*log2 e)
    and 2**x replaces e**x, which leaves softmax unchanged;  the score of one (query, key)
    pair is the single FP32 rounding of  acc * c + D  with c = fl32(fl32(dQ*dK) * kappa)
    and D = fl32(kappa * <qbar_i, gamma(K)_t>)  (inner product in float64);
  * the inner loop is evaluated in the order Algorithm 1 prints it, one FP32 rounding per line:
    P~ = fl32(2**fl32(S - m)), l = fl32(fl32(alpha * l) + rowsum(P~)) on the unquantized P~, then
    P^ = E4M3(fl32(P~ * 448)), saturating at 448 (`attention_rows`, the oracle of record);
    `attention_rows_kernel_order` is a second, separately named form with the roundings where the
    gfx950 kernel has them (static scale folded into the exponent), pinned against the first;
  * the per-block product R = P^ V^ is the exact sum of the FP8 products rounded once to
    FP32 (an ideal FP32 buffer), then O = fl32(fl32(alpha*O) + R).
Parity pins for every function here live in tests/test_oracle_pins.py.
"""
import numpy as np

LOG2E_F32 = np.float32(1.4426950408889634)
E4M3_MAX = 448.0
LOG2_448_F32 = np.float32(np.log2(448.0))
BQ_SMOOTH = 128   # tokens per Q smoothing block (Algorithm 1's b_q)
BKV_ACC = 64      # keys per level-1 accumulation block (Algorithm 1's b_kv)

f32 = np.float32
f64 = np.float64


# --------------------------------------------------------------------------- FP8 E4M3
def e4m3_decode(codes):
    """OCP FP8 E4M3 ("fn": no infinities, 0x7f/0xff are NaN) byte codes -> float64."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    s = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 3) & 0xF
    m = c & 0x7
    sub = np.ldexp(m.astype(f64), -9)                      # exponent field 0: m * 2^-9
    nor = np.ldexp(1.0 + m.astype(f64) / 8.0, e - 7)       # (1 + m/8) * 2^(e-7)
    v = np.where(e == 0, sub, nor)
    v = np.where((e == 15) & (m == 7), np.nan, v)
    return s * v


def e4m3_encode(x):
    """Round-to-nearest-even, saturating (|x| > 448 -> +-448) encoder to E4M3 byte codes.

    Sec. 3.3 only says values are cast to E4M3 with range [-448, 448]; nearest-even and
    saturation are this repository's reading.
    """
    x = np.asarray(x, dtype=f64)
    sign = np.signbit(x)
    a = np.minimum(np.abs(x), E4M3_MAX)
    # spacing of representable values around a: 2^(floor(log2 a) - 3), at least 2^-9
    _, ex = np.frexp(a)                        # a = mant * 2^ex, mant in [0.5, 1)
    e_unb = np.maximum(ex - 1, -6)             # exponent of the binade, subnormals share -6
    step = np.ldexp(1.0, e_unb - 3)
    q = np.rint(a / step)                      # numpy rint = ties to even; a/step is exact
    v = q * step                               # may round up into the next binade (exact)
    v = np.minimum(v, E4M3_MAX)
    # re-derive the fields from the rounded value
    _, ex2 = np.frexp(v)
    e_unb2 = np.maximum(ex2 - 1, -6)
    is_sub = v < 2.0 ** -6
    mant = np.where(is_sub, np.rint(v * 2.0 ** 9), np.rint((v / np.ldexp(1.0, e_unb2) - 1.0) * 8.0))
    efield = np.where(is_sub, 0, e_unb2 + 7)
    code = (efield.astype(np.int64) << 3) | mant.astype(np.int64)
    code = np.where(v == 0, 0, code)
    code = code | np.where(sign, 0x80, 0)
    return code.astype(np.uint8)


# --------------------------------------------------------------------------- FP8 E5M2
# The other 8-bit float the paper weighs for P~ and V (Sec. 3.3 and the data-type table: E4M3 is
# chosen because it is the more accurate one); kept as a variant so that the comparison can be made.
E5M2_MAX = 57344.0
LOG2_57344_F32 = np.float32(np.log2(57344.0))


def e5m2_decode(codes):
    """OCP FP8 E5M2 byte codes (IEEE-like: exponent field 31 is inf / NaN) -> float64."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    s = np.where(c & 0x80, -1.0, 1.0)
    e = (c >> 2) & 0x1F
    m = c & 0x3
    sub = np.ldexp(m.astype(f64), -16)                     # exponent field 0: m * 2^-16
    nor = np.ldexp(1.0 + m.astype(f64) / 4.0, e - 15)
    v = np.where(e == 0, sub, nor)
    v = np.where(e == 31, np.where(m == 0, np.inf, np.nan), v)
    return s * v


def e5m2_encode(x):
    """Round-to-nearest-even, saturating (|x| > 57344 -> +-57344) encoder to E5M2 byte codes."""
    x = np.asarray(x, dtype=f64)
    sign = np.signbit(x)
    a = np.minimum(np.abs(x), E5M2_MAX)
    _, ex = np.frexp(a)
    e_unb = np.maximum(ex - 1, -14)            # subnormals share the exponent -14
    step = np.ldexp(1.0, e_unb - 2)            # 2 mantissa bits
    v = np.minimum(np.rint(a / step) * step, E5M2_MAX)
    _, ex2 = np.frexp(v)
    e_unb2 = np.maximum(ex2 - 1, -14)
    is_sub = v < 2.0 ** -14
    mant = np.where(is_sub, np.rint(v * 2.0 ** 16), np.rint((v / np.ldexp(1.0, e_unb2) - 1.0) * 4.0))
    efield = np.where(is_sub, 0, e_unb2 + 15)
    code = (efield.astype(np.int64) << 2) | mant.astype(np.int64)
    code = np.where(v == 0, 0, code)
    code = code | np.where(sign, 0x80, 0)
    return code.astype(np.uint8)


# INT8 for P~ and V, the third data type of the paper's comparison for the P~V product: P~ in [0, 1] with
# the static scale 1/127, V per channel with max|V|/127, round-half-even, integer product.
INT8_MAX = 127.0
LOG2_127_F32 = np.float32(np.log2(127.0))


def int8_encode(x):
    return np.clip(np.rint(np.asarray(x, dtype=f64)), -INT8_MAX, INT8_MAX).astype(np.int8)


def int8_decode(codes):
    return np.asarray(codes, dtype=np.int8).astype(f64)


# name -> (largest code magnitude, its log2 in FP32, encoder, decoder)
_FP8 = {"e4m3": (E4M3_MAX, LOG2_448_F32, e4m3_encode, e4m3_decode),
        "e5m2": (E5M2_MAX, LOG2_57344_F32, e5m2_encode, e5m2_decode),
        "int8": (INT8_MAX, LOG2_127_F32, int8_encode, int8_decode)}


# --------------------------------------------------------------------------- group maps
def group_map(name, N, which):
    """Token -> quantization-group index, for `which` in {"q", "k"}.

    "g950":  the groups of this repository's gfx950 kernels - the tokens whose products
             land in one lane's accumulator registers (the per-thread principle of
             Sec. 3.2): queries {2n, 2n+1}; keys in runs of 16.
    "nv_m16n8": the paper's own grouping for mma.m16n8k64 with b_q=128, c_w=4, b_k=64
             (Appendix "Per-Thread Quantization Formulation", last two paragraphs):
             within a warp's 32 queries, tokens i, 8+i, 16+i, 24+i; within a 64-key block,
             keys congruent to {2i, 2i+1} modulo 8.
    "per_token", "per_block" (128 queries / 64 keys), "per_tensor": the granularities the
             paper compares against (Sec. 2.2, Sec. 2.3, Sec. 3.2).
    "fine":  every query on its own, keys in runs of 4: finer than "g950", still one scale per
             accumulator quad of a gfx950 lane.
    """
    n = np.arange(N)
    if name == "g950":
        return n // 2 if which == "q" else n // 16
    if name == "nv_m16n8":
        if which == "q":
            return (n // 32) * 8 + (n % 8)
        return (n // 64) * 4 + (n % 8) // 2
    if name == "fine":
        return n if which == "q" else n // 4
    if name == "per_token":
        return n
    if name == "per_block":
        return n // (BQ_SMOOTH if which == "q" else BKV_ACC)
    if name == "per_tensor":
        return np.zeros(N, dtype=np.int64)
    raise ValueError(name)


# --------------------------------------------------------------------------- smoothing
def token_mean(X):
    """Mean over the token axis (axis 0) of an [n, d] float32 array: exact sum in float64,
    one division, one rounding to FP32 (Sec. 3.1, text under Eq. 2)."""
    X = np.asarray(X, dtype=f64)
    return (X.sum(axis=0) / X.shape[0]).astype(f32)


def smooth_k(K):
    """gamma(K) = K - mean(K) over all tokens of the head (Eq. 2; Algorithm 1 preprocessing)."""
    kbar = token_mean(K)
    gK = (np.asarray(K, f64) - kbar.astype(f64)).astype(f32)
    return kbar, gK


def smooth_q(Q, bq=BQ_SMOOTH):
    """gamma(Q_i) = Q_i - mean(Q_i) per block of bq tokens (Eq. 2; Algorithm 1, first line
    of the outer loop).  A ragged last block averages its valid tokens."""
    N, d = Q.shape
    nblk = (N + bq - 1) // bq
    qbar = np.zeros((nblk, d), f32)
    gQ = np.empty((N, d), f32)
    for i in range(nblk):
        blk = slice(i * bq, min((i + 1) * bq, N))
        qbar[i] = token_mean(Q[blk])
        gQ[blk] = (np.asarray(Q[blk], f64) - qbar[i].astype(f64)).astype(f32)
    return qbar, gQ


def delta_s(qbar, gK, kappa):
    """D[i, t] = fl32(kappa * <qbar_i, gamma(K)_t>): the Delta-S bias of Sec. 3.1 (the
    "GEMV" of Algorithm 1's score line), already multiplied by kappa = sm_scale * log2 e."""
    acc = qbar.astype(f64) @ gK.astype(f64).T
    return (f64(kappa) * acc).astype(f32)


# --------------------------------------------------------------------------- quantizers
def quantize_groups(X, groups, qmax):
    """psi of Sec. 2.2 applied per quantization group of tokens (Sec. 3.2, Appendix
    Eq. "per_thread_quant"): delta_g = max over the group's tokens and all channels of |x|,
    divided by qmax; codes = round-to-nearest-even(x / delta_g), clipped to [-qmax, qmax].

    X: [N, d] float32;  groups: [N] ints.  Returns (delta [n_groups] float32, codes [N, d] int8).
    """
    X = np.asarray(X, f32)
    groups = np.asarray(groups)
    ng = int(groups.max()) + 1
    row_max = np.abs(X).max(axis=1)
    gmax = np.zeros(ng, f32)
    np.maximum.at(gmax, groups, row_max)
    delta = (gmax / f32(qmax)).astype(f32)                 # IEEE FP32 division
    drow = delta[groups][:, None]
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = (X / drow).astype(f32)                     # IEEE FP32 division
    ratio = np.where(drow > 0, ratio, f32(0))
    codes = np.clip(np.rint(ratio), -qmax, qmax).astype(np.int8 if qmax <= 127 else np.int32)
    return delta, codes


def quantize_v(V, pv_fmt="e4m3"):
    """Per-channel FP8 quantization of V (Sec. 3.3; Algorithm 1 preprocessing):
    delta_V[c] = max_n |V[n, c]| / 448, codes = E4M3(V / delta_V)  (57344 and E5M2 for the variant)."""
    fmax, _, enc, _ = _FP8[pv_fmt]
    V = np.asarray(V, f32)
    delta = (np.abs(V).max(axis=0) / f32(fmax)).astype(f32)
    with np.errstate(divide="ignore", invalid="ignore"):
        ratio = (V / delta[None, :]).astype(f32)
    ratio = np.where(delta[None, :] > 0, ratio, f32(0))
    return delta, enc(ratio)


# --------------------------------------------------------------------------- prologue
def quantize_head(Q, K, V, mode="int4_fp8", sm_scale=None, gmap="g950", bq=BQ_SMOOTH,
                  smooth_q_on=None, smooth_k_on=True, pv_exact=False, ds_blocks=None,
                  smooth_v_on=False, pv_fmt="e4m3"):
    """Everything Algorithm 1 computes before the inner loop, for one (batch, head).

    Q: [N, d], K and V: [N_kv, d] float32 holding exactly representable 16-bit values (N_kv = N in
    Algorithm 1; other key lengths - cross attention, chunked prefill - change nothing in it).
    mode "int4_fp8": Q and K smoothed, INT4 range [-7, 7] (SageAttn2-4b);
    mode "int8_fp8": only K smoothed, INT8 range [-127, 127] (SageAttn2-8b, Table
    "Two kernel implementations").  An integer `mode` is used as qmax directly, smooth_*_on
    override the mode and pv_exact keeps P~ and V unquantized: all three exist only so the
    pins can take the quantizers to their high-precision limit.  ds_blocks, if given, lists
    the smoothing blocks whose Delta-S rows are wanted (the other rows are left zero): sampling
    support for sequences where the full [N/b_q, N] bias would not fit in host memory.
    smooth_v_on: the optional technique at the end of Sec. 3.4 (Appendix "Smoothing V"): the
    token mean of V is subtracted per channel before the FP8 quantization and added back to the
    output (rows of the softmax sum to 1); the mean is kept in FP32.
    """
    N, d = Q.shape
    Nk = K.shape[0]
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    qmax = {"int4_fp8": 7, "int8_fp8": 127}[mode] if isinstance(mode, str) else int(mode)
    if smooth_q_on is None:
        smooth_q_on = (mode == "int4_fp8")
    kappa = f32(f32(sm_scale) * LOG2E_F32)
    if smooth_k_on:
        kbar, gK = smooth_k(K)
    else:
        kbar, gK = np.zeros(d, f32), np.asarray(K, f32)
    if smooth_q_on:
        qbar, gQ = smooth_q(Q, bq)
        if ds_blocks is None:
            D = delta_s(qbar, gK, kappa)
        else:
            D = np.zeros((qbar.shape[0], Nk), f32)
            D[list(ds_blocks)] = delta_s(qbar[list(ds_blocks)], gK, kappa)
    else:
        qbar, gQ, D = None, np.asarray(Q, f32), None
    # The 4-bit variant's score line always carries the Delta-S addend (zeros when Q is left unsmoothed for the
    # smoothing ablation); the 8-bit variant's has none (table "Two kernel implementations").
    ds_step = bool(smooth_q_on) or mode == "int4_fp8"
    gq, gk = group_map(gmap, N, "q"), group_map(gmap, Nk, "k")
    dq, qc = quantize_groups(gQ, gq, qmax)
    dk, kc = quantize_groups(gK, gk, qmax)
    if smooth_v_on:
        vbar = token_mean(V)
        V = (np.asarray(V, f32) - vbar[None, :]).astype(f32)
    else:
        vbar = None
    if pv_exact:
        dv, vc, vdec = np.ones(d, f32), None, np.asarray(V, f64)
    else:
        dv, vc = quantize_v(V, pv_fmt)
        vdec = _FP8[pv_fmt][3](vc)                        # [N, d] float64, exact
    return dict(N=N, Nk=Nk, d=d, kappa=kappa, qmax=qmax, kbar=kbar, qbar=qbar, delta_s=D, Q=np.asarray(Q, f32),
                pv_fmt=pv_fmt,
                ds_step=ds_step, q_codes=qc, q_scale=dq, q_groups=gq, k_codes=kc, k_scale=dk, k_groups=gk,
                v_codes=vc, v_scale=dv, v_dec=vdec, pv_exact=pv_exact, bq=bq, vbar=vbar)


# --------------------------------------------------------------------------- attention
def _exp2_f32(x):
    """2**x evaluated in float64 and rounded to FP32 (2**-inf = 0)."""
    with np.errstate(under="ignore"):
        return np.exp2(np.asarray(x, f64)).astype(f32)


def int_scores(q_codes, k_codes):
    """acc[r, t] = sum_c Qhat[r, c] * Khat[t, c] as exact integers (the integer Matmul of
    Algorithm 1's score line).  A float64 matmul is exact here: |acc| <= 127^2 * d << 2^53."""
    return np.rint(q_codes.astype(f64) @ k_codes.astype(f64).T).astype(np.int64)


def _row_setup(pro, rows, causal, bkv):
    """What both forms of the inner loop share before their first block: the rows' codes and scales, the
    smoothing block they lie in, and the number of key blocks they walk."""
    N, Nk = pro["N"], pro["Nk"]
    coff = Nk - N
    assert not causal or coff >= 0, "a causal mask needs N_kv >= N"
    rows = np.arange(N)[rows]
    blk = int(rows[0]) // pro["bq"]
    assert int(rows[-1]) // pro["bq"] == blk, "rows must lie in one smoothing block"
    last_key = int(rows[-1]) + coff if causal else Nk - 1
    return rows, blk, coff, last_key // bkv + 1


def _block_scores(pro, rows, blk, coff, causal, j, bkv):
    """Score line of Algorithm 1 for key block j: S = psi^-1(Qhat Khat^T) + Delta-S, in base 2.
    Returns (ks, s, S): the block's key indices, the unrounded float64 value acc * c (+ D) and its single
    FP32 rounding with masked positions at -inf."""
    ks = np.arange(j * bkv, min((j + 1) * bkv, pro["Nk"]))
    acc = int_scores(pro["q_codes"][rows], pro["k_codes"][ks])
    dq = pro["q_scale"][pro["q_groups"][rows]]
    dk = pro["k_scale"][pro["k_groups"][ks]]
    c = ((dq[:, None] * dk[None, :]).astype(f32) * pro["kappa"]).astype(f32)
    s = acc.astype(f64) * c.astype(f64)
    if pro["delta_s"] is not None:
        s = s + pro["delta_s"][blk, ks].astype(f64)[None, :]
    S = s.astype(f32)                                     # one rounding of acc*c + D
    if causal:
        S = np.where(ks[None, :] > rows[:, None] + coff, f32(-np.inf), S)
    return ks, s, S


def _epilogue(pro, O, l, fmax, out_dtype):
    """Last line of Algorithm 1: O / l / 448 * delta_V (+ mean(V) with the smooth-V option), rounded to the
    output type.  fmax is the static scale still to be divided out (1 when l already carries it)."""
    out = (O / l[:, None]).astype(f32)
    if fmax != 1.0:
        out = (out / f32(fmax)).astype(f32)
    out = (out * pro["v_scale"][None, :]).astype(f32)
    if pro.get("vbar") is not None:                       # smooth V: O = O + mean(V)
        out = (out + pro["vbar"][None, :]).astype(f32)
    return _round_out(out, out_dtype)


def attention_rows(pro, rows, causal, bkv=BKV_ACC, out_dtype="bf16", return_state=False, p_codes=None,
                   return_codes=False, blocks=None):
    """THE ORACLE OF RECORD for the inner loop + epilogue of Algorithm 1, evaluated in the order the
    algorithm prints its lines, every line rounded once to FP32:

        S    = psi^-1(Matmul(Qhat_i, Khat_j^T)) + Delta-S_ij            (one rounding of acc * c + D)
        m_ij = max(m_i,j-1, rowmax(S))
        P~   = exp(S - m_ij)                                           (base 2: kappa carries log2 e)
        l_ij = exp(m_i,j-1 - m_ij) * l_i,j-1 + rowsum(P~)              (the unquantized P~)
        P^   = (P~ * 448).to(FP8 E4M3)                                 (Sec. 3.3 static scale)
        O_ij = diag(exp(m_i,j-1 - m_ij)) O_i,j-1 + Matmul(P^, V^_j)    (Sec. 3.4: block product exact,
                                                                        rounded once; then the FP32 sum)
        O_i  = diag(l)^-1 O / 448 * delta_V

    for the query rows `rows` (a slice or index array inside ONE smoothing block) of a head prepared by
    `quantize_head`.  Returns the [len(rows), d] output rounded to out_dtype (as float32).  With N_kv != N
    a causal mask is aligned to the last query and key: query r sees keys t <= r + (N_kv - N).

    blocks: optional (j0, j1): walk only the key blocks j0 <= j < j1 (a chunk of a split key range; the state
    returned is then that chunk's, see `merge_key_chunks`).
    p_codes: optional uint8 / int8 array [len(rows), n_blocks * bkv]: 8-bit codes to use for P^ INSTEAD of
    the ones this function would compute (everything else - m, P~, l - as printed).  It exists so that a test
    can show that a deviating result is explained by nothing but the codes of P^ (a floating-point value
    decides an integer there).  return_codes: also return the codes of P^ that were used, same shape.
    """
    rows, blk, coff, n_blocks = _row_setup(pro, rows, causal, bkv)
    d = pro["d"]
    vdec = pro["v_dec"]
    nr = len(rows)
    fmax, _, enc, dec = _FP8[pro["pv_fmt"]]               # static scale of P~: 1/448 (Sec. 3.3)
    m = np.full(nr, -np.inf, f32)
    l = np.zeros(nr, f32)
    O = np.zeros((nr, d), f32)
    codes = np.zeros((nr, n_blocks * bkv), np.uint8)
    for j in range(n_blocks) if blocks is None else range(blocks[0], min(blocks[1], n_blocks)):
        ks, _, S = _block_scores(pro, rows, blk, coff, causal, j, bkv)
        m_new = np.maximum(m, S.max(axis=1))
        with np.errstate(invalid="ignore"):
            P = _exp2_f32((S - m_new[:, None]).astype(f32))
            alpha = _exp2_f32((m - m_new).astype(f32))
        l = ((alpha * l).astype(f32).astype(f64) + P.astype(f64).sum(axis=1)).astype(f32)
        if pro["pv_exact"]:
            Phat = (P * f32(fmax)).astype(f32).astype(f64)
        else:
            if p_codes is None:
                cj = enc((P * f32(fmax)).astype(f32)).view(np.uint8)
            else:
                cj = np.asarray(p_codes)[:, j * bkv: j * bkv + len(ks)].view(np.uint8)
            codes[:, j * bkv: j * bkv + len(ks)] = cj
            Phat = dec(cj.view(np.int8) if pro["pv_fmt"] == "int8" else cj)
        R = (Phat @ vdec[ks]).astype(f32)                 # exact block sum, one rounding
        O = ((alpha[:, None] * O).astype(f32) + R).astype(f32)
        m = m_new
    res = _epilogue(pro, O, l, fmax, out_dtype)
    ret = (res,)
    if return_state:
        ret += (dict(m=m, e=m, l=l, O=O),)                # e: the exponent offset l is summed under (here m itself)
    if return_codes:
        ret += (codes,)
    return ret if len(ret) > 1 else res


def attention_rows_kernel_order(pro, rows, causal, bkv=BKV_ACC, out_dtype="bf16", return_state=False,
                                return_codes=False, return_e=False, blocks=None):
    """NOT the oracle of record: the same inner loop with the FP32 roundings placed where the gfx950 kernel
    places them.  Mathematically it is Algorithm 1 line for line; it differs from `attention_rows` in three
    rounding decisions, each of which tests/test_oracle_pins.py compares with the printed form:

      * the static scale 448 of P~ (Sec. 3.3) is folded into the exponent: E = 448 P~ = 2^(S - e) with the
        offset e = fl32(m' - fl32(log2 448)), one exponential and no multiplication; l and O are carried as
        sums of E (448 l, 448 O), so the epilogue divides O by l only;
      * before the subtraction m is nudged upward, m' = fl32(m + 2^-22 |m|) (one fused multiply-add), so that the
        row's largest E stays <= 448 whatever way e rounds - P~ is thereby scaled by 2^-(2^-22 |m|), which
        cancels in O / l - and the running sums are rescaled by 2^(e_old - e_new);
      * the 8-bit variant (no Delta-S addend in its score line) forms the exponent's argument acc * c - e with
        one rounding (a fused multiply-add) while the running maximum is that of the rounded products.

    The GPU tests compare the kernel with this function at a tolerance that only leaves room for the
    hardware's exponential, summation order and reciprocal, and with `attention_rows` at the stated bar.
    return_e: also return the unrounded-to-8-bit values E [len(rows), n_blocks * bkv] (float32).
    """
    rows, blk, coff, n_blocks = _row_setup(pro, rows, causal, bkv)
    d = pro["d"]
    vdec = pro["v_dec"]
    nr = len(rows)
    fmax, log2_fmax, enc, dec = _FP8[pro["pv_fmt"]]
    m = np.full(nr, -np.inf, f32)
    e = np.full(nr, -np.inf, f32)                         # exponent offset of the running sums: E = 2^(S - e)
    l = np.zeros(nr, f32)                                 # fmax * (running sum of P~)
    O = np.zeros((nr, d), f32)
    codes = np.zeros((nr, n_blocks * bkv), np.uint8)
    Eall = np.zeros((nr, n_blocks * bkv), f32)
    for j in range(n_blocks) if blocks is None else range(blocks[0], min(blocks[1], n_blocks)):
        ks, s, S = _block_scores(pro, rows, blk, coff, causal, j, bkv)
        m_new = np.maximum(m, S.max(axis=1))
        with np.errstate(invalid="ignore"):
            t = np.where(np.isfinite(m_new), (np.abs(m_new).astype(f64) * 2.0 ** -22 + m_new.astype(f64)).astype(f32), m_new)
        e_new = (t - log2_fmax).astype(f32)
        with np.errstate(invalid="ignore"):
            if pro["ds_step"]:
                arg = (S - e_new[:, None]).astype(f32)    # the rounded score, then the subtraction
            else:
                arg = np.where(np.isneginf(S), f32(-np.inf), (s - e_new[:, None].astype(f64)).astype(f32))
            E = _exp2_f32(arg)                            # E = fmax * P~
            alpha = _exp2_f32((e - e_new).astype(f32))    # rescales what was summed under the previous offset
        l = ((alpha * l).astype(f32).astype(f64) + E.astype(f64).sum(axis=1)).astype(f32)
        if pro["pv_exact"]:
            Phat = E.astype(f64)
        else:
            cj = enc(E).view(np.uint8)
            codes[:, j * bkv: j * bkv + len(ks)] = cj
            Phat = dec(cj.view(np.int8) if pro["pv_fmt"] == "int8" else cj)
        Eall[:, j * bkv: j * bkv + len(ks)] = E
        R = (Phat @ vdec[ks]).astype(f32)
        O = ((alpha[:, None] * O).astype(f32) + R).astype(f32)
        m, e = m_new, e_new
    res = _epilogue(pro, O, l, 1.0, out_dtype)            # O and l both carry the factor fmax
    ret = (res,)
    if return_state:
        ret += (dict(m=m, e=e, l=l, O=O),)
    if return_codes:
        ret += (codes,)
    if return_e:
        ret += (Eall,)
    return ret if len(ret) > 1 else res


def key_chunks(pro, first_row, last_row, causal, splits, bkv=BKV_ACC):
    """The chunks [(j0, j1), ...] into which the key blocks of a query tile (rows first_row .. last_row) are split
    for `splits` workgroups: every chunk must start with a block in which every query of the tile sees a key,
    so the n_vis leading blocks visible to the tile's first query are divided evenly, C = ceil(n_vis / splits)
    each, and the last non-empty chunk runs on to the tile's last block."""
    coff = pro["Nk"] - pro["N"]
    nblk = (pro["Nk"] + bkv - 1) // bkv
    n_vis = nblk
    if causal:
        nblk = min(nblk, (last_row + coff) // bkv + 1)
        n_vis = min(nblk, (first_row + coff) // bkv + 1)
    C = (n_vis + splits - 1) // splits
    used = (n_vis + C - 1) // C
    return [(s * C, nblk if s + 1 >= used else (s + 1) * C) for s in range(used)]


def merge_key_chunks(pro, states, form, out_dtype="bf16"):
    """Online softmax over disjoint key sets (Sec. 2.1, Eq. 1 applied to chunks instead of consecutive blocks):
    each state holds a chunk's final (e, l, O) - the sums l = sum 2^(S - e) and O under the chunk's own exponent
    offset e.  Under the largest offset e* the sums add up with weights 2^(e_s - e*); then Algorithm 1's last
    line.  Evaluated in float64 from the FP32 states, one rounding to FP32 before the output cast.
    Returns (output rows, merged state)."""
    e = np.stack([st["e"].astype(f64) for st in states])              # [S, rows]
    e_max = e.max(axis=0)
    with np.errstate(invalid="ignore"):
        w = np.where(np.isneginf(e), 0.0, np.exp2(e - e_max[None, :]))
    l = sum(w[s] * st["l"].astype(f64) for s, st in enumerate(states))
    O = sum(w[s][:, None] * st["O"].astype(f64) for s, st in enumerate(states))
    fmax = 1.0 if form == "kernel" else _FP8[pro["pv_fmt"]][0]        # the kernel-order sums carry the static scale
    out = (O / l[:, None] / fmax * pro["v_scale"].astype(f64)[None, :]).astype(f32)
    if pro.get("vbar") is not None:
        out = (out.astype(f64) + pro["vbar"].astype(f64)[None, :]).astype(f32)
    return _round_out(out, out_dtype), dict(m=np.max(np.stack([st["m"] for st in states]), axis=0), e=e_max.astype(f32),
                                            l=l.astype(f32), O=O.astype(f32))


def row_lse(pro, rows, state):
    """Natural-log-sum-exp of the scores sm_scale * <q_r, k_t> over the visible keys, as the quantized
    path evaluates them: from the final exponent offset e the sum l is carried under (the running maximum of
    Algorithm 1 in `attention_rows`; the maximum minus log2 448 in `attention_rows_kernel_order`), in base 2
    sum_t 2^S_t = l * 2^e, plus the one row constant the smoothing of K drops from every score of a row
    (Sec. 3.1: <q_r, mean(K)>, invisible to the softmax but part of the sum's scale):
        lse_r = ln 2 * (e_r + log2(l_r) + kappa * <q_r, mean(K)>),
    evaluated in float64 from the FP32 state and rounded once to FP32.  This is what lets partial
    results over disjoint key sets be merged (weights exp(lse_part - lse_total))."""
    rows = np.arange(pro["N"])[rows]
    e, l = state["e"].astype(f64), state["l"].astype(f64)
    corr = f64(pro["kappa"]) * (pro["Q"][rows].astype(f64) @ pro["kbar"].astype(f64))
    with np.errstate(divide="ignore"):
        return (np.log(2.0) * (e + np.log2(l) + corr)).astype(f32)


def _round_out(x, dtype):
    if dtype == "fp16":
        return x.astype(np.float16).astype(f32)
    if dtype == "bf16":
        u = np.ascontiguousarray(x, f32).view(np.uint32).astype(np.uint64)
        u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
        return u.astype(np.uint32).view(f32).reshape(x.shape)
    if dtype == "fp32":
        return x
    raise ValueError(dtype)


FORMS = {"printed": attention_rows, "kernel": attention_rows_kernel_order}


def sage_attention_head(Q, K, V, causal=False, mode="int4_fp8", sm_scale=None, gmap="g950",
                        bq=BQ_SMOOTH, bkv=BKV_ACC, out_dtype="bf16", q_blocks=None, want_lse=False,
                        form="printed", **kw):
    """Algorithm 1 for one (batch, head); `q_blocks` restricts the outer loop to some
    smoothing blocks (rows of the others are left zero).  With want_lse the prologue dict also
    carries "lse" [N] (see row_lse).  form: "printed" (`attention_rows`, the oracle of record) or "kernel"
    (`attention_rows_kernel_order`)."""
    attention_rows = FORMS[form]
    pro = quantize_head(Q, K, V, mode, sm_scale, gmap, bq, **kw)
    N, d = Q.shape
    out = np.zeros((N, d), f32)
    lse = np.zeros(N, f32)
    nblk = (N + bq - 1) // bq
    for i in (range(nblk) if q_blocks is None else q_blocks):
        rows = slice(i * bq, min((i + 1) * bq, N))
        if want_lse:
            out[rows], st = attention_rows(pro, rows, causal, bkv, out_dtype, return_state=True)
            lse[rows] = row_lse(pro, rows, st)
        else:
            out[rows] = attention_rows(pro, rows, causal, bkv, out_dtype)
    if want_lse:
        pro["lse"] = lse
    return out, pro


def sage_attention(q, k, v, causal=False, mode="int4_fp8", sm_scale=None, gmap="g950",
                   bq=BQ_SMOOTH, bkv=BKV_ACC, out_dtype="bf16", form="printed", **kw):
    """Batched form: q [B, H, N, d], k and v [B, H_kv, N, d]; query head h reads KV head
    h // (H / H_kv).  Returns [B, H, N, d] float32 (values rounded to out_dtype)."""
    B, H, N, d = q.shape
    g = H // k.shape[1]
    out = np.empty((B, H, N, d), f32)
    for b in range(B):
        for h in range(H):
            out[b, h], _ = sage_attention_head(q[b, h], k[b, h // g], v[b, h // g], causal, mode,
                                               sm_scale, gmap, bq, bkv, out_dtype, form=form, **kw)
    return out


# --------------------------------------------------------------------------- definition
def ref_lse_fp64(Q, K, causal=False, sm_scale=None, rows=None):
    """ln sum_t exp(sm_scale * <q_r, k_t>) over the visible keys, float64, one head (the
    normaliser of the softmax in Sec. 2.1, first formula)."""
    Q, K = np.asarray(Q, f64), np.asarray(K, f64)
    N, Nk = Q.shape[0], K.shape[0]
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(Q.shape[1])
    ridx = np.arange(N) if rows is None else np.arange(N)[rows]
    S = (Q[ridx] @ K.T) * sm_scale
    if causal:
        S = np.where(np.arange(Nk)[None, :] > ridx[:, None] + (Nk - N), -np.inf, S)
    mx = S.max(axis=1)
    return mx + np.log(np.exp(S - mx[:, None]).sum(axis=1))



def ref_attn_fp64(Q, K, V, causal=False, sm_scale=None, rows=None):
    """softmax(Q K^T * sm_scale) V in float64 (Sec. 2.1, first formula), one head;
    `rows` restricts the queries.  K, V may have another length than Q; the causal mask is then
    aligned to the last query and key."""
    Q, K, V = (np.asarray(x, f64) for x in (Q, K, V))
    N, d = Q.shape
    Nk = K.shape[0]
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    ridx = np.arange(N) if rows is None else np.arange(N)[rows]
    S = (Q[ridx] @ K.T) * sm_scale
    if causal:
        S = np.where(np.arange(Nk)[None, :] > ridx[:, None] + (Nk - N), -np.inf, S)
    S = S - S.max(axis=1, keepdims=True)
    P = np.exp(S)
    return (P / P.sum(axis=1, keepdims=True)) @ V
