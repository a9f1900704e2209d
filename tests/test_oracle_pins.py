"""Pins that tie the CPU oracle to facts fixed by the paper and by mathematics, so that the
oracle is trusted for reasons other than itself.  Each test names the passage it checks.
None of these tests touches a GPU or the HIP library."""
import json
import os

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import sage_oracle as so

f32, f64 = np.float32, np.float64


def _head(N=200, d=32, seed=0, k_off=3.0, q_off=1.0, outliers=0, dtype="fp16"):
    spec = wl.WorkloadSpec("t", 1, 1, 1, N, d, dtype, False, k_off, q_off, outliers, 10.0, 1.0, 77)
    return (wl.make_head(spec, "q", 0, 0, seed), wl.make_head(spec, "k", 0, 0, seed),
            wl.make_head(spec, "v", 0, 0, seed))


@pytest.fixture(scope="module")
def facts(golden_dir):
    with open(os.path.join(golden_dir, "paper_facts.json")) as f:
        return json.load(f)


# ---- P9: the plain definition itself (Sec. 2.1) against a library routine ------------------
@pytest.mark.parametrize("causal", [False, True])
def test_ref_attention_matches_library_sdpa(causal):
    q, k, v = _head(N=77, d=16)
    ref = so.ref_attn_fp64(q, k, v, causal=causal)
    tq, tk, tv = (torch.from_numpy(x).double()[None, None] for x in (q, k, v))
    lib = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=causal)[0, 0].numpy()
    assert np.allclose(ref, lib, rtol=1e-12, atol=1e-13)


# ---- P1: smoothing K leaves softmax unchanged (Sec. 3.1: a common bias on a row of S) ------
def test_k_smoothing_is_result_neutral_in_fp64():
    q, k, v = _head()
    kbar, gk = so.smooth_k(k)
    a = so.ref_attn_fp64(q, k, v)
    b = so.ref_attn_fp64(q, k.astype(f64) - kbar.astype(f64), v)
    assert np.abs(a - b).max() < 1e-11
    # the oracle's gamma(K) is that same matrix rounded once to FP32
    assert np.array_equal(gk, (k.astype(f64) - kbar.astype(f64)).astype(f32))


# ---- P10: smoothed K has zero channel mean and variance (N-1)/N (Appendix, smoothing theory)
def test_smoothed_k_mean_zero_and_variance_ratio():
    rng = np.random.default_rng(5)
    N, d = 8, 20000                    # tiny N makes the (N-1)/N factor visible
    x = wl.round_to_dtype(rng.standard_normal((N, d)).astype(f32) * 2 + 5, "fp16")
    kbar, gk = so.smooth_k(x)
    assert np.abs(gk.astype(f64).mean(axis=0)).max() < 1e-6
    assert np.allclose(kbar, x.astype(f64).mean(axis=0), rtol=1e-7, atol=1e-7)
    ratio = gk.astype(f64).var() / 4.0            # population variance of N(5, 2^2) draws
    assert abs(ratio - (N - 1) / N) < 0.01


# ---- P2: gamma(Q)gamma(K)^T + DeltaS + b == Q K^T exactly (Sec. 3.1 decomposition) ---------
def test_smoothing_decomposition_reproduces_scores():
    q, k, v = _head(N=300, d=32)
    bq = 128
    kbar, gk = so.smooth_k(k)
    qbar, gq = so.smooth_q(q, bq)
    # block means are means of the block's valid rows (ragged tail: 300 = 2*128 + 44)
    assert np.allclose(qbar[2], q[256:].astype(f64).mean(axis=0), rtol=1e-7, atol=1e-7)
    assert qbar.shape == (3, 32)
    D = so.delta_s(qbar, gk, f32(1.0))            # kappa = 1: the raw Delta S
    full = q.astype(f64) @ k.astype(f64).T
    for i in range(3):
        rows = slice(i * bq, min((i + 1) * bq, 300))
        b = (qbar[i].astype(f64) @ kbar.astype(f64)
             + gq[rows].astype(f64) @ kbar.astype(f64))[:, None]      # N x 1, row-constant
        rebuilt = gq[rows].astype(f64) @ gk.astype(f64).T + D[i].astype(f64)[None, :] + b
        assert np.abs(rebuilt - full[rows]).max() < 2e-4 * np.abs(full).max()
        # Delta S is a 1 x N vector per block: <qbar_i, gamma(K)_t>, brute force on a few t
        for t in (0, 17, 299):
            brute = sum(float(qbar[i, c]) * float(gk[t, c]) for c in range(32))
            assert abs(D[i, t] - brute) <= 1e-6 * (1 + abs(brute))
    # dropping b leaves softmax rows unchanged
    S1 = full[:128]
    S2 = gq[:128].astype(f64) @ gk.astype(f64).T + D[0].astype(f64)[None, :]
    sm = lambda s: np.exp(s - s.max(1, keepdims=True)) / np.exp(s - s.max(1, keepdims=True)).sum(1, keepdims=True)
    assert np.abs(sm(S1 * 0.1) - sm(S2 * 0.1)).max() < 1e-6


def test_delta_s_carries_kappa():
    q, k, _ = _head(N=64, d=16)
    _, gk = so.smooth_k(k)
    qbar, _ = so.smooth_q(q, 32)
    kap = f32(0.25 * so.LOG2E_F32)
    a = so.delta_s(qbar, gk, kap).astype(f64)
    b = so.delta_s(qbar, gk, f32(1.0)).astype(f64) * float(kap)
    assert np.allclose(a, b, rtol=3e-7, atol=1e-9)


# ---- P4: closed forms of the quantizer psi (Sec. 2.2; Sec. 3.1 first paragraph) -------------
@pytest.mark.parametrize("qmax_key", ["int4", "int8"])
def test_quantizer_closed_forms(facts, qmax_key):
    qmax = facts["int4_code_range"]["value"][1] if qmax_key == "int4" else facts["int8_code_max"]["value"]
    rng = np.random.default_rng(3)
    x = rng.standard_normal((96, 24)).astype(f32) * np.exp(rng.uniform(-2, 2, (96, 1))).astype(f32)
    groups = so.group_map("g950", 96, "k")
    delta, codes = so.quantize_groups(x, groups, qmax)
    assert codes.min() >= -qmax and codes.max() <= qmax
    for g in range(groups.max() + 1):
        sel = groups == g
        M = np.abs(x[sel]).max()
        assert delta[g] == f32(M / f32(qmax))
        # the group's largest element maps to +-qmax
        idx = np.unravel_index(np.abs(x[sel]).argmax(), x[sel].shape)
        assert abs(int(codes[sel][idx])) == qmax
        # reconstruction error at most half a step
        err = np.abs(x[sel].astype(f64) - codes[sel].astype(f64) * float(delta[g]))
        assert err.max() <= 0.5 * float(delta[g]) * (1 + 1e-6)
        if qmax_key == "int4":
            ratio = facts["int4_zero_ratio"]["value"]
            small = np.abs(x[sel]) < M / ratio * (1 - 1e-6)
            assert np.all(codes[sel][small] == 0)
            assert np.all(codes[sel][np.abs(x[sel]) > M / ratio * (1 + 1e-6)] != 0)


def test_quantizer_ties_to_even_and_zero_group():
    # delta = 7/7 = 1: the values below are exact halves
    x = np.array([[7.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5]], f32)
    delta, codes = so.quantize_groups(x, np.zeros(1, int), 7)
    assert delta[0] == 1.0
    assert codes.tolist() == [[7, 0, 2, 2, 0, -2, -2, 4]]
    delta, codes = so.quantize_groups(np.zeros((4, 3), f32), np.array([0, 0, 1, 1]), 7)
    assert np.all(delta == 0) and np.all(codes == 0)


# ---- P5: group maps (Sec. 3.2, Appendix formulation) ----------------------------------------
def test_group_maps(facts):
    N = 256
    q_nv, k_nv = so.group_map("nv_m16n8", N, "q"), so.group_map("nv_m16n8", N, "k")
    per_block = facts["nv_groups_per_128x64_block"]
    assert len(set(q_nv[:128])) == per_block["q"] and len(set(k_nv[:64])) == per_block["k"]
    for i in range(8):   # query tokens i, 8+i, 16+i, 24+i of a warp's 32 share a scale
        assert len({q_nv[i], q_nv[8 + i], q_nv[16 + i], q_nv[24 + i]}) == 1
    for i in range(4):   # keys 8k+2i and 8k+2i+1 share a scale within a 64-key block
        assert len({k_nv[8 * kk + 2 * i + e] for kk in range(8) for e in (0, 1)}) == 1
    assert q_nv[0] != q_nv[32] and k_nv[0] != k_nv[64]
    # gfx950 groups: as many K groups per 64-key block as the paper's (4), of the same size
    # (16 keys); Q groups at least as fine as the paper's (64 >= 32 per 128 queries)
    q_g, k_g = so.group_map("g950", N, "q"), so.group_map("g950", N, "k")
    assert len(set(k_g[:64])) == per_block["k"] and np.bincount(k_g).max() == 16
    assert len(set(q_g[:128])) == 64 and np.bincount(q_g).max() == 2
    assert len(set(so.group_map("per_tensor", N, "q"))) == 1
    assert np.array_equal(so.group_map("per_token", N, "k"), np.arange(N))
    assert len(set(so.group_map("per_block", N, "q"))) == 2 and len(set(so.group_map("per_block", N, "k"))) == 4


def test_per_tensor_map_is_sec22_example():
    # Sec. 2.2: delta_A = max|A| / 7 for the whole tensor
    rng = np.random.default_rng(0)
    x = rng.standard_normal((40, 8)).astype(f32)
    delta, codes = so.quantize_groups(x, so.group_map("per_tensor", 40, "q"), 7)
    assert delta.shape == (1,) and delta[0] == f32(np.abs(x).max() / f32(7))
    assert np.abs(codes).max() == 7


# ---- P3: integer QK^T against brute force ----------------------------------------------------
def test_int_scores_brute_force():
    rng = np.random.default_rng(11)
    qc = rng.integers(-7, 8, (5, 6)).astype(np.int8)
    kc = rng.integers(-7, 8, (4, 6)).astype(np.int8)
    acc = so.int_scores(qc, kc)
    for r in range(5):
        for t in range(4):
            assert acc[r, t] == sum(int(qc[r, c]) * int(kc[t, c]) for c in range(6))
    assert acc.shape == (5, 4)      # queries index rows, keys index columns
    big = so.int_scores(np.full((1, 128), 127, np.int8), np.full((1, 128), -127, np.int8))
    assert big[0, 0] == -127 * 127 * 128


# ---- P7: E4M3 codec (Sec. 3.3) ---------------------------------------------------------------
def test_e4m3_codec_against_format_table_and_library(facts, golden_dir):
    with open(os.path.join(golden_dir, "e4m3_codes.txt")) as f:
        rows = [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]
    for val, code in rows:
        assert so.e4m3_decode(np.array([int(code, 16)], np.uint8))[0] == float(val)
        assert so.e4m3_encode(np.array([float(val)]))[0] == int(code, 16)
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], np.uint8)
    vals = so.e4m3_decode(codes)
    assert np.nanmax(np.abs(vals)) == facts["e4m3_max"]["value"]
    assert np.array_equal(so.e4m3_encode(vals)[vals != 0], codes[vals != 0])   # round trip
    lib = torch.from_numpy(codes).view(torch.float8_e4m3fn).double().numpy()
    assert np.array_equal(vals, lib)
    rng = np.random.default_rng(2)
    x = (rng.standard_normal(300000) * np.exp(rng.uniform(-14, 6.2, 300000))).astype(f32)
    x = np.clip(x, -448, 448)
    lib_codes = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(so.e4m3_encode(x), lib_codes)
    # ties to even between neighbours (17 -> 16, 19 -> 20) and saturation above the range
    assert so.e4m3_decode(so.e4m3_encode(np.array([17.0, 19.0, 1000.0, -1e9, 464.0]))).tolist() == \
        [16.0, 20.0, 448.0, -448.0, 448.0]


def test_v_quantizer_is_per_channel(facts):
    rng = np.random.default_rng(4)
    v = rng.standard_normal((50, 6)).astype(f32) * np.array([1, 10, 0.1, 5, 0, 2], f32)
    delta, codes = so.quantize_v(v)
    assert delta.shape == (6,) and delta[4] == 0 and np.all(codes[:, 4] == 0)
    dec = so.e4m3_decode(codes)
    for c in (0, 1, 2, 3, 5):
        assert delta[c] == f32(np.abs(v[:, c]).max() / f32(facts["e4m3_max"]["value"]))
        assert np.abs(dec[:, c]).max() == 448.0                      # the channel max maps to 448
        rel = np.abs(dec[:, c] * float(delta[c]) - v[:, c]) / np.abs(v[:, c]).max()
        assert rel.max() <= 2.0 ** -4                                # half an ulp of 3 mantissa bits


# ---- P8: online softmax + two-level accumulation == two-pass softmax V (Sec. 2.1, Sec. 3.4) --
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N", [256, 203])
def test_identity_quantizers_reduce_to_plain_attention(causal, N):
    q, k, v = _head(N=N, d=32, k_off=1.0)
    out, _ = so.sage_attention_head(q, k, v, causal=causal, mode=32767, out_dtype="fp32",
                                    smooth_q_on=True, pv_exact=True)
    ref = so.ref_attn_fp64(q, k, v, causal=causal)
    assert np.abs(out - ref).max() < 2e-3 * np.abs(ref).max()
    assert wl.cos_sim(out, ref) > 1 - 1e-6


def test_block_sizes_do_not_change_the_mathematics():
    # any b_q / b_kv gives the same attention when nothing is quantized (Sec. 2.1 tiling)
    q, k, v = _head(N=150, d=16, k_off=1.0)
    ref = so.ref_attn_fp64(q, k, v, causal=True)
    for bq, bkv in ((128, 64), (32, 16), (64, 128)):
        out, _ = so.sage_attention_head(q, k, v, causal=True, mode=32767, out_dtype="fp32", bq=bq,
                                        bkv=bkv, smooth_q_on=True, pv_exact=True)
        assert np.abs(out - ref).max() < 2e-3 * np.abs(ref).max()


@pytest.mark.parametrize("form", ["printed", "kernel"])
def test_online_state_matches_two_pass(form):
    q, k, v = _head(N=192, d=16, k_off=1.0)
    pro = so.quantize_head(q, k, v, mode=32767, smooth_q_on=True, pv_exact=True)
    _, st = so.FORMS[form](pro, slice(0, 128), False, out_dtype="fp32", return_state=True)
    carried = 448.0 if form == "kernel" else 1.0       # the kernel-order form carries 448 * l
    S = (q[:128].astype(f64) @ (k.astype(f64) - pro["kbar"].astype(f64)).T) / np.sqrt(16) * np.log2(np.e)
    # m is the row max of the base-2 scores up to a row constant: compare differences
    m_ref = S.max(axis=1)
    shift = st["m"].astype(f64) - m_ref
    l_ref = np.exp2(S - m_ref[:, None]).sum(axis=1)
    assert np.allclose(st["l"] / carried, l_ref, rtol=2e-3)
    # the constant is the dropped bias b of Sec. 3.1 (times kappa): it varies per row only
    assert shift.shape == (128,)


@pytest.mark.parametrize("form", ["printed", "kernel"])
def test_static_p_scale_is_448(form):
    # Sec. 3.3: P~ in [0, 1] is quantized with the static scale 1/448, i.e. the FP8 code is taken of
    # 448 * P~.  With a single key P~ = 1: its code is that of 448, the denominator is 1 (448 in the form that
    # carries 448 * l) and the output is exactly the dequantized FP8 value of V; with two equal keys the
    # denominator doubles and the output is the average.
    attention_rows = so.FORMS[form]
    carried = 448.0 if form == "kernel" else 1.0
    q = np.ones((1, 16), f32); k = np.ones((1, 16), f32)
    v = np.linspace(-3, 3, 16, dtype=f32)[None, :].astype(np.float16).astype(f32)
    pro = so.quantize_head(q, k, v, mode="int8_fp8")
    out, st, codes = attention_rows(pro, slice(0, 1), False, out_dtype="fp32", return_state=True, return_codes=True)
    assert abs(float(st["l"][0]) - carried) < carried * 1e-6
    assert codes[0, 0] == so.e4m3_encode(448.0) and not codes[0, 1:].any()
    dec = so.e4m3_decode(pro["v_codes"]) * pro["v_scale"].astype(f64)[None, :]
    assert np.allclose(out, dec, rtol=1e-6, atol=0)
    q2, k2, v2 = np.ones((2, 16), f32), np.ones((2, 16), f32), np.concatenate([v, v])
    pro2 = so.quantize_head(q2, k2, v2, mode="int8_fp8")
    _, st2 = attention_rows(pro2, slice(0, 2), False, out_dtype="fp32", return_state=True)
    assert np.allclose(st2["l"], 2 * carried, rtol=1e-6)


# ---- P6: the quantized pipeline approaches FP64 attention as bit-width grows -----------------
def test_error_decreases_with_bit_width():
    q, k, v = _head(N=256, d=64, seed=1)
    ref = so.ref_attn_fp64(q, k, v)
    errs = []
    for qmax in (7, 127, 32767):
        out, _ = so.sage_attention_head(q, k, v, mode=qmax, out_dtype="fp32", smooth_q_on=True, pv_exact=True)
        errs.append(wl.rel_l1(out, ref))
    assert errs[0] > 5 * errs[1] > 25 * errs[2]
    assert errs[2] < 1e-4
    # with FP8 P~ and V the 8-bit variant stays close to the definition
    out8, _ = so.sage_attention_head(q, k, v, mode="int8_fp8", out_dtype="fp32")
    assert wl.cos_sim(out8, ref) > 0.998
    out4, _ = so.sage_attention_head(q, k, v, mode="int4_fp8", out_dtype="fp32")
    assert 0.95 < wl.cos_sim(out4, ref) < wl.cos_sim(out8, ref)


def test_fp8_stage_error_is_bounded_by_format_precision():
    # E4M3 keeps 3 mantissa bits: each of P^ and V^ is within 2^-4 relative (Sec. 3.3), so the
    # FP8 output differs from the exact-PV output by at most about 2*2^-4 of sum_t p_t |v_t|.
    q, k, v = _head(N=256, d=32, seed=2)
    a, _ = so.sage_attention_head(q, k, v, mode="int8_fp8", out_dtype="fp32")
    b, _ = so.sage_attention_head(q, k, v, mode="int8_fp8", out_dtype="fp32", pv_exact=True)
    bound = 0.14 * np.abs(v).max()
    assert np.abs(a - b).max() < bound
    assert np.abs(a - b).max() > 1e-6                 # and FP8 really is in the path


# ---- P5/P11: orderings the paper reports, on synthetic outlier-bearing data ------------------
def test_granularity_and_smoothing_orderings(facts):
    spec = wl.CONFIGS["prefill4k"].with_(N=512, H=1, H_kv=1, B=1)
    q, k, v = (wl.make_head(spec, w, 0, 0, 3) for w in "qkv")
    ref = so.ref_attn_fp64(q, k, v)
    cs = {}
    for g in ("per_token", "g950", "nv_m16n8", "per_block", "per_tensor"):
        out, _ = so.sage_attention_head(q, k, v, gmap=g, out_dtype="fp32")
        cs[g] = wl.cos_sim(out, ref)
    assert cs["per_token"] >= cs["per_block"] > cs["per_tensor"] - 1e-3
    assert cs["g950"] > cs["per_block"] and cs["nv_m16n8"] > cs["per_block"]
    sm = {}
    for name, (sq, sk) in dict(qk=(True, True), q=(True, False), k=(False, True), none=(False, False)).items():
        out, _ = so.sage_attention_head(q, k, v, out_dtype="fp32", smooth_q_on=sq, smooth_k_on=sk)
        sm[name] = wl.cos_sim(out, ref)
    assert sm["qk"] > sm["k"] > sm["none"] and sm["qk"] > sm["q"] > sm["none"]


# ---- optional smooth V (end of Sec. 3.4; Appendix "Smoothing V") ------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_smooth_v_is_result_neutral_and_added_back(causal):
    q, k, v = _head(N=200, d=32, seed=4)
    v = (v + np.linspace(-9, 9, 32, dtype=f32)[None, :]).astype(np.float16).astype(f32)   # channel biases
    ref = so.ref_attn_fp64(q, k, v, causal=causal)
    vm = v.astype(f64).mean(axis=0)
    # rows of the softmax sum to 1, so P (V - vm) + vm = P V: plain float64 identity
    shifted = so.ref_attn_fp64(q, k, (v.astype(f64) - vm), causal=causal) + vm
    assert np.abs(shifted - ref).max() < 1e-12 * np.abs(ref).max()
    # the oracle's path with quantizers at their high-precision limit keeps that identity
    out, pro = so.sage_attention_head(q, k, v, causal=causal, mode=32767, out_dtype="fp32",
                                      smooth_q_on=True, pv_exact=True, smooth_v_on=True)
    assert np.array_equal(pro["vbar"], vm.astype(f32))
    assert np.abs(out - ref).max() < 2e-3 * np.abs(ref).max()
    assert wl.cos_sim(out, ref) > 1 - 1e-6


def test_smooth_v_quantizes_the_centred_values_and_helps_with_channel_bias(facts):
    q, k, v = _head(N=256, d=32, seed=5)
    v = (v + np.float32(8.5)).astype(np.float16).astype(f32)        # the 8..9 bias quoted for CogVideoX
    pro = so.quantize_head(q, k, v, smooth_v_on=True)
    centred = (v - pro["vbar"][None, :]).astype(f32)
    assert np.array_equal(pro["v_scale"], (np.abs(centred).max(axis=0) / f32(facts["e4m3_max"]["value"])).astype(f32))
    dec = so.e4m3_decode(pro["v_codes"]) * pro["v_scale"].astype(f64)[None, :]
    assert np.abs(dec - centred).max() <= np.abs(centred).max() * 2.0 ** -4 * 1.001
    ref = so.ref_attn_fp64(q, k, v)
    plain, _ = so.sage_attention_head(q, k, v, mode="int8_fp8", out_dtype="fp32")
    smooth, _ = so.sage_attention_head(q, k, v, mode="int8_fp8", out_dtype="fp32", smooth_v_on=True)
    # the paper's table for this technique reports a lower error with it (ordering only)
    assert wl.rmse(smooth, ref) < 0.5 * wl.rmse(plain, ref)
    assert wl.cos_sim(smooth, ref) >= wl.cos_sim(plain, ref)


# ---- key length different from query length ------------------------------------------------------
@pytest.mark.parametrize("causal", [False, True])
def test_other_key_length(causal):
    # the definition against a library routine with an explicit mask aligned to the last query and key,
    # and the oracle's path with its quantizers at their high-precision limit against the definition
    rng = np.random.default_rng(7)
    Nq, Nk, d = 70, 203, 32
    q = rng.standard_normal((Nq, d)).astype(np.float16).astype(f32)
    k = (rng.standard_normal((Nk, d)) + 1.5).astype(np.float16).astype(f32)
    v = rng.standard_normal((Nk, d)).astype(np.float16).astype(f32)
    ref = so.ref_attn_fp64(q, k, v, causal=causal)
    mask = None
    if causal:
        mask = torch.from_numpy(np.arange(Nk)[None, :] <= np.arange(Nq)[:, None] + (Nk - Nq))
    lib = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double()[None], torch.from_numpy(k).double()[None], torch.from_numpy(v).double()[None],
        attn_mask=mask).numpy()[0]
    assert np.abs(ref - lib).max() < 1e-12
    out, pro = so.sage_attention_head(q, k, v, causal=causal, mode=32767, out_dtype="fp32", smooth_q_on=True,
                                      pv_exact=True)
    assert pro["delta_s"].shape == (1, Nk) and pro["k_codes"].shape == (Nk, d) and pro["q_codes"].shape == (Nq, d)
    assert np.abs(out - ref).max() < 2e-3 * np.abs(ref).max()
    assert wl.cos_sim(out, ref) > 1 - 1e-6
    if causal:      # the last query sees every key, the first one Nk - Nq + 1 of them
        first = so.ref_attn_fp64(q[:1], k[: Nk - Nq + 1], v[: Nk - Nq + 1])
        assert np.abs(ref[0] - first[0]).max() < 1e-12


# ---- misc structure -------------------------------------------------------------------------
def test_int8_mode_does_not_smooth_q():
    q, k, v = _head(N=128, d=16)
    pro = so.quantize_head(q, k, v, mode="int8_fp8")
    assert pro["qbar"] is None and pro["delta_s"] is None and pro["qmax"] == 127
    # codes are those of the raw Q
    _, codes = so.quantize_groups(q, so.group_map("g950", 128, "q"), 127)
    assert np.array_equal(pro["q_codes"], codes)


def test_gqa_head_mapping_and_batched_form():
    spec = wl.CONFIGS["tiny"].with_(H=4, H_kv=2, N=128, d=16)
    d = wl.make_inputs(spec)
    out = so.sage_attention(d["q"], d["k"], d["v"], out_dtype="fp16")
    one, _ = so.sage_attention_head(d["q"][0, 3], d["k"][0, 1], d["v"][0, 1], out_dtype="fp16")
    assert np.array_equal(out[0, 3], one)
    one, _ = so.sage_attention_head(d["q"][0, 1], d["k"][0, 0], d["v"][0, 0], out_dtype="fp16")
    assert np.array_equal(out[0, 1], one)


def test_causal_rows_ignore_future_keys():
    q, k, v = _head(N=256, d=16)
    pro = so.quantize_head(q, k, v)
    a = so.attention_rows(pro, slice(0, 128), True, out_dtype="fp32")
    # future keys' codes/values cannot matter: scramble them
    pro2 = dict(pro)
    pro2["k_codes"] = pro["k_codes"].copy(); pro2["k_codes"][128:] = 7
    pro2["v_dec"] = pro["v_dec"].copy(); pro2["v_dec"][128:] = 400.0
    b = so.attention_rows(pro2, slice(0, 128), True, out_dtype="fp32")
    assert np.array_equal(a, b)
    # row 0 attends to key 0 only: output = dequantized V^[0]
    assert np.allclose(a[0], pro["v_dec"][0] * pro["v_scale"], rtol=1e-6)


def test_metrics_formulas():
    # Appendix "Datasets and Metrics": CosSim, relative L1, RMSE of flattened outputs
    a = np.array([[1.0, 2.0], [3.0, 4.0]]); b = np.array([[1.0, 2.0], [3.0, 5.0]])
    assert abs(wl.cos_sim(a, b) - 34 / np.sqrt(30 * 39)) < 1e-12
    assert abs(wl.rel_l1(a, b) - 1 / 11) < 1e-12
    assert abs(wl.rmse(a, b) - 0.5) < 1e-12
    assert abs(wl.max_abs_over_row_linf(a, b) - 0.2) < 1e-12


def test_output_rounding_matches_library_casts():
    # Algorithm 1 writes O in the input's 16-bit type; the cast is round-to-nearest-even
    rng = np.random.default_rng(9)
    x = (rng.standard_normal(100000) * np.exp(rng.uniform(-8, 8, 100000))).astype(f32)
    ties = np.array([1.00390625, 1.01171875, -1.00390625, 3.0078125], f32)   # exact bf16 halves
    x = np.concatenate([x, ties])
    for name, td in (("bf16", torch.bfloat16), ("fp16", torch.float16)):
        lib = torch.from_numpy(x).to(td).float().numpy()
        assert np.array_equal(so._round_out(x, name), lib)
        assert np.array_equal(wl.round_to_dtype(x, name), lib)


# ---- log-sum-exp of a row: the normaliser of Sec. 2.1 in the scale of the unsmoothed scores ----
@pytest.mark.parametrize("causal", [False, True])
def test_ref_lse_matches_library_logsumexp(causal):
    q, k, _ = _head(N=90, d=16)
    s = torch.from_numpy(q).double() @ torch.from_numpy(k).double().T / 4.0
    if causal:
        s = s.masked_fill(torch.ones(90, 90, dtype=torch.bool).triu(1), float("-inf"))
    assert np.allclose(so.ref_lse_fp64(q, k, causal=causal), torch.logsumexp(s, dim=1).numpy(), rtol=1e-13, atol=1e-12)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("smooth_q_on", [False, True])
def test_lse_approaches_the_definition_in_the_high_precision_limit(causal, smooth_q_on):
    """With 16-bit codes the dequantized scores are the true ones to 1e-4, so m + log2 l plus the row
    constant that smoothing K removed (Sec. 3.1) must reproduce ln sum exp(sm_scale q.k): a missing or
    mis-signed constant, a missing log2(448) or a wrong base would be off by units."""
    q, k, v = _head(N=300, d=32, seed=5, k_off=3.0, q_off=2.0)
    _, pro = so.sage_attention_head(q, k, v, causal=causal, mode=32767, smooth_q_on=smooth_q_on, out_dtype="fp32",
                                    want_lse=True)
    ref = so.ref_lse_fp64(q, k, causal=causal)
    assert np.abs(ref).max() > 5.0                      # the K offset makes the dropped constant large
    assert np.abs(pro["lse"] - ref).max() < 2e-3
    # and the quantized modes stay within their score error of it
    for mode, tol in (("int8_fp8", 0.1), ("int4_fp8", 1.0)):
        _, p2 = so.sage_attention_head(q, k, v, causal=causal, mode=mode, out_dtype="fp32", want_lse=True)
        assert np.abs(p2["lse"] - ref).max() < tol


def test_lse_merges_partial_results_over_disjoint_key_sets():
    """out = sum_parts exp(lse_part - lse) out_part with lse = ln sum_parts exp(lse_part): the identity the
    row statistic exists for, checked on the oracle's own outputs (each part smooths K with its own mean)."""
    q, k, v = _head(N=256, d=32, seed=6)
    full = so.ref_attn_fp64(q, k, v)
    parts = [so.sage_attention_head(q, k[a:b], v[a:b], mode="int8_fp8", out_dtype="fp32", want_lse=True)
             for a, b in ((0, 100), (100, 256))]
    lse = np.stack([p[1]["lse"].astype(f64) for p in parts])
    tot = np.log(np.exp(lse - lse.max(axis=0)).sum(axis=0)) + lse.max(axis=0)
    merged = sum(np.exp(l - tot)[:, None] * p[0] for l, p in zip(lse, parts))
    whole, _ = so.sage_attention_head(q, k, v, mode="int8_fp8", out_dtype="fp32")
    assert wl.cos_sim(merged, full) > 0.998
    assert wl.rel_l1(merged, full) < 1.5 * wl.rel_l1(whole, full) + 1e-3


# ---- the E5M2 variant of the FP8 stage (Sec. 3.3 / the data-type table compare it with E4M3) ----
def test_e5m2_codec_matches_library_cast_and_round_trips():
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes).view(torch.float8_e5m2).to(torch.float64).numpy()
    dec = so.e5m2_decode(codes)
    assert np.array_equal(np.isnan(dec), np.isnan(lib)) and np.array_equal(dec[~np.isnan(dec)], lib[~np.isnan(lib)])
    finite = np.isfinite(dec)
    assert np.array_equal(so.e5m2_encode(dec[finite]), codes[finite])      # every finite code is a fixed point
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.uniform(-57344, 57344, 4000), rng.normal(0, 1e-4, 2000), rng.normal(0, 3, 2000),
                        [1.25 * 2.0 ** k for k in range(-16, 15)], [1.125, 1.375, 1.625, 1.875, 3.0e-5]]).astype(f32)
    lib_codes = torch.from_numpy(x).to(torch.float8_e5m2).view(torch.uint8).numpy()
    assert np.array_equal(so.e5m2_encode(x), lib_codes)          # round to nearest, ties to even, in range
    assert so.e5m2_decode(so.e5m2_encode(np.array([1e9, -1e9]))).tolist() == [57344.0, -57344.0]   # saturating


def test_e5m2_stage_is_less_accurate_than_e4m3():
    """Two mantissa bits instead of three: the ordering of the paper's data-type comparison for P~V."""
    q, k, v = _head(N=256, d=32, seed=2)
    ref = so.ref_attn_fp64(q, k, v)
    a, pa_ = so.sage_attention_head(q, k, v, mode="int8_fp8", out_dtype="fp32")
    b, pb_ = so.sage_attention_head(q, k, v, mode="int8_fp8", out_dtype="fp32", pv_fmt="e5m2")
    assert np.array_equal(pb_["v_scale"], (np.abs(v).max(axis=0) / f32(57344.0)).astype(f32))
    assert wl.rel_l1(a, ref) < wl.rel_l1(b, ref) < 4 * wl.rel_l1(a, ref)
    assert wl.cos_sim(b, ref) > 0.995


def test_int8_pv_variant_is_an_integer_product_with_static_scale_127():
    """The INT8 choice for P~V of the paper's data-type comparison: V codes are the psi of Sec. 2.2 per channel
    with qmax 127, P~ codes are rint(127 P~) (a row's largest P~ is 1 -> 127).  A uniform 7-bit grid loses the
    many small P~ of a long row (below 1/254 they round to 0), a floating-point format does not: the INT8 error
    grows with the sequence length and passes E4M3's, which is why the paper settles on E4M3 (Sec. 3.3)."""
    errs = {}
    for N in (256, 4096):
        q, k, v = _head(N=N, d=32, seed=2)
        ref = so.ref_attn_fp64(q, k, v)
        a, _ = so.sage_attention_head(q, k, v, mode="int8_fp8", out_dtype="fp32")
        b, pro = so.sage_attention_head(q, k, v, mode="int8_fp8", out_dtype="fp32", pv_fmt="int8")
        errs[N] = (wl.rel_l1(a, ref), wl.rel_l1(b, ref))
        if N == 256:
            dv = (np.abs(v).max(axis=0) / f32(127.0)).astype(f32)
            assert np.array_equal(pro["v_scale"], dv)
            assert np.array_equal(pro["v_codes"],
                                  np.clip(np.rint((v / dv[None, :]).astype(f32)), -127, 127).astype(np.int8))
            assert np.abs(pro["v_codes"]).max() == 127
            out, st, codes = so.attention_rows(pro, slice(0, 128), False, out_dtype="fp32", return_state=True,
                                               return_codes=True)
            assert np.all(st["l"] >= 1.0)                # the row maximum alone contributes 1 to l ...
            assert np.all(codes.view(np.int8).max(axis=1) == 127)    # ... and its code is 127
            _, stk = so.attention_rows_kernel_order(pro, slice(0, 128), False, out_dtype="fp32", return_state=True)
            assert np.all(stk["l"] >= 127.0 - 1e-3)     # the form that carries 127 * l
    assert errs[4096][1] > 1.5 * errs[256][1]           # INT8 degrades with the length ...
    assert abs(errs[4096][0] - errs[256][0]) < 0.3 * errs[256][0]   # ... E4M3 does not
    assert errs[4096][1] > errs[4096][0]
