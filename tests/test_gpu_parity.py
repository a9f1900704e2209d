"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element,
on seeded inputs that span several tiles, ragged tails, both modes, both head dims, causal
masks and grouped KV heads.

Bars: codes, scales, means and int32 score accumulators bit-equal; Delta-S equal up to the
last FP32 bit of a float64-accumulated value; outputs within 2e-3 max-abs after dividing by
the row's L-inf norm and cosine >= 0.9999 against Algorithm 1 evaluated as printed, within 5e-4 against
its kernel-order form, every row beyond either bar explained by one-step codes of P~ (oracle/parity.py)."""
import ctypes

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import parity
from oracle import sage_oracle as so

pytestmark = pytest.mark.gpu

OUT_TOL, COS_TOL = parity.OUT_TOL, parity.COS_TOL
_half_ulp16 = parity.half_ulp16


def _pa():
    import paper_2411_10958_amd as pa
    pa.load_library()
    return pa


def _spec(N, d, dtype="bf16", H=2, Hkv=2, B=1, causal=False, outliers=0, cfg=91):
    return wl.WorkloadSpec(f"t{N}x{d}", B, H, Hkv, N, d, dtype, causal, 3.0, 1.5, outliers, 10.0, 1.0, cfg)


def _gpu_inputs(spec, seed=0):
    data = wl.make_inputs(spec, seed)
    dev = torch.device("cuda:0")
    return data, tuple(wl.to_torch(data[n], spec.dtype, dev) for n in "qkv")


CASES = [
    # N, d, dtype, H, Hkv, causal
    (256, 64, "fp16", 2, 2, False),     # the tiny configuration
    (256, 64, "fp16", 2, 2, True),
    (250, 64, "fp16", 2, 2, False),     # ragged last tiles
    (333, 128, "bf16", 2, 1, True),     # ragged + causal + grouped KV heads + d=128
    (640, 128, "bf16", 4, 2, False),    # several Q blocks and 10 KV blocks
    (1, 64, "bf16", 1, 1, True),        # degenerate: a single token
    (17, 128, "fp16", 1, 1, False),     # shorter than one group-of-16 plus one
    (300, 256, "bf16", 2, 1, True),     # head dimension 256: ragged + causal + grouped KV heads
    (256, 256, "fp16", 2, 2, False),
    (1300, 128, "bf16", 8, 2, True),    # 11 query blocks x 4 heads of a KV group: the Delta-S rows of the group share passes
    (2100, 64, "fp16", 4, 2, False),    # 17 x 2 rows: a second pass with two rows
]


@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("N,d,dtype,H,Hkv,causal", CASES)
def test_prologue_bit_exact(N, d, dtype, H, Hkv, causal, mode):
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, causal=causal)
    data, (q, k, v) = _gpu_inputs(spec)
    print(f"case N={N} d={d} {dtype} H={H}/{Hkv} mode={mode}", flush=True)
    got, args, ws = pa.sage_attn_quant(q, k, v, causal=causal, mode=mode)
    torch.cuda.synchronize()
    got = {n: t.cpu().numpy() for n, t in got.items()}
    g = H // Hkv
    for b in range(spec.B):
        for h in range(H):
            pro = so.quantize_head(data["q"][b, h], data["k"][b, h // g], data["v"][b, h // g], mode=mode)
            assert np.array_equal(got["q_codes"][b, h], pro["q_codes"]), "q codes"
            assert np.array_equal(got["q_scale"][b, h], pro["q_scale"]), "q scales"
            assert np.array_equal(got["k_codes"][b, h // g], pro["k_codes"]), "k codes"
            assert np.array_equal(got["k_scale"][b, h // g], pro["k_scale"]), "k scales"
            assert np.array_equal(got["v_codes"][b, h // g], pro["v_codes"]), "v codes"
            assert np.array_equal(got["v_scale"][b, h // g], pro["v_scale"]), "v scales"
            assert np.array_equal(got["k_mean"][b, h // g], pro["kbar"]), "k mean"
            if mode == "int4_fp8":
                assert np.array_equal(got["q_mean"][b, h], pro["qbar"]), "q block means"
                D = pro["delta_s"]
                diff = np.abs(got["delta_s"][b, h].astype(np.float64) - D.astype(np.float64))
                # float64 accumulation in another order, one rounding to FP32: at most the last bit
                assert np.all(diff <= np.spacing(np.abs(D)).astype(np.float64)), "delta S"
                assert (diff > 0).mean() < 1e-3
            # int32 score accumulators of every (q tile, kv block) through the MFMA path
            nqb, nkb = (N + 127) // 128, (N + 63) // 64
            for qt in range(nqb):
                for kb in range(nkb):
                    acc = pa.sage_attn_debug_qk(args, b, h, qt, kb).cpu().numpy()
                    rows = slice(qt * 128, min(qt * 128 + 128, N))
                    keys = slice(kb * 64, min(kb * 64 + 64, N))
                    ref = so.int_scores(pro["q_codes"][rows], pro["k_codes"][keys])
                    assert np.array_equal(acc[: ref.shape[0], : ref.shape[1]], ref), "int32 accumulators"
                    assert not acc[ref.shape[0]:].any() and not acc[:, ref.shape[1]:].any()


@pytest.mark.parametrize("form", ["digits", "fp64"])
@pytest.mark.parametrize("N,d,dtype,H,Hkv,causal", [CASES[3], CASES[4], CASES[6], CASES[7], CASES[9], CASES[10],
                                                    (4200, 64, "bf16", 2, 1, True),      # 33 query blocks: two passes per head, causal skipping
                                                    (4100, 128, "fp16", 1, 1, False)])
def test_both_exact_forms_of_delta_s(N, d, dtype, H, Hkv, causal, form):
    """Delta-S (Sec. 3.1) by digit products on the INT8 matrix unit and by the FP64 matrix instruction, each forced: within
    the last bit of the oracle's correctly rounded float64 inner product, and different from it at most once in 10^3."""
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, causal=causal)
    data, (q, k, v) = _gpu_inputs(spec)
    got, _, _ = pa.sage_attn_quant(q, k, v, causal=causal, want=("delta_s", "q_mean"), delta_s=form)
    torch.cuda.synchronize()
    ds = got["delta_s"].cpu().numpy()
    g = H // Hkv
    for h in range(H):
        pro = so.quantize_head(data["q"][0, h], data["k"][0, h // g], data["v"][0, h // g])
        D = pro["delta_s"].astype(np.float64)
        diff = np.abs(ds[0, h].astype(np.float64) - D)
        if causal:      # rows are defined up to the keys their queries can see (in groups of 32 blocks)
            vis = np.arange(N)[None, :] < 4096 * (np.arange(D.shape[0])[:, None] // 32 + 1)
            diff = np.where(vis, diff, 0.0)
        assert np.all(diff <= np.spacing(np.abs(D.astype(np.float32))).astype(np.float64)), f"delta S ({form})"
        assert (diff > 0).mean() < 1e-3


@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("N,d,dtype,H,Hkv,causal", CASES)
def test_attention_output_matches_oracle(N, d, dtype, H, Hkv, causal, mode):
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, causal=causal)
    data, (q, k, v) = _gpu_inputs(spec)
    print(f"case N={N} d={d} {dtype} H={H}/{Hkv} causal={causal} mode={mode}", flush=True)
    out = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode)
    torch.cuda.synchronize()
    got = wl.from_torch(out)
    # (few tiles and many keys: the library splits the key range by itself, and says so)
    splits = pa.sage_attn_kv_splits(pa.make_args(q, k, v, causal=causal, mode=mode))
    parity.check_heads(got, data, causal, mode, dtype, splits=splits)
    # accuracy against the unquantized definition is reported, not asserted tightly
    g = H // Hkv
    full = np.stack([so.ref_attn_fp64(data["q"][0, h], data["k"][0, h // g], data["v"][0, h // g], causal)
                     for h in range(H)])
    print(f"  vs FP64 attention: cos {wl.cos_sim(got[0], full):.5f} relL1 {wl.rel_l1(got[0], full):.4f}", flush=True)
    assert wl.cos_sim(got[0], full) > (0.9 if mode == "int4_fp8" else 0.99)


# ---- optional smooth V (Sec. 3.4 last paragraph; Appendix "Smoothing V") ----------------------
SMOOTH_V_CASES = [
    (250, 64, "fp16", 2, 2, False),
    (333, 128, "bf16", 2, 1, True),
    (640, 128, "bf16", 4, 2, False),
]


@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("N,d,dtype,H,Hkv,causal", SMOOTH_V_CASES)
def test_smooth_v_matches_oracle(N, d, dtype, H, Hkv, causal, mode):
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, causal=causal).with_(v_bias=8.5)
    data, (q, k, v) = _gpu_inputs(spec)
    print(f"smooth-V case N={N} d={d} {dtype} H={H}/{Hkv} causal={causal} mode={mode}", flush=True)
    got, args, ws = pa.sage_attn_quant(q, k, v, causal=causal, mode=mode, smooth_v=True,
                                       want=("v_codes", "v_scale", "v_mean", "k_codes", "k_scale"))
    torch.cuda.synchronize()
    got = {n: t.cpu().numpy() for n, t in got.items()}
    for b in range(spec.B):
        for hk in range(Hkv):
            pro = so.quantize_head(data["q"][b, hk * (H // Hkv)], data["k"][b, hk], data["v"][b, hk], mode=mode,
                                   smooth_v_on=True)
            assert np.array_equal(got["v_mean"][b, hk], pro["vbar"]), "v mean"
            assert np.array_equal(got["v_scale"][b, hk], pro["v_scale"]), "v scales of the centred values"
            assert np.array_equal(got["v_codes"][b, hk], pro["v_codes"]), "v codes of the centred values"
            assert np.array_equal(got["k_codes"][b, hk], pro["k_codes"]), "k codes unaffected"
    out = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, smooth_v=True)
    plain = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode)
    torch.cuda.synchronize()
    got_out, got_plain = wl.from_torch(out), wl.from_torch(plain)
    parity.check_heads(got_out, data, causal, mode, dtype, smooth_v_on=True)
    g = H // Hkv
    full = np.stack([so.ref_attn_fp64(data["q"][0, h], data["k"][0, h // g], data["v"][0, h // g], causal)
                     for h in range(H)])
    e_s, e_p = wl.rmse(got_out[0], full), wl.rmse(got_plain[0], full)
    print(f"  RMSE vs FP64 attention: smooth V {e_s:.4f}, plain {e_p:.4f}", flush=True)
    assert e_s < e_p        # the ordering the paper's table for this technique reports


# ---- smoothing ablation (Sec. 3.1, Eq. 2; the paper's table of smoothing variants: none / only K / Q and K) ----
@pytest.mark.parametrize("smooth_k,smooth_q", [(False, False), (True, False), (False, True)])
@pytest.mark.parametrize("N,d,dtype,H,Hkv,causal", [(300, 64, "fp16", 2, 2, False), (448, 128, "bf16", 4, 2, True)])
def test_smoothing_switched_off_matches_oracle(N, d, dtype, H, Hkv, causal, smooth_k, smooth_q):
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, causal=causal)
    data, (q, k, v) = _gpu_inputs(spec)
    print(f"smoothing ablation N={N} d={d} {dtype} H={H}/{Hkv} causal={causal} K={smooth_k} Q={smooth_q}", flush=True)
    got, args, ws = pa.sage_attn_quant(q, k, v, causal=causal, smooth_k=smooth_k, smooth_q=smooth_q)
    torch.cuda.synchronize()
    got = {n: t.cpu().numpy() for n, t in got.items()}
    g = H // Hkv
    for b in range(spec.B):
        for h in range(H):
            pro = so.quantize_head(data["q"][b, h], data["k"][b, h // g], data["v"][b, h // g],
                                   smooth_q_on=smooth_q, smooth_k_on=smooth_k)
            assert np.array_equal(got["q_codes"][b, h], pro["q_codes"]), "q codes"
            assert np.array_equal(got["q_scale"][b, h], pro["q_scale"]), "q scales"
            assert np.array_equal(got["k_codes"][b, h // g], pro["k_codes"]), "k codes"
            assert np.array_equal(got["k_scale"][b, h // g], pro["k_scale"]), "k scales"
            assert np.array_equal(got["k_mean"][b, h // g], pro["kbar"]), "k mean (zeros without K smoothing)"
            if smooth_q:
                assert np.array_equal(got["q_mean"][b, h], pro["qbar"]), "q block means"
                D = pro["delta_s"].astype(np.float64)
                diff = np.abs(got["delta_s"][b, h].astype(np.float64) - D)
                assert np.all(diff <= np.spacing(np.abs(D.astype(np.float32))).astype(np.float64)), "delta S"   # one unit of the FP32 value's last place
            else:
                assert not got["q_mean"][b, h].any() and not got["delta_s"][b, h].any(), "no Q smoothing: zeros"
    out, lse = pa.sage_attn_fwd_ex(q, k, v, causal=causal, smooth_k=smooth_k, smooth_q=smooth_q, return_lse=True)
    torch.cuda.synchronize()
    pros = parity.check_heads(wl.from_torch(out), data, causal, "int4_fp8", dtype, want_lse=True,
                              smooth_q_on=smooth_q, smooth_k_on=smooth_k)
    for b in range(spec.B):
        for h in range(H):
            _lse_close(lse[b, h].cpu().numpy(), pros[b][h]["lse"], pros[b][h])


# ---- Delta-S accumulated in FP32 (an option of the boundary: faster preprocessing, approximate Delta-S) ----
def _delta_s_within_fp32_bound(got, pro, K, seen=None):
    """The kernel's FP32-accumulated Delta-S against the oracle's (float64 inner product, one rounding): the
    textbook bound of an FP32 dot product of d terms, |error| <= (d + 2) 2^-24 kappa sum_c |q_bar_c| |gamma(K)_c|
    (+ the oracle's own final rounding), and - independent roundings largely cancel - a mean error below two
    units of 2^-24 of that magnitude, which a lost operand bit (16-bit operands, say) would exceed."""
    D = pro["delta_s"].astype(np.float64)
    gK = (np.asarray(K, np.float32) - pro["kbar"][None, :]).astype(np.float32)
    mag = float(pro["kappa"]) * (np.abs(pro["qbar"]).astype(np.float64) @ np.abs(gK).astype(np.float64).T)
    diff = np.abs(np.asarray(got, np.float64) - D)
    if seen is not None:
        diff = np.where(seen, diff, 0.0)
    u, d = 2.0 ** -24, gK.shape[1]
    assert np.all(diff <= (d + 2) * u * mag + np.spacing(np.abs(D))), "delta S beyond the FP32 dot-product bound"
    if diff.size >= 4096:       # a statement about many independent roundings
        assert diff.mean() <= 2 * u * max(mag.mean(), 1e-30), "delta S: mean error too large for FP32 operands"


@pytest.mark.parametrize("N,d,dtype,H,Hkv,causal", [(640, 128, "bf16", 4, 2, False), (300, 64, "fp16", 2, 2, True)])
def test_fp32_delta_s_option(N, d, dtype, H, Hkv, causal):
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, causal=causal, outliers=2)
    data, (q, k, v) = _gpu_inputs(spec)
    print(f"FP32 Delta-S N={N} d={d} {dtype} H={H}/{Hkv} causal={causal}", flush=True)
    got, args, ws = pa.sage_attn_quant(q, k, v, causal=causal, fp32_delta_s=True)
    torch.cuda.synchronize()
    got = {n: t.cpu().numpy() for n, t in got.items()}
    g = H // Hkv
    for b in range(spec.B):
        for h in range(H):
            pro = so.quantize_head(data["q"][b, h], data["k"][b, h // g], data["v"][b, h // g])
            # everything else of the preprocessing is untouched by the option
            assert np.array_equal(got["q_codes"][b, h], pro["q_codes"]) and np.array_equal(got["k_codes"][b, h // g], pro["k_codes"])
            assert np.array_equal(got["q_mean"][b, h], pro["qbar"]) and np.array_equal(got["k_scale"][b, h // g], pro["k_scale"])
            _delta_s_within_fp32_bound(got["delta_s"][b, h], pro, data["k"][b, h // g])
    out = pa.sage_attn_fwd_ex(q, k, v, causal=causal, fp32_delta_s=True)
    exact = pa.sage_attn_fwd_ex(q, k, v, causal=causal)
    torch.cuda.synchronize()
    # Same bars as the default path.  The scores now differ from the oracle's in their last bits, so more codes of
    # P~ can come out one step away; the ones that can are those whose value lies within the FP32 dot-product bound of
    # Delta-S (times ln 2: a difference in the base-2 score is that relative difference in 2^score) of a rounding
    # boundary, and a row beyond a bar must be explained by moving one or two of exactly those.
    u = 2.0 ** -24

    def ds_width(pro, r):
        gK = (pro_k[id(pro)] - pro["kbar"][None, :]).astype(np.float32)
        mag = float(pro["kappa"]) * (np.abs(pro["qbar"][r // 128]).astype(np.float64) @ np.abs(gK).astype(np.float64).T)
        return np.log(2.0) * ((d + 2) * u * mag + np.spacing(np.abs(pro["delta_s"][r // 128]).astype(np.float64)))

    pro_k = {}
    chk = parity.OutputCheck(dtype, "FP32 Delta-S: ", near=ds_width)
    got16 = wl.from_torch(out)
    for b in range(spec.B):
        for h in range(H):
            pro = so.quantize_head(data["q"][b, h], data["k"][b, h // g], data["v"][b, h // g])
            pro_k[id(pro)] = data["k"][b, h // g]
            chk.add_head(got16[b, h], pro, causal)
    chk.finish()
    # and against the default path the outputs agree to the same bar, but for the rows with such a code
    r = wl.from_torch(exact).astype(np.float64).reshape(-1, d)
    linf = np.abs(r).max(axis=1, keepdims=True)
    d2 = np.abs(got16.astype(np.float64).reshape(-1, d) - r)
    assert (d2.max(axis=1) > 2 * OUT_TOL * linf[:, 0] + 2 * _half_ulp16(r, dtype).max(axis=1)).mean() <= 0.005


# ---- statistics of K and V supplied by the caller (the producer of K and V, or the keeper of a KV cache) ----
@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("N,Nk,d,dtype,H,Hkv,causal,pv", [(300, 300, 128, "bf16", 4, 2, True, "e4m3"),
                                                       (200, 450, 64, "fp16", 2, 2, False, "e5m2")])
def test_supplied_kv_statistics(N, Nk, d, dtype, H, Hkv, causal, pv, mode):
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, B=2, causal=causal).with_(N_kv=Nk)
    data, (q, k, v) = _gpu_inputs(spec)
    print(f"supplied statistics N={N} N_kv={Nk} d={d} {dtype} H={H}/{Hkv} causal={causal} {pv} mode={mode}", flush=True)
    km, vs = pa.sage_attn_kv_stats(k, v, pv_format=pv)
    torch.cuda.synchronize()
    for b in range(2):
        for hk in range(Hkv):
            pro = so.quantize_head(data["q"][b, hk * (H // Hkv)], data["k"][b, hk], data["v"][b, hk], mode=mode, pv_fmt=pv)
            assert np.array_equal(km[b, hk].cpu().numpy(), pro["kbar"]), "mean(K)"
            assert np.array_equal(vs[b, hk].cpu().numpy(), pro["v_scale"]), "delta_V"
    plain, lse0 = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, pv_format=pv, return_lse=True)
    out, lse1 = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, pv_format=pv, return_lse=True, kv_stats=(km, vs))
    torch.cuda.synchronize()
    assert torch.equal(out, plain) and torch.equal(lse0, lse1)      # the same path minus the statistics pass
    # the arrays are read, not copied: other values give another result
    out2 = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, pv_format=pv, kv_stats=(km + 0.25, vs))
    torch.cuda.synchronize()
    assert not torch.equal(out2, plain)
    # one array without the other, or together with an option that needs more statistics
    a = pa.make_args(q, k, v, torch.empty_like(q), causal=causal, mode=mode, pv_format=pv, kv_stats=(km, vs))
    ws = torch.empty(pa.sage_attn_workspace_bytes(a), dtype=torch.uint8, device=q.device)
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
    lib = pa.load_library()
    a.v_scale_in = 0
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -1
    a.v_scale_in = vs.data_ptr()
    a.flags = 1
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -2
    a.flags = 0
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("d,dtype,pv", [(128, "bf16", "e4m3"), (64, "fp16", "e5m2"), (256, "bf16", "e4m3")])
def test_running_kv_statistics_of_a_growing_cache(d, dtype, pv):
    """Statistics kept as running state while K and V grow chunk by chunk: after every chunk mean(K) and delta_V equal
    the oracle's on the prefix, bit for bit, and at the end the one-pass statistics; attention with them equals the
    plain call."""
    pa = _pa()
    N, Nk, H, Hkv = 40, 1501, 4, 2
    spec = _spec(N, d, dtype, H, Hkv, B=2, causal=True).with_(N_kv=Nk)
    data, (q, k, v) = _gpu_inputs(spec)
    state, n = None, 0
    for n_new in (700, 800, 1):
        km, vs, state = pa.sage_attn_kv_stats_update(k[:, :, n:n + n_new].contiguous(), v[:, :, n:n + n_new].contiguous(),
                                                     state, pv_format=pv)
        n += n_new
        torch.cuda.synchronize()
        assert state[2] == n
        for b in range(2):
            for hk in range(Hkv):
                kbar = so.token_mean(data["k"][b, hk][:n])
                dv = so.quantize_v(data["v"][b, hk][:n], pv)[0]
                assert np.array_equal(km[b, hk].cpu().numpy(), kbar), f"mean(K) of the first {n} tokens"
                assert np.array_equal(vs[b, hk].cpu().numpy(), dv), f"delta_V of the first {n} tokens"
    km1, vs1 = pa.sage_attn_kv_stats(k, v, pv_format=pv)
    torch.cuda.synchronize()
    assert torch.equal(km, km1) and torch.equal(vs, vs1)
    plain = pa.sage_attn_fwd_ex(q, k, v, causal=True, pv_format=pv)
    out = pa.sage_attn_fwd_ex(q, k, v, causal=True, pv_format=pv, kv_stats=(km, vs))
    torch.cuda.synchronize()
    assert torch.equal(out, plain)


def test_supplied_kv_statistics_of_a_packed_batch():
    pa = _pa()
    lens_q, lens_k, H, Hkv, d = [70, 200, 129], [300, 64, 129], 4, 2, 128
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(5)
    tq, tk = sum(lens_q), sum(lens_k)
    q = torch.tensor(rng.standard_normal((tq, H, d)), dtype=torch.bfloat16, device=dev)
    k = torch.tensor(rng.standard_normal((tk, Hkv, d)) + 2.0, dtype=torch.bfloat16, device=dev)
    v = torch.tensor(rng.standard_normal((tk, Hkv, d)), dtype=torch.bfloat16, device=dev)
    cu = lambda lens: torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=dev)
    cu_q, cu_k = cu(lens_q), cu(lens_k)
    km, vs = pa.sage_attn_kv_stats(k, v, cu_seqlens_k=cu_k, max_seqlen_k=max(lens_k))
    assert km.shape == (3, Hkv, d)
    plain = pa.sage_attn_fwd_ex(q, k, v, cu_seqlens_q=cu_q, cu_seqlens_k=cu_k)
    out = pa.sage_attn_fwd_ex(q, k, v, cu_seqlens_q=cu_q, cu_seqlens_k=cu_k, kv_stats=(km, vs))
    torch.cuda.synchronize()
    assert torch.equal(out, plain)
    # sequence 1's mean is that of its own 64 keys
    ref = k[300:364, 1].float().double().sum(dim=0) / 64
    assert torch.equal(km[1, 1].cpu(), ref.float().cpu())


# ---- per-block and per-tensor granularity (Sec. 2.2 / 2.3 / 3.2: the coarser groupings the paper compares with) ----
@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("group_map,gmap", [("block", "per_block"), ("tensor", "per_tensor")])
@pytest.mark.parametrize("N,d,dtype,H,Hkv,causal", [(333, 128, "bf16", 2, 1, True), (640, 64, "fp16", 2, 2, False)])
def test_coarser_groups_match_oracle(N, d, dtype, H, Hkv, causal, group_map, gmap, mode):
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, causal=causal, outliers=2)
    data, (q, k, v) = _gpu_inputs(spec)
    print(f"{group_map} case N={N} d={d} {dtype} H={H}/{Hkv} causal={causal} mode={mode}", flush=True)
    got, args, ws = pa.sage_attn_quant(q, k, v, causal=causal, mode=mode, group_map=group_map,
                                       want=("q_codes", "k_codes", "q_scale", "k_scale"))
    out = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, group_map=group_map)
    fine = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode)
    torch.cuda.synchronize()
    got = {n: t.cpu().numpy() for n, t in got.items()}
    g = H // Hkv
    for h in range(H):
        pro = so.quantize_head(data["q"][0, h], data["k"][0, h // g], data["v"][0, h // g], mode=mode,
                               gmap=gmap)
        assert np.array_equal(got["q_codes"][0, h], pro["q_codes"]), "q codes"
        assert np.array_equal(got["k_codes"][0, h // g], pro["k_codes"]), "k codes"
        # the library keeps its scale arrays' shapes: one entry per query pair / per 16 keys
        assert np.array_equal(got["q_scale"][0, h], pro["q_scale"][pro["q_groups"][::2]]), "q scales"
        assert np.array_equal(got["k_scale"][0, h // g], pro["k_scale"][pro["k_groups"][::16]]), "k scales"
    parity.check_heads(wl.from_torch(out), data, causal, mode, dtype, gmap=gmap)
    full = np.stack([so.ref_attn_fp64(data["q"][0, h], data["k"][0, h // g], data["v"][0, h // g], causal)
                     for h in range(H)])
    e_b, e_f = wl.rel_l1(wl.from_torch(out)[0], full), wl.rel_l1(wl.from_torch(fine)[0], full)
    print(f"  rel-L1 vs FP64 attention: {group_map} {e_b:.4f}, default groups {e_f:.4f}", flush=True)
    assert e_f <= e_b * 1.02      # finer groups are not worse (the paper's granularity table)


# ---- finer granularities: every query its own scale, keys in runs of 4 ("fine") or one by one ("token") ----
@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("group_map,gmap", [("fine", "fine"), ("token", "per_token")])
@pytest.mark.parametrize("N,d,dtype,H,Hkv,causal", [(333, 128, "bf16", 2, 1, True), (640, 64, "fp16", 2, 2, False)])
def test_finer_groups_match_oracle(N, d, dtype, H, Hkv, causal, group_map, gmap, mode):
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, causal=causal, outliers=2)
    data, (q, k, v) = _gpu_inputs(spec)
    print(f"{group_map} case N={N} d={d} {dtype} H={H}/{Hkv} causal={causal} mode={mode}", flush=True)
    got, args, ws = pa.sage_attn_quant(q, k, v, causal=causal, mode=mode, group_map=group_map,
                                       want=("q_codes", "k_codes", "q_scale", "k_scale"))
    out = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, group_map=group_map)
    lane = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode)
    torch.cuda.synchronize()
    got = {n: t.cpu().numpy() for n, t in got.items()}
    g = H // Hkv
    for h in range(H):
        pro = so.quantize_head(data["q"][0, h], data["k"][0, h // g], data["v"][0, h // g], mode=mode, gmap=gmap)
        assert np.array_equal(got["q_codes"][0, h], pro["q_codes"]), "q codes"
        assert np.array_equal(got["k_codes"][0, h // g], pro["k_codes"]), "k codes"
        assert np.array_equal(got["q_scale"][0, h], pro["q_scale"]), "q scales"
        assert np.array_equal(got["k_scale"][0, h // g], pro["k_scale"]), "k scales"
    parity.check_heads(wl.from_torch(out), data, causal, mode, dtype, gmap=gmap)
    full = np.stack([so.ref_attn_fp64(data["q"][0, h], data["k"][0, h // g], data["v"][0, h // g], causal)
                     for h in range(H)])
    e_f, e_l = wl.rel_l1(wl.from_torch(out)[0], full), wl.rel_l1(wl.from_torch(lane)[0], full)
    print(f"  rel-L1 vs FP64 attention: {group_map} {e_f:.4f}, default groups {e_l:.4f}", flush=True)
    assert e_f <= e_l * 1.02      # finer groups are not worse (the paper's granularity table)


# ---- E5M2 or INT8 instead of E4M3 for P~ and V (the other data types of the paper's comparison) ----
@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("pv", ["e5m2", "int8"])
@pytest.mark.parametrize("N,d,dtype,H,Hkv,causal", [(333, 128, "bf16", 2, 1, True), (640, 64, "fp16", 2, 2, False)])
def test_other_pv_data_types_match_oracle(N, d, dtype, H, Hkv, causal, pv, mode):
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, causal=causal)
    data, (q, k, v) = _gpu_inputs(spec)
    print(f"{pv} case N={N} d={d} {dtype} H={H}/{Hkv} causal={causal} mode={mode}", flush=True)
    got, args, ws = pa.sage_attn_quant(q, k, v, causal=causal, mode=mode, pv_format=pv, want=("v_codes", "v_scale"))
    out = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, pv_format=pv)
    e4 = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode)
    torch.cuda.synchronize()
    g = H // Hkv
    for h in range(Hkv):
        pro = so.quantize_head(data["q"][0, h * g], data["k"][0, h], data["v"][0, h], mode=mode, pv_fmt=pv)
        assert np.array_equal(got["v_scale"][0, h].cpu().numpy(), pro["v_scale"]), "v scales"
        assert np.array_equal(got["v_codes"][0, h].cpu().numpy(), pro["v_codes"].view(np.uint8)), "v codes"
    parity.check_heads(wl.from_torch(out), data, causal, mode, dtype, pv_fmt=pv)
    if mode == "int8_fp8" and pv == "e5m2":   # where the FP8 stage dominates the error, E4M3 is the better format (Sec. 3.3)
        full = np.stack([so.ref_attn_fp64(data["q"][0, h], data["k"][0, h // g], data["v"][0, h // g], causal)
                         for h in range(H)])
        assert wl.rel_l1(wl.from_torch(e4)[0], full) < wl.rel_l1(wl.from_torch(out)[0], full)


# ---- key length different from query length (cross attention, chunked prefill, decode) ---------
CROSS_CASES = [
    # N, N_kv, d, dtype, H, Hkv, causal
    (200, 333, 128, "bf16", 2, 1, False),
    (333, 70, 64, "fp16", 2, 2, False),       # fewer keys than queries
    (130, 640, 128, "bf16", 2, 2, True),      # chunked prefill: the last 130 queries of 640 tokens
    (1, 300, 128, "bf16", 4, 1, True),        # one decode step
]


@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("N,Nk,d,dtype,H,Hkv,causal", CROSS_CASES)
def test_other_key_length_matches_oracle(N, Nk, d, dtype, H, Hkv, causal, mode):
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, causal=causal).with_(N_kv=Nk)
    data, (q, k, v) = _gpu_inputs(spec)
    assert k.shape[2] == Nk and q.shape[2] == N
    print(f"cross case N={N} N_kv={Nk} d={d} {dtype} H={H}/{Hkv} causal={causal} mode={mode}", flush=True)
    got, args, ws = pa.sage_attn_quant(q, k, v, causal=causal, mode=mode)
    out = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode)
    torch.cuda.synchronize()
    got = {n: t.cpu().numpy() for n, t in got.items()}
    g = H // Hkv
    for h in range(H):
        pro = so.quantize_head(data["q"][0, h], data["k"][0, h // g], data["v"][0, h // g], mode=mode)
        assert np.array_equal(got["q_codes"][0, h], pro["q_codes"]), "q codes"
        assert np.array_equal(got["q_scale"][0, h], pro["q_scale"]), "q scales"
        assert np.array_equal(got["k_codes"][0, h // g], pro["k_codes"]), "k codes"
        assert np.array_equal(got["k_scale"][0, h // g], pro["k_scale"]), "k scales"
        assert np.array_equal(got["v_codes"][0, h // g], pro["v_codes"]), "v codes"
        assert np.array_equal(got["k_mean"][0, h // g], pro["kbar"]), "k mean"
        if mode == "int4_fp8":
            D = pro["delta_s"].astype(np.float64)
            diff = np.abs(got["delta_s"][0, h].astype(np.float64) - D)
            assert np.all(diff <= np.spacing(np.abs(D.astype(np.float32))).astype(np.float64)), "delta S"   # one unit of the FP32 value's last place
    parity.check_heads(wl.from_torch(out), data, causal, mode, dtype)
    full = np.stack([so.ref_attn_fp64(data["q"][0, h], data["k"][0, h // g], data["v"][0, h // g], causal)
                     for h in range(H)])
    assert wl.cos_sim(wl.from_torch(out)[0], full) > (0.9 if mode == "int4_fp8" else 0.99)


# ---- key range of a tile split over several workgroups (decode steps, few queries against a long cache) ----------
SPLIT_CASES = [
    # N, N_kv, d, dtype, H, Hkv, causal, kv_splits (0: the library decides)
    (1, 1500, 128, "bf16", 4, 1, True, 0),        # one decode step
    (32, 2000, 128, "bf16", 2, 2, True, 4),       # a short chunk of queries at the end of a cache
    (130, 1100, 64, "fp16", 2, 1, False, 3),      # two query tiles, the second one ragged
    (7, 1700, 256, "bf16", 2, 2, True, 0),
    (200, 1030, 128, "bf16", 1, 1, True, 5),      # chunks of different lengths per tile, a diagonal inside the last one
    # grouped KV heads, all queries of a group within 128: the group's query heads share one tile
    (1, 2100, 128, "bf16", 8, 1, True, 0),        # a decode step, 8 query heads per KV head
    (16, 1600, 64, "fp16", 4, 2, True, 0),        # 2 heads x 16 queries: one wavefront's columns
    (32, 1100, 128, "bf16", 4, 1, False, 2),      # 4 heads x 32 queries: the whole tile
    (5, 1100, 256, "bf16", 6, 2, True, 0),        # 3 heads x 5 queries
    (40, 1300, 128, "fp16", 3, 1, True, 4),       # 3 heads x 40 queries: heads straddle the wavefronts' column ranges
]


@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("N,Nk,d,dtype,H,Hkv,causal,kv_splits", SPLIT_CASES)
def test_split_key_range_matches_oracle(N, Nk, d, dtype, H, Hkv, causal, kv_splits, mode):
    """Every chunk is Algorithm 1 on its key blocks; the merge is Eq. 1's rule for disjoint key sets.  The oracle walks
    the same chunks (oracle.key_chunks mirrors the documented rule) and merges them in float64."""
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, B=2, causal=causal).with_(N_kv=Nk)
    data, (q, k, v) = _gpu_inputs(spec)
    S = pa.sage_attn_kv_splits(pa.make_args(q, k, v, causal=causal, mode=mode, kv_splits=kv_splits))
    print(f"split case N={N} N_kv={Nk} d={d} {dtype} H={H}/{Hkv} causal={causal} mode={mode}: {S} chunks per tile", flush=True)
    assert S > 1 and (kv_splits == 0 or S == min(kv_splits, ((Nk + 63) // 64) // 8))     # at least 8 key blocks per chunk
    out, lse = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, kv_splits=kv_splits, return_lse=True)
    whole = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, kv_splits=1)
    torch.cuda.synchronize()
    pros = parity.check_heads(wl.from_torch(out), data, causal, mode, dtype, want_lse=True, splits=S)
    for b in range(2):
        for h in range(H):
            _lse_close(lse[b, h].cpu().numpy(), pros[b][h]["lse"], pros[b][h])
    # the unsplit path is checked against the unsplit oracle, and both approximate the same attention
    parity.check_heads(wl.from_torch(whole), data, causal, mode, dtype)
    g = H // Hkv
    full = np.stack([so.ref_attn_fp64(data["q"][0, h], data["k"][0, h // g], data["v"][0, h // g], causal) for h in range(H)])
    e_split, e_whole = wl.rel_l1(wl.from_torch(out)[0], full), wl.rel_l1(wl.from_torch(whole)[0], full)
    print(f"  rel-L1 vs FP64 attention: split {e_split:.4f}, one piece {e_whole:.4f}", flush=True)
    assert e_split < 1.3 * e_whole + 1e-3


def test_split_key_range_is_refused_where_it_does_not_apply():
    pa = _pa()
    spec = _spec(16, 128, "bf16", 2, 2).with_(N_kv=2048)
    _, (q, k, v) = _gpu_inputs(spec)
    assert pa.sage_attn_kv_splits(pa.make_args(q, k, v)) > 1                        # few tiles, many keys: split
    assert pa.sage_attn_kv_splits(pa.make_args(q, k, v, kv_splits=1)) == 1          # switched off
    assert pa.sage_attn_kv_splits(pa.make_args(q, k, v, group_map="fine")) == 1     # default groups only
    assert pa.sage_attn_kv_splits(pa.make_args(q, k, v, pv_format="e5m2")) == 1
    a = pa.make_args(q, k, v, torch.empty_like(q), kv_splits=65)
    assert pa.sage_attn_workspace_bytes(a) == 0
    big = _spec(4096, 128, "bf16", 8, 8)                                             # 256 tiles: no split (shapes only)
    a = pa.make_args(q, k, v)
    a.N, a.N_kv, a.H, a.H_kv = 4096, 4096, 8, 8
    assert pa.sage_attn_kv_splits(a) == 1


# ---- [B, N, H, d] memory order ------------------------------------------------------------------
@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("N,Nk,d,H,Hkv,causal", [(333, 333, 128, 4, 2, True), (200, 450, 64, 2, 2, False)])
def test_nhd_layout_equals_hnd(N, Nk, d, H, Hkv, causal, mode):
    """The same tensors handed over token-major give bit-identical results (the workspace layouts and
    the arithmetic do not depend on the memory order of the inputs)."""
    pa = _pa()
    spec = _spec(N, d, "bf16", H, Hkv, B=2, causal=causal).with_(N_kv=Nk)
    _, (q, k, v) = _gpu_inputs(spec)
    ref = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode)
    qn, kn, vn = (t.permute(0, 2, 1, 3).contiguous() for t in (q, k, v))
    out = pa.sage_attn_fwd_ex(qn, kn, vn, causal=causal, mode=mode, layout="NHD")
    torch.cuda.synchronize()
    assert out.shape == qn.shape
    assert torch.equal(out.permute(0, 2, 1, 3), ref)


# ---- packed variable-length batches ---------------------------------------------------------------
def _packed_batch(lens_q, lens_k, d, dtype, H, Hkv, causal):
    """Sequences of the given lengths, each drawn like a one-sequence workload, packed along the token
    axis: q [total_q, H, d], k / v [total_k, H_kv, d] on the GPU, plus the per-sequence numpy arrays."""
    seqs, qs, ks, vs = [], [], [], []
    for i, (n, nk) in enumerate(zip(lens_q, lens_k)):
        spec = _spec(max(n, 1), d, dtype, H, Hkv, causal=causal, cfg=120 + i).with_(N_kv=max(nk, 1))
        data = wl.make_inputs(spec, seed=i)
        qn, kn, vn = data["q"][0][:, :n], data["k"][0][:, :nk], data["v"][0][:, :nk]     # [heads, tokens, d]
        seqs.append((qn, kn, vn))
        qs.append(qn.transpose(1, 0, 2)); ks.append(kn.transpose(1, 0, 2)); vs.append(vn.transpose(1, 0, 2))
    dev = torch.device("cuda:0")
    pack = lambda parts: wl.to_torch(np.ascontiguousarray(np.concatenate(parts, axis=0)), dtype, dev)
    cu = lambda lens: torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=dev)
    return seqs, pack(qs), pack(ks), pack(vs), cu(lens_q), cu(lens_k)


VARLEN_CASES = [
    # lens_q, lens_k, d, dtype, H, Hkv, causal
    ([200, 1, 333, 128], [200, 1, 333, 128], 128, "bf16", 4, 2, True),      # self attention, ragged, grouped KV heads
    ([200, 1, 333, 128], [260, 5, 333, 640], 64, "fp16", 2, 2, True),       # more keys than queries per sequence
    ([70, 300, 0, 129], [500, 64, 40, 1], 128, "bf16", 2, 1, False),        # cross lengths, a sequence without queries
    ([50, 120], [0, 90], 64, "bf16", 2, 2, False),                          # a sequence without keys: zeros
]


@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("lens_q,lens_k,d,dtype,H,Hkv,causal", VARLEN_CASES)
def test_varlen_batch_equals_one_sequence_at_a_time(lens_q, lens_k, d, dtype, H, Hkv, causal, mode):
    """Every sequence of a packed batch must come out exactly as when it is passed alone (same kernels,
    same arithmetic: bit-identical), and one of them is checked against the oracle."""
    pa = _pa()
    seqs, q, k, v, cu_q, cu_k = _packed_batch(lens_q, lens_k, d, dtype, H, Hkv, causal)
    print(f"varlen case q={lens_q} k={lens_k} d={d} {dtype} H={H}/{Hkv} causal={causal} mode={mode}", flush=True)
    same = lens_q == lens_k
    out = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, cu_seqlens_q=cu_q, cu_seqlens_k=None if same else cu_k)
    torch.cuda.synchronize()
    assert out.shape == q.shape
    oq, ok = np.concatenate([[0], np.cumsum(lens_q)]), np.concatenate([[0], np.cumsum(lens_k)])
    checked = False
    for b, (n, nk) in enumerate(zip(lens_q, lens_k)):
        part = out[oq[b]:oq[b + 1]]
        if n == 0:
            continue
        if nk == 0:
            assert torch.count_nonzero(part) == 0
            continue
        alone = pa.sage_attn_fwd_ex(q[oq[b]:oq[b + 1]].unsqueeze(0).contiguous(), k[ok[b]:ok[b + 1]].unsqueeze(0).contiguous(),
                                    v[ok[b]:ok[b + 1]].unsqueeze(0).contiguous(), causal=causal, mode=mode, layout="NHD")
        torch.cuda.synchronize()
        assert torch.equal(alone[0], part), f"sequence {b}"
        if not checked and n >= 100:
            qn, kn, vn = seqs[b]
            parity.check_heads(wl.from_torch(part).transpose(1, 0, 2)[None], dict(q=qn[None], k=kn[None], v=vn[None]),
                               causal, mode, dtype)
            checked = True
    assert checked


PACKED_DECODE_CASES = [
    # lens_q, lens_k, d, dtype, H, Hkv, causal, kv_splits: few queries per sequence on grouped KV heads - the query heads
    # of a KV head share one tile per sequence
    ([1, 1, 1, 1], [1100, 1300, 2048, 70], 128, "bf16", 8, 2, True, 2),            # decode steps against caches of different lengths
    ([3, 8, 0, 1, 5], [1500, 1200, 900, 0, 1024], 64, "fp16", 4, 2, True, 2),      # a sequence without queries, one without keys
    ([16, 2], [640, 1280], 128, "bf16", 6, 2, False, 2),
]


@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("lens_q,lens_k,d,dtype,H,Hkv,causal,kv_splits", PACKED_DECODE_CASES)
def test_varlen_batch_of_short_queries_on_grouped_kv_heads(lens_q, lens_k, d, dtype, H, Hkv, causal, kv_splits, mode):
    """Every sequence against the oracle walking the same key chunks, and bit-identical to the sequence passed alone
    where the chunk count of the two calls is the same (enough key blocks for it in the sequence itself)."""
    pa = _pa()
    seqs, q, k, v, cu_q, cu_k = _packed_batch(lens_q, lens_k, d, dtype, H, Hkv, causal)
    S = min(kv_splits, ((max(lens_k) + 63) // 64) // 8)
    assert S >= 2 and (H // Hkv) * max(lens_q) <= 128
    print(f"packed decode case q={lens_q} k={lens_k} d={d} {dtype} H={H}/{Hkv} causal={causal} mode={mode}: {S} chunks", flush=True)
    out, lse = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, cu_seqlens_q=cu_q, cu_seqlens_k=cu_k, kv_splits=kv_splits,
                                   return_lse=True)
    torch.cuda.synchronize()
    oq, ok = np.concatenate([[0], np.cumsum(lens_q)]), np.concatenate([[0], np.cumsum(lens_k)])
    for b, (n, nk) in enumerate(zip(lens_q, lens_k)):
        part = out[oq[b]:oq[b + 1]]
        if n == 0:
            continue
        if nk == 0:
            assert torch.count_nonzero(part) == 0
            continue
        qn, kn, vn = seqs[b]
        pros = parity.check_heads(wl.from_torch(part).transpose(1, 0, 2)[None], dict(q=qn[None], k=kn[None], v=vn[None]),
                                  causal, mode, dtype, want_lse=True, splits=S)
        for h in range(H):
            _lse_close(lse[h, oq[b]:oq[b + 1]].cpu().numpy(), pros[0][h]["lse"], pros[0][h])
        if (nk + 63) // 64 >= 8 * kv_splits:
            alone = pa.sage_attn_fwd_ex(q[oq[b]:oq[b + 1]].unsqueeze(0).contiguous(), k[ok[b]:ok[b + 1]].unsqueeze(0).contiguous(),
                                        v[ok[b]:ok[b + 1]].unsqueeze(0).contiguous(), causal=causal, mode=mode, layout="NHD",
                                        kv_splits=kv_splits)
            torch.cuda.synchronize()
            assert torch.equal(alone[0], part), f"sequence {b}"


# ---- row log-sum-exp (the weight for merging results over disjoint key sets) ---------------------
LSE_CASES = [
    # N, N_kv, d, dtype, H, Hkv, causal
    (333, 333, 128, "bf16", 2, 1, True),
    (640, 640, 64, "fp16", 2, 2, False),
    (130, 500, 128, "bf16", 2, 2, True),
]


def _lse_close(got, ref, pro=None):
    """Both sides round the same real number to FP32 after a few FP32 operations (running sum in another order,
    hardware log2 to 1 ulp, the row constant kappa <q, mean(K)> stored as FP32): a few units of the last place of
    the largest TERM, which is not the result when the running maximum and the row constant cancel (inputs
    with a large common offset); with `pro` (the oracle's record of the head) the row constant is taken into
    the scale of the tolerance."""
    big = np.abs(ref).astype(np.float64)
    if pro is not None:
        corr = np.log(2.0) * float(pro["kappa"]) * (pro["Q"].astype(np.float64) @ pro["kbar"].astype(np.float64))
        big = np.maximum(big, np.maximum(np.abs(corr), np.abs(ref.astype(np.float64) - corr)))
    tol = 1e-5 * np.maximum(1.0, big) + 1e-5
    assert np.all(np.abs(got.astype(np.float64) - ref.astype(np.float64)) <= tol), \
        f"worst {np.abs(got - ref).max():.3e}"


@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("N,Nk,d,dtype,H,Hkv,causal", LSE_CASES)
def test_lse_matches_oracle(N, Nk, d, dtype, H, Hkv, causal, mode):
    pa = _pa()
    spec = _spec(N, d, dtype, H, Hkv, B=2, causal=causal).with_(N_kv=Nk)
    data, (q, k, v) = _gpu_inputs(spec)
    print(f"lse case N={N} N_kv={Nk} d={d} {dtype} H={H}/{Hkv} causal={causal} mode={mode}", flush=True)
    plain = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode)
    out, lse = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, return_lse=True)
    torch.cuda.synchronize()
    assert torch.equal(out, plain)                      # asking for it changes nothing else
    assert lse.shape == (2, H, N)
    pros = parity.check_heads(wl.from_torch(out), data, causal, mode, dtype, want_lse=True)
    for b in range(2):
        for h in range(H):
            _lse_close(lse[b, h].cpu().numpy(), pros[b][h]["lse"], pros[b][h])
    full = so.ref_lse_fp64(data["q"][1, 0], data["k"][1, 0], causal=causal)
    assert np.abs(lse[1, 0].cpu().numpy() - full).max() < (1.0 if mode == "int4_fp8" else 0.1)


def test_lse_of_a_packed_batch_and_merge_of_key_halves():
    """[H, total_q] layout for a variable-length batch; and the use the statistic exists for: the keys of
    every sequence split in two, both parts attended separately, merged with their lse."""
    pa = _pa()
    lens = [200, 77, 333]
    seqs, q, k, v, cu_q, _ = _packed_batch(lens, lens, 128, "bf16", 4, 2, False)
    out, lse = pa.sage_attn_fwd_ex(q, k, v, mode="int8_fp8", cu_seqlens_q=cu_q, return_lse=True)
    torch.cuda.synchronize()
    assert lse.shape == (4, sum(lens))
    off = np.concatenate([[0], np.cumsum(lens)])
    for b, n in enumerate(lens):
        sl = slice(off[b], off[b + 1])
        o1, l1 = pa.sage_attn_fwd_ex(q[sl].unsqueeze(0).contiguous(), k[sl].unsqueeze(0).contiguous(),
                                     v[sl].unsqueeze(0).contiguous(), mode="int8_fp8", layout="NHD", return_lse=True)
        torch.cuda.synchronize()
        assert torch.equal(l1[0], lse[:, sl]) and torch.equal(o1[0], out[sl])
        # two key halves of sequence b, merged
        parts = []
        for a0, a1 in ((0, n // 2), (n // 2, n)):
            ks = k[off[b] + a0:off[b] + a1].unsqueeze(0).contiguous()
            vs = v[off[b] + a0:off[b] + a1].unsqueeze(0).contiguous()
            parts.append(pa.sage_attn_fwd_ex(q[sl].unsqueeze(0).contiguous(), ks, vs, mode="int8_fp8", layout="NHD",
                                             return_lse=True))
        torch.cuda.synchronize()
        ls = torch.stack([p[1][0] for p in parts]).double()                # [2, H, n]
        tot = torch.logsumexp(ls, dim=0)
        merged = sum(torch.exp(l - tot).transpose(0, 1)[..., None] * p[0][0].double() for l, p in zip(ls, parts))
        qn, kn, vn = seqs[b]
        full = np.stack([so.ref_attn_fp64(qn[h], kn[h // 2], vn[h // 2]) for h in range(4)])   # [H, n, d]
        got = merged.cpu().numpy().transpose(1, 0, 2)
        whole = wl.from_torch(out[sl]).transpose(1, 0, 2)
        assert wl.cos_sim(got, full) > 0.997
        assert wl.rel_l1(got, full) < 1.5 * wl.rel_l1(whole, full) + 1e-3
        lse_full = np.stack([so.ref_lse_fp64(qn[h], kn[h // 2]) for h in range(4)])
        assert np.abs(tot.cpu().numpy() - lse_full).max() < 0.1


def test_plain_signature_and_repeatability():
    pa = _pa()
    spec = _spec(384, 128, "bf16", 2, 2)
    data, (q, k, v) = _gpu_inputs(spec)
    out1 = torch.empty_like(q)
    out2 = torch.full_like(q, 7.0)
    pa.sage_attn_fwd(q, k, v, out1, causal=True, mode="int4_fp8")
    pa.sage_attn_fwd(q, k, v, out2, causal=True, mode="int4_fp8")
    torch.cuda.synchronize()
    assert torch.equal(out1, out2)                       # deterministic
    ref = pa.sage_attn_fwd_ex(q, k, v, causal=True, mode="int4_fp8")
    torch.cuda.synchronize()
    assert torch.equal(out1, ref)                        # both entry points agree
    pa.sage_attn_release()


def test_error_codes_from_the_boundary():
    pa = _pa()
    spec = _spec(128, 64, "bf16", 2, 2)
    _, (q, k, v) = _gpu_inputs(spec)
    a = pa.make_args(q, k, v, torch.empty_like(q))
    lib = pa.load_library()
    import ctypes
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -3          # no workspace
    a.d = 96
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -2          # unsupported head dim
    assert pa.sage_attn_workspace_bytes(a) == 0
    a.d = 64; a.H_kv = 3
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -1          # H % H_kv != 0
    a.H_kv = 2; a.q = 0
    ws = torch.empty(1 << 22, dtype=torch.uint8, device="cuda")
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -1          # null pointer
    a.q = q.data_ptr(); a.workspace_bytes = 1024
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -3          # workspace too small
    a.workspace_bytes = ws.numel(); a.mode = 5
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -2
    a.mode = 0; a.causal = 1; a.N_kv = a.N - 1
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -2          # causal mask with fewer keys than queries
    a.N_kv = -3
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -1


def test_side_stream_and_workspace_reuse():
    """Work is enqueued on the stream the caller names; one workspace serves consecutive calls on
    that stream (different shapes, the larger first), and the results equal the default-stream ones."""
    pa = _pa()
    big, small = _spec(640, 128, "bf16", 2, 2), _spec(250, 128, "bf16", 2, 2, causal=True)
    _, (qb, kb, vb) = _gpu_inputs(big)
    _, (qs, ks, vs) = _gpu_inputs(small, seed=1)
    ref_b = pa.sage_attn_fwd_ex(qb, kb, vb)
    ref_s = pa.sage_attn_fwd_ex(qs, ks, vs, causal=True)
    torch.cuda.synchronize()
    ws = torch.empty(pa.sage_attn_workspace_bytes(pa.make_args(qb, kb, vb)), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        out_b = pa.sage_attn_fwd_ex(qb, kb, vb, workspace=ws, stream=side)
        out_s = pa.sage_attn_fwd_ex(qs, ks, vs, causal=True, workspace=ws, stream=side)
        out_b2 = pa.sage_attn_fwd_ex(qb, kb, vb, workspace=ws, stream=side)
    side.synchronize()
    assert torch.equal(out_b, ref_b) and torch.equal(out_s, ref_s) and torch.equal(out_b2, ref_b)


def test_graph_capture_and_replay():
    """The whole forward pass (caller-provided workspace, no allocation, no host synchronisation)
    can be captured into a HIP graph; every replay, with eager work and synchronisations in between
    and with new input values in the captured buffers, equals the eager result."""
    pa = _pa()
    spec = _spec(333, 128, "bf16", 2, 1, causal=True)
    _, (q, k, v) = _gpu_inputs(spec)
    _, (q2, k2, v2) = _gpu_inputs(spec, seed=3)
    eager1 = pa.sage_attn_fwd_ex(q, k, v, causal=True)
    eager2 = pa.sage_attn_fwd_ex(q2, k2, v2, causal=True)
    torch.cuda.synchronize()
    qg, kg, vg = q.clone(), k.clone(), v.clone()
    out = torch.zeros_like(q)
    ws = torch.empty(pa.sage_attn_workspace_bytes(pa.make_args(qg, kg, vg)), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # one eager run on the capture stream first
        pa.sage_attn_fwd_ex(qg, kg, vg, out=out, causal=True, workspace=ws, stream=side)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pa.sage_attn_fwd_ex(qg, kg, vg, out=out, causal=True, workspace=ws, stream=torch.cuda.current_stream())
    for rep, (src, want) in enumerate([((q, k, v), eager1), ((q2, k2, v2), eager2), ((q, k, v), eager1)]):
        for dst, s in zip((qg, kg, vg), src):
            dst.copy_(s)
        out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"replay {rep}"
        _ = pa.sage_attn_fwd_ex(q2, k2, v2, causal=True)       # eager work between replays
        torch.cuda.synchronize()
