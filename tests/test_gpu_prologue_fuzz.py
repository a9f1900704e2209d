"""Seeded fuzz of the preprocessing alone: random shapes, group maps, P~V data types and smoothing switches on
inputs with awkward values - heads scaled by large and small powers of two, all-zero tokens and channels, values
that repeat (ties at the rounding boundary of the quantizer) - compared bit for bit with the CPU oracle through
sage_attn_quant.  This is where the division-free quantizer's exact fall-back, zero scales and the fragment-order
packing are exercised beyond the fixed cases of tests/test_gpu_parity.py."""
import os

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import sage_oracle as so
from test_gpu_parity import _pa, _delta_s_within_fp32_bound

pytestmark = pytest.mark.gpu

N_SEEDS = int(os.environ.get("SAGE_FUZZ_SEEDS", "32"))
GMAPS = {"lane": "g950", "block": "per_block", "fine": "fine", "token": "per_token", "tensor": "per_tensor"}


_awkward = wl.awkward_values       # seeded generator of awkward inputs (shared with the CPU pins)


@pytest.mark.parametrize("seed", range(N_SEEDS))
def test_preprocessing_fuzz(seed):
    pa = _pa()
    rng = np.random.default_rng(7000 + seed)
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2]))
    H = Hkv * int(rng.choice([1, 2]))
    n = int(rng.choice([1, 2, 15, 16, 17, 63, 64, 65, 127, 128, 129, 200, 300]))
    nk = n if rng.random() < 0.5 else int(rng.choice([1, 3, 16, 31, 64, 100, 129, 260]))
    dtype = str(rng.choice(["bf16", "fp16"]))
    mode = str(rng.choice(["int4_fp8", "int8_fp8"]))
    group_map = str(rng.choice(list(GMAPS)))
    pv = str(rng.choice(["e5m2", "int8"])) if (group_map in ("lane", "block", "tensor") and rng.random() < 0.4) else "e4m3"
    smooth_v = bool(rng.random() < 0.3)
    smooth_k = bool(rng.random() >= 0.25)
    smooth_q = bool(rng.random() >= 0.25)
    fp32_ds = bool(rng.random() < 0.25)          # Delta-S accumulated in FP32: checked against its error bound instead
    # which exact form of the Delta-S product (from a generator of its own, so that the cases stay what they were)
    ds_form = [None, "digits", "fp64"][int(np.random.default_rng(9000 + seed).integers(3))]
    print(f"fuzz {seed}: d={d} H={H}/{Hkv} n={n} nk={nk} {dtype} {mode} {group_map} {pv} smooth v/k/q={smooth_v}/{smooth_k}/{smooth_q} fp32_ds={fp32_ds} ds_form={ds_form}",
          flush=True)
    qn, kn, vn = _awkward(rng, (H, n, d), dtype), _awkward(rng, (Hkv, nk, d), dtype), _awkward(rng, (Hkv, nk, d), dtype)
    dev = torch.device("cuda:0")
    q, k, v = (wl.to_torch(x[None], dtype, dev) for x in (qn, kn, vn))
    got, args, ws = pa.sage_attn_quant(q, k, v, mode=mode, group_map=group_map, pv_format=pv, smooth_v=smooth_v,
                                       smooth_k=smooth_k, smooth_q=smooth_q, fp32_delta_s=fp32_ds, delta_s=ds_form)
    torch.cuda.synchronize()
    got = {name: t.cpu().numpy() for name, t in got.items()}
    g = H // Hkv
    int4 = mode == "int4_fp8"
    for h in range(H):
        pro = so.quantize_head(qn[h], kn[h // g], vn[h // g], mode=mode, gmap=GMAPS[group_map], pv_fmt=pv,
                               smooth_v_on=smooth_v, smooth_k_on=smooth_k, smooth_q_on=smooth_q and int4)
        # the library keeps one scale per stored group (query pair or query; 16, 4 or 1 keys) also for the coarser maps
        qg, kg = (1, 4) if group_map == "fine" else ((1, 1) if group_map == "token" else (2, 16))
        assert np.array_equal(got["q_codes"][0, h], pro["q_codes"]), "q codes"
        assert np.array_equal(got["q_scale"][0, h], pro["q_scale"][pro["q_groups"][::qg]]), "q scales"
        assert np.array_equal(got["k_scale"][0, h // g], pro["k_scale"][pro["k_groups"][::kg]]), "k scales"
        for name, ref in (("k_codes", pro["k_codes"]), ("v_codes", pro["v_codes"]),
                          ("v_scale", pro["v_scale"]), ("k_mean", pro["kbar"])):
            if name == "v_codes" and ref.dtype == np.int8:          # INT8 codes of V: the library hands out the same bytes as unsigned
                ref = ref.view(np.uint8)
            assert np.array_equal(got[name][0, h // g], ref), name
        if smooth_v:
            assert np.array_equal(got["v_mean"][0, h // g], pro["vbar"]), "v mean"
        if int4 and smooth_q:
            assert np.array_equal(got["q_mean"][0, h], pro["qbar"]), "q block means"
            if fp32_ds:
                _delta_s_within_fp32_bound(got["delta_s"][0, h], pro, kn[h // g])
                continue
            D = pro["delta_s"].astype(np.float64)
            diff = np.abs(got["delta_s"][0, h].astype(np.float64) - D)
            assert np.all(diff <= np.spacing(np.abs(D.astype(np.float32))).astype(np.float64)), "delta S"   # one unit of the FP32 value's last place
        elif int4:
            assert not got["delta_s"][0, h].any() and not got["q_mean"][0, h].any()
        # the integer score accumulators of one random (128-query tile, 64-key block) through the kernel's MFMA code
        qt, kb = int(rng.integers((n + 127) // 128)), int(rng.integers((nk + 63) // 64))
        acc = pa.sage_attn_debug_qk(args, 0, h, qt, kb).cpu().numpy()
        ref = so.int_scores(pro["q_codes"][qt * 128:qt * 128 + 128], pro["k_codes"][kb * 64:kb * 64 + 64])
        assert np.array_equal(acc[: ref.shape[0], : ref.shape[1]], ref), "int32 accumulators"
        assert not acc[ref.shape[0]:].any() and not acc[:, ref.shape[1]:].any()
