"""GPU parity at the full sizes of the measured workloads, through the same entry points and
launch configuration that bench.py times.  The whole tensor goes through the HIP path; the
CPU oracle recomputes sampled (batch, head) slices and query blocks - the first, the last
(ragged where N is ragged), blocks straddling the causal diagonal region and a few random
ones - and every sampled element is compared (same bars as tests/test_gpu_parity.py)."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import sage_oracle as so
from oracle import parity
from test_gpu_parity import _pa

pytestmark = pytest.mark.gpu

# workload -> ((batch, head) samples, number of random query blocks besides first/middle/last)
PLAN = {
    "prefill4k": ([(0, 0), (3, 31), (1, 17), (2, 8)], 8),
    "causal8k": ([(0, 0), (0, 21), (0, 31)], 6),
    "causal16k": ([(0, 5), (0, 18)], 5),
    "causal32k": ([(0, 30), (0, 7)], 4),
    "video17k": ([(0, 0), (1, 47), (1, 20)], 6),
    "long128k": ([(0, 2), (0, 29), (0, 12)], 3),
    "causal8k_d256": ([(0, 3), (0, 15)], 5),
}


def _blocks(spec, n_random, rng):
    nqb = (spec.N + 127) // 128
    fixed = {0, nqb // 2, nqb - 1}
    extra = set(int(x) for x in rng.choice(nqb, size=min(n_random, nqb), replace=False))
    return sorted(fixed | extra)


@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
@pytest.mark.parametrize("name", list(PLAN))
def test_full_size_sampled_parity(name, mode):
    pa = _pa()
    spec = wl.CONFIGS[name]
    heads, n_random = PLAN[name]
    rng = np.random.default_rng(1234)
    print(f"workload {name} mode {mode}: generating inputs", flush=True)
    data = wl.make_inputs(spec, seed=0)
    dev = torch.device("cuda:0")
    q, k, v = (wl.to_torch(data[n], spec.dtype, dev) for n in "qkv")
    print("  running the HIP path", flush=True)
    out = pa.sage_attn_fwd_ex(q, k, v, causal=spec.causal, mode=mode)
    torch.cuda.synchronize()
    want = ["q_codes", "k_codes", "v_codes", "q_scale", "k_scale", "v_scale", "k_mean", "q_mean"]
    if name != "long128k":
        want.append("delta_s")      # 17 GB for the long workload: its rows are checked through the output
    quant, args, ws = pa.sage_attn_quant(q, k, v, causal=spec.causal, mode=mode, want=want)
    torch.cuda.synchronize()
    g = spec.H // spec.H_kv
    for (b, h) in heads:
        blocks = _blocks(spec, n_random, rng)
        print(f"  oracle on (b={b}, h={h}), query blocks {blocks}", flush=True)
        Q, K, V = data["q"][b, h], data["k"][b, h // g], data["v"][b, h // g]
        pro = so.quantize_head(Q, K, V, mode=mode, ds_blocks=blocks)
        # preprocessing: bit-exact, whole head (O(N d) data)
        assert np.array_equal(quant["q_codes"][b, h].cpu().numpy(), pro["q_codes"])
        assert np.array_equal(quant["k_codes"][b, h // g].cpu().numpy(), pro["k_codes"])
        assert np.array_equal(quant["v_codes"][b, h // g].cpu().numpy(), pro["v_codes"])
        assert np.array_equal(quant["q_scale"][b, h].cpu().numpy(), pro["q_scale"])
        assert np.array_equal(quant["k_scale"][b, h // g].cpu().numpy(), pro["k_scale"])
        assert np.array_equal(quant["v_scale"][b, h // g].cpu().numpy(), pro["v_scale"])
        assert np.array_equal(quant["k_mean"][b, h // g].cpu().numpy(), pro["kbar"])
        if mode == "int4_fp8":
            assert np.array_equal(quant["q_mean"][b, h].cpu().numpy(), pro["qbar"])
            if "delta_s" in quant:
                got_ds = quant["delta_s"][b, h][blocks].cpu().numpy().astype(np.float64)
                ref_ds = pro["delta_s"][blocks].astype(np.float64)
                # the bar of the small cases: an exact inner product formed another way, one rounding to FP32 - at most
                # the last bit of the FP32 value (its spacing, not that of the float64 copy), and rarely
                diff = np.abs(got_ds - ref_ds)
                if spec.causal:     # rows are computed up to the key a query block's group can see
                    seen = np.arange(spec.N)[None, :] < 4096 * (np.asarray(blocks)[:, None] // 32 + 1)
                    diff = np.where(seen, diff, 0.0)
                assert np.all(diff <= np.spacing(np.abs(pro["delta_s"][blocks])).astype(np.float64))
                assert (diff > 0).mean() < 1e-3
        # int32 score accumulators of a few (query tile, key block) pairs through the MFMA path
        nkb = (spec.N + 63) // 64
        for qt in (blocks[0], blocks[-1]):
            for kb in (0, min(nkb - 1, 2 * qt + 1)):
                acc = pa.sage_attn_debug_qk(args, b, h, qt, kb).cpu().numpy()
                rows = slice(qt * 128, min(qt * 128 + 128, spec.N))
                keys = slice(kb * 64, min(kb * 64 + 64, spec.N))
                ref = so.int_scores(pro["q_codes"][rows], pro["k_codes"][keys])
                assert np.array_equal(acc[: ref.shape[0], : ref.shape[1]], ref)
        # outputs of the sampled query blocks
        chk = parity.OutputCheck(spec.dtype, f"(b={b}, h={h}) ")
        for i in blocks:
            rows = slice(i * 128, min(i * 128 + 128, spec.N))
            chk.add(wl.from_torch(out[b, h, rows]), pro, rows, spec.causal)
        chk.finish()


def test_full_size_smooth_v_sampled_parity():
    """The optional smooth-V technique at the full size of the video-like workload with a channel
    bias in V: preprocessing of V bit-exact on a whole head, outputs of sampled query blocks."""
    pa = _pa()
    spec = wl.CONFIGS["video17k_vbias"]
    rng = np.random.default_rng(4321)
    print("workload video17k_vbias, smooth V: generating inputs", flush=True)
    data = wl.make_inputs(spec, seed=0)
    dev = torch.device("cuda:0")
    q, k, v = (wl.to_torch(data[n], spec.dtype, dev) for n in "qkv")
    print("  running the HIP path", flush=True)
    out = pa.sage_attn_fwd_ex(q, k, v, causal=spec.causal, mode="int4_fp8", smooth_v=True)
    quant, args, ws = pa.sage_attn_quant(q, k, v, causal=spec.causal, mode="int4_fp8", smooth_v=True,
                                         want=["v_codes", "v_scale", "v_mean"])
    torch.cuda.synchronize()
    b, h = 1, 20
    blocks = _blocks(spec, 3, rng)
    print(f"  oracle on (b={b}, h={h}), query blocks {blocks}", flush=True)
    pro = so.quantize_head(data["q"][b, h], data["k"][b, h], data["v"][b, h], ds_blocks=blocks, smooth_v_on=True)
    assert np.array_equal(quant["v_mean"][b, h].cpu().numpy(), pro["vbar"])
    assert np.array_equal(quant["v_scale"][b, h].cpu().numpy(), pro["v_scale"])
    assert np.array_equal(quant["v_codes"][b, h].cpu().numpy(), pro["v_codes"])
    chk = parity.OutputCheck(spec.dtype)
    for i in blocks:
        rows = slice(i * 128, min(i * 128 + 128, spec.N))
        chk.add(wl.from_torch(out[b, h, rows]), pro, rows, spec.causal)
    chk.finish()


@pytest.mark.parametrize("group_map,gmap", [("fine", "fine"), ("token", "per_token")])
def test_full_size_finer_groups_sampled_parity(group_map, gmap):
    """The finer quantization granularities at the full size of the benchmark workload: codes and scales of a
    whole head bit-exact, outputs of sampled query blocks."""
    pa = _pa()
    spec = wl.CONFIGS["prefill4k"]
    rng = np.random.default_rng(99)
    print(f"workload prefill4k, group map {group_map}: generating inputs", flush=True)
    data = wl.make_inputs(spec, seed=0)
    dev = torch.device("cuda:0")
    q, k, v = (wl.to_torch(data[n], spec.dtype, dev) for n in "qkv")
    print("  running the HIP path", flush=True)
    out = pa.sage_attn_fwd_ex(q, k, v, causal=spec.causal, mode="int4_fp8", group_map=group_map)
    quant, args, ws = pa.sage_attn_quant(q, k, v, causal=spec.causal, mode="int4_fp8", group_map=group_map,
                                         want=["q_codes", "k_codes", "q_scale", "k_scale"])
    torch.cuda.synchronize()
    b, h = 2, 9
    blocks = _blocks(spec, 3, rng)
    print(f"  oracle on (b={b}, h={h}), query blocks {blocks}", flush=True)
    pro = so.quantize_head(data["q"][b, h], data["k"][b, h], data["v"][b, h], ds_blocks=blocks, gmap=gmap)
    for name in ("q_codes", "k_codes", "q_scale", "k_scale"):
        assert np.array_equal(quant[name][b, h].cpu().numpy(), pro[name]), name
    chk = parity.OutputCheck(spec.dtype)
    for i in blocks:
        rows = slice(i * 128, min(i * 128 + 128, spec.N))
        chk.add(wl.from_torch(out[b, h, rows]), pro, rows, spec.causal)
    chk.finish()


def test_full_size_varlen_sampled_parity():
    """A packed causal batch of five sequences of very different lengths (18 k tokens, 32 query heads on 8 KV
    heads): every sequence bit-identical to a call on it alone, sampled query blocks of the longest one
    against the oracle."""
    pa = _pa()
    lens = [4096, 1500, 8192, 333, 4200]
    H, Hkv, d, dtype = 32, 8, 128, "bf16"
    dev = torch.device("cuda:0")
    print(f"packed batch {lens}: generating inputs", flush=True)
    seqs = []
    for i, n in enumerate(lens):
        spec = wl.WorkloadSpec(f"seq{i}", 1, H, Hkv, n, d, dtype, True, 3.0, 3.0, 4, 10.0, 1.0, 200 + i)
        seqs.append(wl.make_inputs(spec, seed=0))
    pack = lambda name: wl.to_torch(np.ascontiguousarray(np.concatenate([s[name][0].transpose(1, 0, 2) for s in seqs])),
                                    dtype, dev)
    q, k, v = pack("q"), pack("k"), pack("v")
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=dev)
    print("  running the HIP path", flush=True)
    out = pa.sage_attn_fwd_ex(q, k, v, causal=True, mode="int4_fp8", cu_seqlens_q=cu, max_seqlen_q=max(lens),
                              max_seqlen_k=max(lens))
    torch.cuda.synchronize()
    off = np.concatenate([[0], np.cumsum(lens)])
    for i, n in enumerate(lens):
        sl = slice(off[i], off[i + 1])
        alone = pa.sage_attn_fwd_ex(q[sl].unsqueeze(0).contiguous(), k[sl].unsqueeze(0).contiguous(),
                                    v[sl].unsqueeze(0).contiguous(), causal=True, mode="int4_fp8", layout="NHD")
        torch.cuda.synchronize()
        assert torch.equal(alone[0], out[sl]), f"sequence {i}"
    i, h = 2, 13
    rng = np.random.default_rng(7)
    nqb = (lens[i] + 127) // 128
    blocks = sorted({0, nqb // 2, nqb - 1} | set(int(x) for x in rng.choice(nqb, size=2, replace=False)))
    print(f"  oracle on sequence {i}, head {h}, query blocks {blocks}", flush=True)
    pro = so.quantize_head(seqs[i]["q"][0, h], seqs[i]["k"][0, h // (H // Hkv)], seqs[i]["v"][0, h // (H // Hkv)],
                           ds_blocks=blocks)
    chk = parity.OutputCheck(dtype)
    for bq in blocks:
        rows = slice(bq * 128, min(bq * 128 + 128, lens[i]))
        chk.add(wl.from_torch(out[off[i] + rows.start:off[i] + rows.stop, h]), pro, rows, True)
    chk.finish()
