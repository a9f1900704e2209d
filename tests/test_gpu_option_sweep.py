"""Seeded sweep over combinations of the options of sage_attn_args on small shapes: every combination goes
through the HIP path and is compared with the CPU oracle (same bars as tests/test_gpu_parity.py), so that
interactions - a layout with a group map, smooth V with another key length, the log-sum-exp with a packed
batch - are exercised and not only each option alone."""
import os

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import sage_oracle as so
from oracle import parity
from test_gpu_parity import _pa, _lse_close
from test_gpu_prologue_fuzz import _awkward

pytestmark = pytest.mark.gpu

GMAPS = {"lane": "g950", "block": "per_block", "fine": "fine", "token": "per_token", "tensor": "per_tensor"}


def _draw(rng):
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2]))
    H = Hkv * int(rng.choice([1, 2, 4]))
    causal = bool(rng.integers(2))
    long_run = bool(os.environ.get("SAGE_SWEEP_LONG"))       # one-off runs on longer sequences (slower oracle)
    n = int(rng.choice([513, 700, 1111, 2048] if long_run else [1, 17, 64, 100, 128, 129, 200, 257, 333, 450]))
    nk = n if rng.random() < 0.5 else int(rng.choice([640, 1500, 2500, 3100] if long_run else [1, 63, 64, 65, 190, 300, 520]))
    if causal and nk < n:
        nk = n
    group_map = str(rng.choice(list(GMAPS)))
    pv = str(rng.choice(["e5m2", "int8"])) if (group_map in ("lane", "block", "tensor") and rng.random() < 0.4) else "e4m3"
    c = dict(d=d, H=H, Hkv=Hkv, causal=causal, n=n, nk=nk, group_map=group_map, pv=pv,
             mode=str(rng.choice(["int4_fp8", "int8_fp8"])), dtype=str(rng.choice(["bf16", "fp16"])),
             layout=str(rng.choice(["HND", "NHD"])), smooth_v=bool(rng.random() < 0.3), lse=bool(rng.random() < 0.5),
             vbias=float(rng.choice([0.0, 4.0])))
    # the smoothing switches are drawn last so that the earlier draws of a seed stay what they were
    c["smooth_k"] = bool(rng.random() >= 0.25)
    c["smooth_q"] = bool(rng.random() >= 0.25)
    # statistics of K and V handed over by the caller (only where mean(K) and delta_V are all that pass produces)
    c["kv_stats"] = bool(rng.random() < 0.4) and c["smooth_k"] and not c["smooth_v"]
    # inputs with awkward values (heads scaled by powers of two, all-zero tokens, channels and heads, ties, heavy
    # tails) instead of the workload generator's
    c["awkward"] = bool(rng.random() < 0.3)
    # which exact form of the Delta-S product (None: the library's choice - the FP64 form at these sizes)
    c["delta_s"] = [None, "digits", "fp64"][int(rng.integers(3))]
    return c


def _inputs(c, seed, cfg, n=None, nk=None, B=2):
    n, nk = (c["n"] if n is None else n), (c["nk"] if nk is None else nk)
    if c["awkward"]:
        r = np.random.default_rng(9000 + 17 * seed + cfg)
        mk = lambda heads, tokens, lim: np.stack([_awkward(r, (heads, tokens, c["d"]), c["dtype"], lim) for _ in range(B)])
        lim = int(os.environ.get("SAGE_SWEEP_LIM", "8"))     # heads of Q and K scaled by up to 2^lim either way
        return dict(q=mk(c["H"], n, lim), k=mk(c["Hkv"], nk, lim), v=mk(c["Hkv"], nk, 4))
    spec = wl.WorkloadSpec("sweep", B, c["H"], c["Hkv"], n, c["d"], c["dtype"], c["causal"], 3.0, 1.5, 2, 10.0, 1.0,
                           cfg, c["vbias"], nk)
    return wl.make_inputs(spec, seed=seed)


def _oracle_smoothing(c):
    return dict(smooth_k_on=c["smooth_k"], smooth_q_on=c["smooth_q"] and c["mode"] == "int4_fp8")


# SAGE_SWEEP_SEEDS widens the sweep for a one-off longer run (the default keeps the suite short)
N_SEEDS = int(os.environ.get("SAGE_SWEEP_SEEDS", "48"))


# Seeds kept as fixed regression cases whatever SAGE_SWEEP_SEEDS says.  7631: the dominant key of some rows has
# an all-zero V row, so the whole output row lies below the smallest normal FP32 number, where the hardware
# exponential's flush of subnormal results shows (the absolute floor of oracle/parity.py).  1124: smooth V on
# heavy-tailed values - the products of a channel cancel to a quarter of their magnitude, so the matrix
# instruction's rounding, which is relative to that magnitude, is 5.1e-4 of the row norm (bar B's row scale).
REGRESSION_SEEDS = [7631, 1124]


@pytest.mark.parametrize("seed", list(range(N_SEEDS)) + [s for s in REGRESSION_SEEDS if s >= N_SEEDS])
def test_option_combination_matches_oracle(seed):
    pa = _pa()
    rng = np.random.default_rng(1000 + seed)
    c = _draw(rng)
    print(f"combination {seed}: {c}", flush=True)
    data = _inputs(c, seed, 300 + seed)
    dev = torch.device("cuda:0")
    q, k, v = (wl.to_torch(data[x], c["dtype"], dev) for x in "qkv")
    if c["layout"] == "NHD":
        q, k, v = (t.permute(0, 2, 1, 3).contiguous() for t in (q, k, v))
    stats = pa.sage_attn_kv_stats(k, v, layout=c["layout"], pv_format=c["pv"]) if c["kv_stats"] else None
    res = pa.sage_attn_fwd_ex(q, k, v, causal=c["causal"], mode=c["mode"], smooth_v=c["smooth_v"], group_map=c["group_map"],
                              layout=c["layout"], pv_format=c["pv"], return_lse=c["lse"], smooth_k=c["smooth_k"],
                              smooth_q=c["smooth_q"], kv_stats=stats, delta_s=c["delta_s"])
    torch.cuda.synchronize()
    out, lse = res if c["lse"] else (res, None)
    if c["layout"] == "NHD":
        out = out.permute(0, 2, 1, 3)
    # (few tiles and many keys: the library splits the key range by itself, and says so)
    splits = pa.sage_attn_kv_splits(pa.make_args(q, k, v, causal=c["causal"], mode=c["mode"], smooth_v=c["smooth_v"],
                                                 group_map=c["group_map"], layout=c["layout"], pv_format=c["pv"]))
    pros = parity.check_heads(wl.from_torch(out), data, c["causal"], c["mode"], c["dtype"], want_lse=c["lse"], splits=splits,
                              gmap=GMAPS[c["group_map"]], smooth_v_on=c["smooth_v"], pv_fmt=c["pv"], **_oracle_smoothing(c))
    if c["lse"]:
        for b in range(2):
            for h in range(c["H"]):
                _lse_close(lse[b, h].cpu().numpy(), pros[b][h]["lse"], pros[b][h])


@pytest.mark.parametrize("seed", range(max(6, N_SEEDS // 4)))
def test_packed_batch_combination_matches_oracle(seed):
    pa = _pa()
    rng = np.random.default_rng(2000 + seed)
    c = _draw(rng)
    B = int(rng.integers(2, 5))
    lens_q = [int(rng.choice([0, 1, 40, 128, 150, 300])) for _ in range(B)]
    lens_q[int(rng.integers(B))] = 200                    # at least one sequence worth checking
    lens_k = [n if (c["causal"] or rng.random() < 0.5) else int(rng.choice([1, 64, 90, 260])) for n in lens_q]
    print(f"packed combination {seed}: {c} q={lens_q} k={lens_k}", flush=True)
    dev = torch.device("cuda:0")
    seqs, qs, ks, vs = [], [], [], []
    for i, (n, nk) in enumerate(zip(lens_q, lens_k)):
        dd = _inputs(c, seed, 400 + 10 * seed + i, max(n, 1), max(nk, 1), B=1)
        qn, kn, vn = dd["q"][0][:, :n], dd["k"][0][:, :nk], dd["v"][0][:, :nk]
        seqs.append((qn, kn, vn))
        qs.append(qn.transpose(1, 0, 2)); ks.append(kn.transpose(1, 0, 2)); vs.append(vn.transpose(1, 0, 2))
    pack = lambda parts: wl.to_torch(np.ascontiguousarray(np.concatenate(parts, axis=0)), c["dtype"], dev)
    cu = lambda lens: torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=dev)
    q, k, v = pack(qs), pack(ks), pack(vs)
    stats = pa.sage_attn_kv_stats(k, v, pv_format=c["pv"], cu_seqlens_k=cu(lens_k), max_seqlen_k=max(max(lens_k), 1)) \
        if c["kv_stats"] else None
    res = pa.sage_attn_fwd_ex(q, k, v, causal=c["causal"], mode=c["mode"], smooth_v=c["smooth_v"], group_map=c["group_map"],
                              pv_format=c["pv"], return_lse=c["lse"], cu_seqlens_q=cu(lens_q), cu_seqlens_k=cu(lens_k),
                              smooth_k=c["smooth_k"], smooth_q=c["smooth_q"], kv_stats=stats, delta_s=c["delta_s"])
    torch.cuda.synchronize()
    out, lse = res if c["lse"] else (res, None)
    off = np.concatenate([[0], np.cumsum(lens_q)])
    g = c["H"] // c["Hkv"]
    for i, (n, nk) in enumerate(zip(lens_q, lens_k)):
        if n == 0 or nk == 0:
            continue
        qn, kn, vn = seqs[i]
        pros = parity.check_heads(wl.from_torch(out[off[i]:off[i + 1]]).transpose(1, 0, 2)[None],
                                  dict(q=qn[None], k=kn[None], v=vn[None]), c["causal"], c["mode"], c["dtype"],
                                  want_lse=c["lse"], gmap=GMAPS[c["group_map"]], smooth_v_on=c["smooth_v"], pv_fmt=c["pv"],
                                  **_oracle_smoothing(c))
        if c["lse"]:
            for h in range(c["H"]):
                _lse_close(lse[h, off[i]:off[i + 1]].cpu().numpy(), pros[0][h]["lse"], pros[0][h])
