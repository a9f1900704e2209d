"""Throughput of the quantized attention forward pass on one MI355X.

A step is one pass of the whole hot path - smoothing / Delta-S / quantization prologue plus the
fused attention kernel - over one batch of synthetic, outlier-bearing inputs already resident in
HBM.  Prints ONE JSON line: whole-path TOPS as `value` (operations = 4*B*H*N*N_kv*d, halved under a
causal mask), the attention kernel's own roofline figure, and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TOPS = 5000.0   # MI355X dense int8 / fp8 MFMA peak (both 5.0 POP/s)


def cpu_baseline(spec, mode, budget_s=12.0, max_heads=32, smooth_v=False, gmap="g950", pv_fmt="e4m3",
                 smooth_k=True, smooth_q=True):
    """The CPU oracle as it stands, timed on a bounded sample of the same workload: whole (batch, head) slices,
    as many as fit in about budget_s seconds; for sequences beyond 8192 tokens only an evenly spaced subset of
    the 128-query blocks of each slice (the cost of a slice grows with N^2; the sample keeps it near that of
    an 8192-token slice), with the operation count of the sample scaled accordingly.  Returns the baseline
    record, the sampled heads, their inputs, the oracle's outputs and the sampled rows (None = all)."""
    import numpy as np
    import workloads as wl
    from oracle import sage_oracle as so
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    nqb = (spec.N + 127) // 128
    blocks, rows = None, None
    if spec.N > 8192:
        nsample = max(2, int(round(nqb * (8192.0 / spec.N) ** 2)))
        blocks = sorted(set(int(x) for x in np.linspace(0, nqb - 1, nsample)))
        rows = np.concatenate([np.arange(i * 128, min((i + 1) * 128, spec.N)) for i in blocks])
    heads, ins, outs, dt, ops = [], [], [], 0.0, 0.0
    for h in range(min(max_heads, spec.H)):
        qkv = (wl.make_head(spec, "q", 0, h), wl.make_head(spec, "k", 0, h * spec.H_kv // spec.H),
               wl.make_head(spec, "v", 0, h * spec.H_kv // spec.H))
        t0 = time.perf_counter()
        o = so.sage_attention_head(*qkv, causal=spec.causal, mode=mode, out_dtype="fp32", smooth_v_on=smooth_v, gmap=gmap,
                                   pv_fmt=pv_fmt, smooth_k_on=smooth_k,
                                   smooth_q_on=smooth_q and mode == "int4_fp8", q_blocks=blocks)[0]
        dt += time.perf_counter() - t0
        heads.append((0, h)); ins.append(qkv); outs.append(o if rows is None else o[rows])
        if rows is None:
            ops += 4.0 * float(spec.N) ** 2 * spec.d / (2 if spec.causal else 1)
        else:       # keys a sampled row sees: all of them, or (causal) those up to itself
            seen = (rows + 1 + (spec.kv_len - spec.N)).astype(np.float64) if spec.causal else np.full(len(rows), float(spec.kv_len))
            ops += 4.0 * float(seen.sum()) * spec.d
        if dt > budget_s:
            break
    what = "all query blocks" if blocks is None else f"{len(blocks)} of {nqb} query blocks each"
    return dict(value=ops / dt / 1e12, unit="TOPS", cores=threads, kind="oracle",
                sample=f"{len(heads)} of {spec.B * spec.H} (batch, head) slices of {spec.name}, {what}, "
                       f"{dt:.1f} s"), heads, ins, outs, rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # defaults: the chip needs some tens of milliseconds of back-to-back work before its clocks settle
    # (5 warm-up steps of the 1 ms default workload measure 8 % low); 50 + 100 steps are 0.15 s of GPU time
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="prefill4k")
    ap.add_argument("--mode", default="int4_fp8", choices=["int4_fp8", "int8_fp8"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--group-map", default="lane", choices=["lane", "block", "fine", "token", "tensor"],
                    help="quantization granularity of Q and K: the default lane groups, one scale per block, "
                         "per query and 4 keys, or per token")
    ap.add_argument("--pv-format", default="e4m3", choices=["e4m3", "e5m2", "int8"],
                    help="8-bit data type of P~ and V: the paper's E4M3, or E5M2 / INT8 for the comparison")
    ap.add_argument("--smooth-v", action="store_true",
                    help="the optional smooth-V technique (one more pass over V in the prologue)")
    ap.add_argument("--no-smooth-k", action="store_true", help="smoothing ablation: K is quantized as it is")
    ap.add_argument("--no-smooth-q", action="store_true",
                    help="smoothing ablation: Q is quantized as it is (4-bit mode; the 8-bit mode never smooths Q)")
    ap.add_argument("--fp32-delta-s", action="store_true",
                    help="Delta-S accumulated in FP32 instead of FP64 (SAGE_FLAG_FP32_DELTA_S): faster preprocessing, "
                         "Delta-S approximate instead of correctly rounded")
    ap.add_argument("--given-kv-stats", action="store_true",
                    help="mean(K) and delta_V are computed once, outside the timed region, and supplied to every step "
                         "(k_mean_in / v_scale_in: what a producer of K and V would hand over); the statistics pass is "
                         "then not part of the step")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a kernel of known traffic, for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2411_10958_amd as pa
    import workloads as wl

    pa.load_library()            # fails loudly when the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    spec = wl.CONFIGS[args.workload]
    data = wl.make_inputs(spec, seed=0)
    q, k, v = (wl.to_torch(data[n], spec.dtype, dev) for n in "qkv")
    out = torch.empty_like(q)
    kv_stats = pa.sage_attn_kv_stats(k, v, pv_format=args.pv_format) if args.given_kv_stats else None
    a = pa.make_args(q, k, v, out, causal=spec.causal, mode=args.mode, smooth_v=args.smooth_v, kv_stats=kv_stats,
                     group_map=args.group_map, pv_format=args.pv_format, smooth_k=not args.no_smooth_k,
                     smooth_q=not args.no_smooth_q, fp32_delta_s=args.fp32_delta_s)
    ws = torch.empty(pa.sage_attn_workspace_bytes(a), dtype=torch.uint8, device=dev)
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()

    def step(events=None):
        if events is not None:
            events[0].record()
        pa.sage_attn_prologue(a)
        if events is not None:
            events[1].record()
        pa.sage_attn_core(a)
        if events is not None:
            events[2].record()

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # the per-kernel durations come from HIP events around every EVERY-th step of the timed region (three
    # event records in every step cost about 1 % of the step)
    EVERY = 1 if args.steps < 20 else 5
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range((args.steps + EVERY - 1) // EVERY)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i // EVERY] if i % EVERY == 0 else None)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step = wall * 1e3 / args.steps
    ms_pro = sum(e[0].elapsed_time(e[1]) for e in evs) / len(evs)
    ms_core = sum(e[1].elapsed_time(e[2]) for e in evs) / len(evs)
    ops = wl.flops(spec)
    tops = ops / (ms_step * 1e-3) / 1e12
    core_tops = ops / (ms_core * 1e-3) / 1e12

    # HBM bytes per launch of the attention kernel, from the committed rocprofv3 counter summary
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "attn_kernel_traffic.txt")      # JSON text, one record per workload / mode
    default_options = (args.group_map == "lane" and args.pv_format == "e4m3" and not args.smooth_v and not args.no_smooth_k
                       and not args.no_smooth_q and not args.fp32_delta_s)
    if os.path.exists(tfile) and default_options:         # the counters were collected with the default options
        with open(tfile) as f:
            t = json.load(f).get(f"{args.workload}/{args.mode}")
        if t:
            traffic = t["hbm_read_bytes"] + t["hbm_write_bytes"]
    # algorithmic bytes of the same launch: codes of Q, K (1 B, or 6 bits in the INT4 mode) and V (1 B),
    # Delta-S rows the tiles read,
    # scales, and the 16-bit output
    BH, BHkv = spec.B * spec.H, spec.B * spec.H_kv
    nqb = (spec.N + 127) // 128
    ds_bytes = 0
    if args.mode == "int4_fp8":
        per_row = [min(spec.N, (i * 128 + 128 + 63) // 64 * 64) if spec.causal else spec.N for i in range(nqb)]
        ds_bytes = 4 * BH * sum(per_row)
    qk_code_bytes = 0.75 if args.mode == "int4_fp8" else 1.0      # 6-bit codes in the INT4 mode
    qg, kg = {"lane": (2, 16), "block": (2, 16), "fine": (1, 4), "token": (1, 1), "tensor": (2, 16)}[args.group_map]
    alg_bytes = int((BH + BHkv) * spec.N * spec.d * qk_code_bytes) + BHkv * spec.N * spec.d + ds_bytes \
        + 4 * (BH * spec.N // qg + BHkv * spec.N // kg) + 2 * BH * spec.N * spec.d

    res = {
        "metric": "quantized attention TOPS at d=128 (causal + non-causal), cos-sim vs FP32",
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("int8" if args.mode == "int8_fp8" else "int4") + ("+int8" if args.pv_format == "int8" else "+fp8"),
        "data": "synthetic",
        "config": {"workload": f"{spec.name}: B={spec.B} H={spec.H} H_kv={spec.H_kv} N={spec.N} d={spec.d} "
                               f"{spec.dtype} causal={spec.causal}", "mode": args.mode, "smooth_v": bool(args.smooth_v),
                   "smooth_k": not args.no_smooth_k, "smooth_q": not args.no_smooth_q and args.mode == "int4_fp8",
                   "fp32_delta_s": bool(args.fp32_delta_s), "given_kv_stats": bool(args.given_kv_stats),
                   "group_map": args.group_map, "pv_format": args.pv_format,
                   "ops_formula": "4*B*H*N^2*d" + ("/2" if spec.causal else "")},
        "breakdown_ms": {"prologue": round(ms_pro, 4), "attention_kernel": round(ms_core, 4)},
        "roofline": {"bound": "mfma", "kernel": "k_attn_fwd", "achieved": round(core_tops, 2), "peak": PEAK_TOPS,
                     "unit": "TFLOP/s", "frac": round(core_tops / PEAK_TOPS, 4), "traffic": traffic,
                     "algorithmic_bytes": alg_bytes, "ops_per_launch": ops},
    }

    # accuracy of what was just computed, on sampled heads (outside the timed region)
    torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        from oracle import sage_oracle as so
        base, heads, ins, outs, srows = cpu_baseline(spec, args.mode, smooth_v=args.smooth_v,
                                                       gmap={"lane": "g950", "block": "per_block", "fine": "fine",
                                                             "token": "per_token", "tensor": "per_tensor"}[args.group_map],
                                                       pv_fmt=args.pv_format, smooth_k=not args.no_smooth_k,
                                                       smooth_q=not args.no_smooth_q)
        res["cpu_baseline"] = base
        got = np.stack([wl.from_torch(out[b, h]) for b, h in heads])
        if srows is not None:
            got = got[:, srows]
        ref = np.stack(outs)
        # rows for the comparison with FP64 attention: every (N / 512)-th row, or 512 of the sampled rows
        if srows is None:
            sub = np.arange(0, spec.N, max(1, spec.N // 512))
            frows = sub
        else:
            sub = np.arange(0, len(srows), max(1, len(srows) // 512))
            frows = srows[sub]
        full = np.stack([so.ref_attn_fp64(qh, kh, vh, spec.causal, rows=frows) for qh, kh, vh in ins])
        # the oracle's FP32 output; the kernel rounds once more to the 16-bit output type
        mant = 10 if spec.dtype == "fp16" else 7
        half_ulp = 0.5 * np.exp2(np.floor(np.log2(np.maximum(np.abs(ref), 1e-30))) - mant)
        linf = np.abs(ref).max(axis=-1, keepdims=True)
        excess = (np.abs(got - ref) - half_ulp) / linf
        res["accuracy"] = {"sample": f"{len(heads)} heads" + ("" if srows is None else f", {len(srows)} rows each"),
                           "vs_oracle_max_abs_over_row_linf_beyond_output_rounding": float(max(excess.max(), 0.0)),
                           "vs_oracle_cos": wl.cos_sim(got, ref),
                           "vs_fp64_attention_cos": wl.cos_sim(got[:, sub], full),
                           "vs_fp64_attention_rel_l1": wl.rel_l1(got[:, sub], full)}
    else:
        res["cpu_baseline"] = None
    print(json.dumps(res))


if __name__ == "__main__":
    main()
