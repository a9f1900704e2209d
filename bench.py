"""Throughput of the quantized attention forward pass on one MI355X.

A step is one pass of the whole hot path - smoothing / Delta-S / quantization prologue plus the
fused attention kernel - over one batch of synthetic, outlier-bearing inputs already resident in
HBM.  Prints ONE JSON line: whole-path TOPS as `value` (operations = 4*B*H*N*N_kv*d, halved under a
causal mask) on the headline workload, the attention kernel's own roofline figures, a sweep over the causal
workloads at N >= 8192 in both modes (kernel alone and whole path), and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X dense matrix peaks (TOP/s): the 8-bit formats (INT8, FP8), and the 6- / 4-bit formats of the same instruction
PEAK_8BIT = 5000.0
PEAK_FP6 = 10100.0
GMAPS = {"lane": "g950", "block": "per_block", "fine": "fine", "token": "per_token", "tensor": "per_tensor"}


def mix_peak(mode, pv_format="e4m3"):
    """Matrix peak of the instructions the attention kernel actually issues: half of the operations are the score
    product (FP6 operand format in the INT4 mode, 8-bit otherwise), half the P~V product (8-bit): the harmonic
    mean of the two rates."""
    qk = PEAK_FP6 if mode == "int4_fp8" else PEAK_8BIT
    return 2.0 / (1.0 / qk + 1.0 / PEAK_8BIT)


# Vector-ALU ceiling of Algorithm 1's inner loop on this chip: per score the loop needs, per lane, one multiply-add
# (dequantization + Delta-S), half a three-input maximum, one subtraction, one exponential, one addition (row sum)
# and half a packed FP8 conversion.  Issued back to back in that mix, nothing else running, these ten instructions
# per two scores take 69.3 / 52.5 / 48.7 cycles of a SIMD with 2 / 3 / 4 wavefronts resident (measured by
# paper_2411_10958_amd/csrc/probe_valu_issue.hip, summary under profiles/; the classes alone at 4 wavefronts: add /
# sub / mul / fma 2.6 to 2.9, max3 4.5, exp 8.4, packed FP8 conversion 8.4 cycles per wavefront instruction).  The
# ceiling takes the best of them.  A wavefront instruction covers 64 lanes, so one SIMD finishes 128 scores per that
# many cycles; a score is 4 d operations.
VALU_CYCLES_PER_2_SCORES = 48.7
N_SIMD = 1024
CLOCK_GHZ = 2.4


def alu_ceiling_tops(d):
    scores_per_s = N_SIMD * CLOCK_GHZ * 1e9 * 128.0 / VALU_CYCLES_PER_2_SCORES
    return scores_per_s * 4.0 * d / 1e12


def _oracle_job(job):
    """One (batch, head) slice through the CPU oracle (run in a worker process, one BLAS thread each)."""
    name, h, mode, blocks, kw = job
    import workloads as wl
    from oracle import sage_oracle as so
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(1)
    except Exception:
        pass
    spec = wl.CONFIGS[name]
    qkv = (wl.make_head(spec, "q", 0, h), wl.make_head(spec, "k", 0, h * spec.H_kv // spec.H),
           wl.make_head(spec, "v", 0, h * spec.H_kv // spec.H))
    t0 = time.perf_counter()
    so.sage_attention_head(*qkv, causal=spec.causal, mode=mode, out_dtype="fp32", q_blocks=blocks, **kw)
    return time.perf_counter() - t0


def cpu_baseline(spec, mode, n_heads, oracle_kw):
    """The CPU oracle as it stands (Algorithm 1 as printed, numpy), timed on a bounded sample of the same workload:
    n_heads whole (batch, head) slices, one per worker process over all host cores the box gives this job; for
    sequences beyond 8192 tokens only an evenly spaced subset of the 128-query blocks of each slice (the cost of a
    slice grows with N^2; the sample keeps it near that of an 8192-token slice), with the operation count of
    the sample scaled accordingly.  Must run before this process touches the GPU (it forks)."""
    import multiprocessing as mp
    import numpy as np
    import workloads as wl
    cores = max(1, min(int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1), os.cpu_count() or 1, 16))
    nqb = (spec.N + 127) // 128
    blocks, rows = None, None
    if spec.N > 8192:
        nsample = max(2, int(round(nqb * (8192.0 / spec.N) ** 2)))
        blocks = sorted(set(int(x) for x in np.linspace(0, nqb - 1, nsample)))
        rows = np.concatenate([np.arange(i * 128, min((i + 1) * 128, spec.N)) for i in blocks])
    n_heads = min(n_heads, spec.H)
    jobs = [(spec.name, h, mode, blocks, oracle_kw) for h in range(n_heads)]
    from oracle import sage_oracle  # noqa: F401  (imported before the fork so that the workers start with it)
    with mp.get_context("fork").Pool(min(cores, n_heads)) as pool:
        t0 = time.perf_counter()
        each = pool.map(_oracle_job, jobs, chunksize=1)
        wall = time.perf_counter() - t0
    if rows is None:
        ops_head = wl.flops(spec) / (spec.B * spec.H)
    else:       # keys a sampled row sees: all of them, or (causal) those up to itself
        seen = (rows + 1 + (spec.kv_len - spec.N)).astype(np.float64) if spec.causal else np.full(len(rows), float(spec.kv_len))
        ops_head = 4.0 * float(seen.sum()) * spec.d
    what = "all query blocks" if blocks is None else f"{len(blocks)} of {nqb} query blocks each"
    return dict(value=ops_head * n_heads / wall / 1e12, unit="TOPS", cores=min(cores, n_heads), kind="oracle",
                sample=f"{n_heads} of {spec.B * spec.H} (batch, head) slices of {spec.name}, {what}: {sum(each):.1f} s of "
                       f"CPU work in {wall:.1f} s on {min(cores, n_heads)} worker processes (one thread each)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--preroll-ms", type=float, default=60.0,
                    help="untimed back-to-back steps for at least this long before the warm-up steps: the chip needs some "
                         "tens of milliseconds of work before its clocks settle (5 steps of 1 ms measure 8 %% low)")
    ap.add_argument("--workload", default="prefill4k",
                    help="a configuration of workloads/inputs.py, or an ad-hoc shape such as b4h32n8192d128c "
                         "(batch, heads, tokens, head dimension, c = causal / f = full)")
    ap.add_argument("--mode", default="int4_fp8", choices=["int4_fp8", "int8_fp8"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", action="store_true", help="skip the causal N >= 8192 sweep")
    ap.add_argument("--sweep", default="causal8k,causal16k,causal32k", help="workloads of the sweep (both modes each; names as for --workload)")
    ap.add_argument("--cpu-heads", type=int, default=32, help="(batch, head) slices of the CPU-baseline sample")
    ap.add_argument("--group-map", default="lane", choices=list(GMAPS),
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
    import workloads as wl
    spec = wl.spec_of(args.workload)
    oracle_kw = dict(smooth_v_on=args.smooth_v, gmap=GMAPS[args.group_map], pv_fmt=args.pv_format,
                     smooth_k_on=not args.no_smooth_k, smooth_q_on=not args.no_smooth_q and args.mode == "int4_fp8")
    # The CPU leg runs first: its worker processes are forked, which must not happen once this process holds a GPU.
    base = None if args.no_cpu_baseline else cpu_baseline(spec, args.mode, args.cpu_heads, oracle_kw)

    import torch
    import paper_2411_10958_amd as pa

    pa.load_library()            # fails loudly when the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")

    def prepare(spec, mode, headline):
        data = wl.make_inputs(spec, seed=0)
        q, k, v = (wl.to_torch(data[n], spec.dtype, dev) for n in "qkv")
        out = torch.empty_like(q)
        opts = dict(smooth_v=args.smooth_v, group_map=args.group_map, pv_format=args.pv_format, smooth_k=not args.no_smooth_k,
                    smooth_q=not args.no_smooth_q, fp32_delta_s=args.fp32_delta_s) if headline else {}
        kv_stats = pa.sage_attn_kv_stats(k, v, pv_format=args.pv_format) if (headline and args.given_kv_stats) else None
        a = pa.make_args(q, k, v, out, causal=spec.causal, mode=mode, kv_stats=kv_stats, **opts)
        ws = torch.empty(pa.sage_attn_workspace_bytes(a), dtype=torch.uint8, device=dev)
        a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
        return data, a, (q, k, v, out, ws, kv_stats)

    def step(a, events=None):
        if events is not None:
            events[0].record()
        pa.sage_attn_prologue(a)
        if events is not None:
            events[1].record()
        pa.sage_attn_core(a)
        if events is not None:
            events[2].record()

    def preroll(a, ms):
        """Untimed back-to-back steps for at least `ms` milliseconds of GPU time; returns how long it ran."""
        t0 = time.perf_counter()
        n = 0
        while True:
            for _ in range(4):
                step(a)
            n += 4
            torch.cuda.synchronize()
            if (time.perf_counter() - t0) * 1e3 >= ms:
                return (time.perf_counter() - t0) * 1e3

    def timed(a, steps, every):
        """`steps` steps between two synchronisations (wall clock), with HIP events on the launch stream around the
        prologue and the attention kernel of every `every`-th step (three event records cost about 1 % of a 1 ms
        step).  Returns ms per step, ms prologue, ms attention kernel."""
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range((steps + every - 1) // every)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            step(a, evs[i // every] if i % every == 0 else None)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        return (wall * 1e3 / steps, sum(e[0].elapsed_time(e[1]) for e in evs) / len(evs),
                sum(e[1].elapsed_time(e[2]) for e in evs) / len(evs))

    data, a, keep = prepare(spec, args.mode, True)
    out = keep[3]
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    preroll_ms = preroll(a, args.preroll_ms)
    for _ in range(args.warmup):
        step(a)
    ms_step, ms_pro, ms_core = timed(a, args.steps, 1 if args.steps < 20 else 5)
    ops = wl.flops(spec)
    tops = ops / (ms_step * 1e-3) / 1e12
    core_tops = ops / (ms_core * 1e-3) / 1e12

    # HBM bytes per launch of the attention kernel: quoted from the committed rocprofv3 counter summary (two --pmc runs
    # of this command, FETCH_SIZE then WRITE_SIZE), not measured in this run
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
    # Delta-S rows the tiles read, scales, and the 16-bit output
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

    peak_mix = mix_peak(args.mode, args.pv_format)
    alu = alu_ceiling_tops(spec.d)
    splits = pa.sage_attn_kv_splits(a)
    res = {
        "metric": "quantized attention TOPS at d=128 (causal + non-causal), cos-sim vs FP32",
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "preroll_ms": round(preroll_ms, 1),
        "ms_per_step": round(ms_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": ("int8" if args.mode == "int8_fp8" else "int4") + ("+int8" if args.pv_format == "int8" else "+fp8"),
        "data": "synthetic",
        "config": {"workload": f"{spec.name}: B={spec.B} H={spec.H} H_kv={spec.H_kv} N={spec.N} d={spec.d} "
                               f"{spec.dtype} causal={spec.causal}", "mode": args.mode, "smooth_v": bool(args.smooth_v),
                   "smooth_k": not args.no_smooth_k, "smooth_q": not args.no_smooth_q and args.mode == "int4_fp8",
                   "fp32_delta_s": bool(args.fp32_delta_s), "given_kv_stats": bool(args.given_kv_stats),
                   "group_map": args.group_map, "pv_format": args.pv_format, "kv_splits": splits,
                   "ops_formula": "4*B*H*N^2*d" + ("/2" if spec.causal else "")},
        "breakdown_ms": {"prologue": round(ms_pro, 4), "attention_kernel": round(ms_core, 4)},
        # The attention kernel is a dense contraction whose vector work (the softmax between its two products) takes
        # longer than its matrix work: the counters show the vector ALU as the busy unit, so that is the bound named.
        # `peak` is the matrix peak of the instructions the kernel issues (score product in the FP6 operand format at
        # 10.1 POP/s in the INT4 mode, P~V in FP8 at 5.0: 6.69 POP/s; 5.0 in the INT8 mode); `frac_of_8bit_peak` is the
        # same rate against the 5.0 POP/s the target is stated in; `alu_ceiling` is the rate at which the loop's vector
        # instructions alone could be issued (derivation at the top of this file and in the design doc).
        "roofline": {"bound": "alu", "kernel": "k_attn_fwd", "achieved": round(core_tops, 2), "peak": round(peak_mix, 1),
                     "unit": "TOP/s", "frac": round(core_tops / peak_mix, 4),
                     "peak_8bit": PEAK_8BIT, "frac_of_8bit_peak": round(core_tops / PEAK_8BIT, 4),
                     "alu_ceiling": round(alu, 1), "frac_of_alu_ceiling": round(core_tops / alu, 4),
                     "traffic": traffic, "traffic_source": "profiles/attn_kernel_traffic.txt (rocprofv3 --pmc runs of this "
                                                           "command; quoted, not measured in this run)" if traffic else None,
                     "algorithmic_bytes": alg_bytes, "ops_per_launch": ops},
    }

    if spec.N <= 128 and spec.kv_len >= 64 * spec.N:
        # decode-shaped: a few queries per sequence against a long cache.  The attention kernel then reads every code of
        # K and V once per KV head (query heads of a group find them in the caches) and does next to no arithmetic per
        # byte: its bound is HBM bandwidth, and its figure is bytes per second.
        kv_bytes = int(BHkv * spec.kv_len * spec.d * (qk_code_bytes + 1.0)) + ds_bytes + 4 * BHkv * spec.kv_len // kg
        res["roofline"] = {"bound": "hbm", "kernel": "k_attn_fwd (key range split) + k_merge_splits",
                           "achieved": round(kv_bytes / (ms_core * 1e-3) / 1e9, 1), "peak": 8000.0, "unit": "GB/s",
                           "frac": round(kv_bytes / (ms_core * 1e-3) / 1e9 / 8000.0, 4), "traffic": None,
                           "algorithmic_bytes": kv_bytes, "ops_per_launch": ops}

    # accuracy of what was just computed, on sampled heads (outside the timed region): the comparison the GPU tests make
    torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        from oracle import parity
        from oracle import sage_oracle as so
        res["cpu_baseline"] = base
        g = spec.H // spec.H_kv
        nsample = max(2, int(round(nqb * min(1.0, (4096.0 / spec.N) ** 2))))
        blocks = sorted(set(int(x) for x in np.linspace(0, nqb - 1, nsample)))
        rows = np.concatenate([np.arange(i * 128, min((i + 1) * 128, spec.N)) for i in blocks])
        heads = [(0, 0), (spec.B - 1, spec.H - 1), (spec.B // 2, spec.H // 3)]
        chk = parity.OutputCheck(spec.dtype, "accuracy sample: ")
        got_rows, full_rows = [], []
        sub = np.arange(0, len(rows), max(1, len(rows) // 512))
        for b, h in heads:
            qh, kh, vh = data["q"][b, h], data["k"][b, h // g], data["v"][b, h // g]
            pro = so.quantize_head(qh, kh, vh, mode=args.mode, ds_blocks=blocks, **oracle_kw)
            got = wl.from_torch(out[b, h])
            chk.add_head(got, pro, spec.causal, blocks=blocks, splits=splits)
            got_rows.append(got[rows[sub]])
            full_rows.append(so.ref_attn_fp64(qh, kh, vh, spec.causal, rows=rows[sub]))
        import contextlib
        import io
        verdict = "every row within the bars or explained by one-step codes of P~"
        with contextlib.redirect_stdout(io.StringIO()):       # (the check prints a line of its own; this program prints one)
            try:
                cos = chk.finish()                            # raises if a row beyond a bar is not explained
            except AssertionError as e:
                cos, verdict = float("nan"), "FAILED: " + str(e)[:300]
        res["accuracy"] = {"sample": f"{len(heads)} heads, {len(rows)} rows each", "check": verdict,
                           "vs_oracle_as_printed_max_abs_over_row_linf_beyond_output_rounding": chk.worst_a,
                           "vs_oracle_as_printed_cos": cos,
                           "vs_oracle_kernel_order_max_abs_over_row_linf_beyond_output_rounding": chk.worst_b,
                           "rows_beyond_the_bars_all_explained_by_one_step_codes": [chk.over_a, chk.over_b],
                           "vs_fp64_attention_cos": wl.cos_sim(np.stack(got_rows), np.stack(full_rows)),
                           "vs_fp64_attention_rel_l1": wl.rel_l1(np.stack(got_rows), np.stack(full_rows))}
    else:
        res["cpu_baseline"] = None

    # the regime the target is stated for: d = 128, causal, N >= 8192, both modes; kernel alone (the paper's protocol:
    # operands already quantized) and whole path, default options
    if not args.no_sweep:
        del data, a, keep, out
        torch.cuda.empty_cache()
        sweep = []
        for name in [s for s in args.sweep.split(",") if s]:
            sp = wl.spec_of(name)
            d_in = None
            for mode in ("int4_fp8", "int8_fp8"):
                d_in, a2, keep2 = prepare(sp, mode, False) if d_in is None else (d_in,) + _reuse(pa, torch, sp, mode, keep2)
                preroll(a2, max(20.0, args.preroll_ms / 2))
                ms_s, ms_p, ms_c = timed(a2, 10, 1)
                o = wl.flops(sp)
                kt, wt = o / (ms_c * 1e-3) / 1e12, o / (ms_s * 1e-3) / 1e12
                pm = mix_peak(mode)
                sweep.append({"workload": name, "mode": mode, "N": sp.N, "causal": sp.causal, "d": sp.d,
                              "ms_prologue": round(ms_p, 4), "ms_attention_kernel": round(ms_c, 4), "ms_per_step": round(ms_s, 4),
                              "kernel_tops": round(kt, 1), "kernel_frac": round(kt / pm, 4), "peak": round(pm, 1),
                              "kernel_frac_of_8bit_peak": round(kt / PEAK_8BIT, 4),
                              "whole_path_tops": round(wt, 1), "whole_path_frac_of_8bit_peak": round(wt / PEAK_8BIT, 4)})
            del d_in, a2, keep2
            torch.cuda.empty_cache()
        res["sweep"] = sweep
    print(json.dumps(res))


def _reuse(pa, torch, spec, mode, keep):
    """Arguments for another mode on tensors already on the GPU (the workspace is sized anew)."""
    q, k, v, out, ws, _ = keep
    a = pa.make_args(q, k, v, out, causal=spec.causal, mode=mode)
    need = pa.sage_attn_workspace_bytes(a)
    if need > ws.numel():
        del ws
        ws = torch.empty(need, dtype=torch.uint8, device=q.device)
    a.workspace, a.workspace_bytes = ws.data_ptr(), ws.numel()
    return a, (q, k, v, out, ws, None)


if __name__ == "__main__":
    main()
