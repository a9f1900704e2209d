"""The two forms of Algorithm 1's inner loop in the oracle against each other, on the CPU.

`attention_rows` evaluates the loop in the order the algorithm prints it and is the oracle of record;
`attention_rows_kernel_order` places the FP32 roundings where the gfx950 kernel places them (the static scale
448 of Sec. 3.3 folded into the exponent, the maximum nudged upward first).  These tests pin what the second
form may differ in: codes of P~ one step apart at a small rate, sums and outputs to a stated number of FP32
units otherwise - and they pin the comparison machinery of oracle/parity.py with mistakes planted on the CPU."""
import numpy as np
import pytest

import workloads as wl
from oracle import parity
from oracle import sage_oracle as so

f32, f64 = np.float32, np.float64


def _forms(pro, causal, pv="e4m3"):
    """Both forms over every smoothing block of a prepared head: total scores, mismatching codes, the set of code
    distances, and the largest relative differences of l * 2^e (the softmax denominator with its scale) and of
    the FP32 outputs."""
    N = pro["N"]
    tot = mism = 0
    dist = set()
    l_rel = o_rel = 0.0
    for i in range((N + 127) // 128):
        rows = slice(i * 128, min(i * 128 + 128, N))
        op, sp, cp = so.attention_rows(pro, rows, causal, out_dtype="fp32", return_state=True, return_codes=True)
        ok, sk, ck = so.attention_rows_kernel_order(pro, rows, causal, out_dtype="fp32", return_state=True, return_codes=True)
        cast = (lambda c: c.view(np.int8).astype(int)) if pv == "int8" else (lambda c: c.astype(int))
        dcode = cast(ck) - cast(cp)
        tot += dcode.size
        mism += int((dcode != 0).sum())
        dist |= set(int(x) for x in np.unique(dcode[dcode != 0]))
        # sum_t 2^S_t as either form carries it: l * 2^e (kernel order: e includes -log2 of the static scale)
        with np.errstate(over="ignore", invalid="ignore"):
            lp = np.log2(sp["l"].astype(f64)) + sp["e"].astype(f64)
            lk = np.log2(sk["l"].astype(f64)) + sk["e"].astype(f64)
        fin = np.isfinite(lp) & np.isfinite(lk)
        if fin.any():
            l_rel = max(l_rel, float(np.abs(lp[fin] - lk[fin]).max()))
        linf = np.abs(op).max(axis=1, keepdims=True)
        o_rel = max(o_rel, float((np.abs(ok.astype(f64) - op.astype(f64)) / np.where(linf > 0, linf, 1)).max()))
    return tot, mism, dist, l_rel, o_rel


@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
def test_kernel_order_form_differs_from_the_printed_form_by_single_code_steps_only(mode):
    """More than 10^7 scores of workload-like heads (channel offsets, outlier channels; full and causal): every code
    of P~ on which the two forms disagree is ONE step of the 8-bit format apart, the disagreements are rarer than
    one score in 10^4 (measured: about 2 in 10^5, all toward the smaller code - the upward nudge of the maximum),
    and the denominators agree to 2^-16 in log2 (every term carries the rounding of its exponent's argument,
    up to 2^-20 for |S - e| < 16, under either scale)."""
    total = 0
    for seed, (N, d, causal) in enumerate([(2048, 128, False), (2048, 128, True), (1536, 64, False), (2048, 128, False)]):
        spec = wl.WorkloadSpec("forms", 1, 1, 1, N, d, "bf16", causal, 3.0, 3.0, 4, 10.0, 1.0, 61)
        q, k, v = (wl.make_head(spec, w, 0, 0, seed) for w in "qkv")
        pro = so.quantize_head(q, k, v, mode=mode)
        tot, mism, dist, l_rel, o_rel = _forms(pro, causal)
        print(f"  N={N} d={d} causal={causal}: {tot} scores, {mism} codes differ ({mism / tot:.2e}), distances {dist}, "
              f"log2 denominators within {l_rel:.2e}, outputs within {o_rel:.2e} of the row maximum")
        assert dist <= {-1, 1}
        assert mism <= 1e-4 * tot
        assert l_rel <= 2.0 ** -16
        total += tot
    assert total >= 10_000_000


def test_forms_on_awkward_values_within_the_domain():
    """The awkward-value generator (heads scaled by powers of two, zero tokens / channels / heads, ties, heavy
    tails), scales limited so that |m| stays below 2^12 where the comparison is claimed: distances of differing
    codes still one step, every row the parity bar rejects is explained by those codes."""
    n_rows = 0
    for seed in range(12):
        rng = np.random.default_rng(4200 + seed)
        mode = ["int4_fp8", "int8_fp8"][seed % 2]
        pv = ["e4m3", "e4m3", "e5m2", "int8"][seed % 4]
        q = wl.awkward_values(rng, (1, 300, 64), "bf16", 2)[0]
        k = wl.awkward_values(rng, (1, 300, 64), "bf16", 2)[0]
        v = wl.awkward_values(rng, (1, 300, 64), "bf16", 4)[0]
        pro = so.quantize_head(q, k, v, mode=mode, pv_fmt=pv)
        tot, mism, dist, l_rel, o_rel = _forms(pro, seed % 3 == 0, pv)
        assert dist <= {-1, 1}, (seed, dist)
        # the kernel-order form's own output, rounded to the 16-bit type, passes the parity check against the printed form
        got = np.concatenate([so.attention_rows_kernel_order(pro, slice(i, min(i + 128, 300)), seed % 3 == 0, out_dtype="bf16")
                              for i in range(0, 300, 128)])
        chk = parity.OutputCheck("bf16", f"seed {seed} {mode} {pv}: ")
        chk.add_head(got, pro, seed % 3 == 0)
        chk.finish()
        n_rows += chk.n_rows
    assert n_rows == 12 * 300


@pytest.mark.parametrize("fmt", ["e4m3", "e5m2", "int8"])
def test_nudged_offset_keeps_the_largest_code_in_range(fmt):
    """Kernel-order form, the row's largest score S = m: E = 2^fl32(m - e) with e = fl32(fl32(m + 2^-22 |m|) - log2 fmax)
    stays within a hair of fmax (448, 57344, 127) - at most fmax (1 + 2^-20), far below the point where the 8-bit
    conversion overflows (464 for E4M3) - for |m| up to 2^24, including values chosen so that every rounding goes the
    wrong way; without the nudge it does not (checked, so that the pin would notice a nudge that does nothing: for
    |m| near 2^24 the largest E then lies well beyond fmax); and the price - P~ scaled down - stays between -2^-20 and 2^-21 |m| + 2^-19
    in log2."""
    fmax, log2f, enc, dec = so._FP8[fmt]
    rng = np.random.default_rng(3)
    ms = [rng.uniform(-1, 1, 200000) * np.exp2(rng.integers(-4, 25, 200000))]
    # adversarial: m just below / above the points where m - log2 fmax crosses a power of two (the spacing of e halves)
    for p in range(-3, 25):
        base = f32(2.0 ** p) + log2f
        ms.append(np.nextafter(f32(base), f32(np.inf)) + np.arange(-64, 64) * np.spacing(f32(base)))
        ms.append(-base + np.arange(-64, 64) * np.spacing(f32(base)))
    m = np.concatenate(ms).astype(f32)
    m = m[np.abs(m) <= 2.0 ** 24]
    t = (np.abs(m).astype(f64) * 2.0 ** -22 + m.astype(f64)).astype(f32)
    e = (t - log2f).astype(f32)
    E = np.exp2((m - e).astype(f32).astype(f64)).astype(f32)
    assert (E <= fmax * (1 + 2.0 ** -20)).all(), f"largest E {E.max()}"
    shift = f64(log2f) - (m.astype(f64) - e.astype(f64))           # log2 of the factor P~ is scaled down by
    assert (shift >= -2.0 ** -20).all() and (shift <= 2.0 ** -21 * np.abs(m) + 2.0 ** -19).all()
    e0 = (m - log2f).astype(f32)                                     # no nudge: nearest rounding can land far below
    E0 = np.exp2((m - e0).astype(f32).astype(f64)).astype(f32)
    assert E0.max() >= fmax + 1           # (for the INT8 variant that is the byte 128, which the integer product reads as -128)


def test_parity_check_rejects_planted_mistakes():
    """The comparison of oracle/parity.py must fail on outputs that are wrong in ways the bar is meant to catch.
    The mistakes are planted on the CPU, in a copy of the kernel-order evaluation: a dropped Delta-S, a code two
    steps off on a heavy key, a row scaled by 1 + 2^-8."""
    spec = wl.WorkloadSpec("plant", 1, 1, 1, 384, 64, "bf16", False, 3.0, 3.0, 2, 10.0, 1.0, 62)
    q, k, v = (wl.make_head(spec, w, 0, 0, 0) for w in "qkv")
    pro = so.quantize_head(q, k, v)
    good = np.concatenate([so.attention_rows_kernel_order(pro, slice(i, i + 128), False, out_dtype="bf16") for i in range(0, 384, 128)])
    chk = parity.OutputCheck("bf16"); chk.add_head(good, pro, False); chk.finish()
    # (1) Delta-S dropped
    broken = dict(pro); broken["delta_s"] = np.zeros_like(pro["delta_s"])
    bad = np.concatenate([so.attention_rows_kernel_order(broken, slice(i, i + 128), False, out_dtype="bf16") for i in range(0, 384, 128)])
    chk = parity.OutputCheck("bf16"); chk.add_head(bad, pro, False)
    with pytest.raises(AssertionError):
        chk.finish()
    # (2) the heaviest key's code two steps down in every row of one block
    rows = slice(0, 128)
    _, codes = so.attention_rows(pro, rows, False, out_dtype="fp32", return_codes=True)
    codes = codes.copy()
    codes[np.arange(128), codes.argmax(axis=1)] -= 2
    bad = good.copy()
    bad[rows] = wl.round_to_dtype(so.attention_rows(pro, rows, False, out_dtype="fp32", p_codes=codes), "bf16")
    chk = parity.OutputCheck("bf16"); chk.add_head(bad, pro, False)
    with pytest.raises(AssertionError):
        chk.finish()
    # (3) one row scaled by 1 + 2^-8
    bad = good.copy(); bad[200] = wl.round_to_dtype(bad[200] * (1 + 2.0 ** -8), "bf16")
    if not np.array_equal(bad[200], good[200]):
        chk = parity.OutputCheck("bf16"); chk.add_head(bad, pro, False)
        with pytest.raises(AssertionError):
            chk.finish()


def test_fine_group_map_members():
    """"fine": every query its own group; keys in runs of 4 (16 groups per 64-key block, 4 consecutive members)."""
    gq, gk = so.group_map("fine", 300, "q"), so.group_map("fine", 300, "k")
    assert np.array_equal(gq, np.arange(300))
    assert gk.max() + 1 == 75 and all((gk == g).sum() == 4 for g in range(75))
    assert all(np.array_equal(np.nonzero(gk == g)[0], np.arange(4 * g, 4 * g + 4)) for g in (0, 17, 74))
    assert len(np.unique(gk[:64])) == 16
