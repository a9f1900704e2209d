"""Output parity of the HIP path against the CPU oracle: the comparison the GPU tests, the smoke check and the
benchmark's accuracy report share.  TEST INFRASTRUCTURE, like the rest of this package: the product never imports it.

Two comparisons per row, both element by element on the same seeded inputs:

  A. against `oracle.sage_oracle.attention_rows`, Algorithm 1 evaluated as printed (the oracle of record), at the
     stated bar: |out - ref| <= 2e-3 * ||ref row||_inf (+ half a unit of the 16-bit output format, because the
     bar is meant for the FP32 result and the kernel rounds once more), cosine >= 0.9999 over everything a test
     compares;
  B. against `attention_rows_kernel_order`, the same algorithm with the FP32 roundings where the kernel has
     them, at KERNEL_TOL: what is left there is the hardware's own arithmetic (exponential to 1 ulp, summation
     order of l, the matrix instruction's internal alignment of the 64 products of a block, reciprocal
     instead of division).  Those errors are relative to the magnitude of the terms that are summed, not to the
     sum: bar B is therefore taken relative to the larger of the row norm of bar A and the norm of the same row
     computed with |V^| in place of V^ (sum_t P^_t |V^_tc| delta_V[c] / l / 448) - the two coincide unless the
     products of a channel cancel (Sec. 3.4 is about exactly this accumulation; the width of the gfx950
     instruction's internal alignment is what tests/test_gpu_accumulator_probe.py measures).  Bar A stays
     relative to the row norm alone, as stated.

A floating-point value decides an integer in this method - the 8-bit code of P~ - so two correct FP32
evaluations of Algorithm 1 can disagree on a code by one step, and a row in which such a code carries a large
softmax weight then differs by more than either bar.  No allowance is made for that: every row beyond a bar
must be EXPLAINED, i.e. the test shows that it differs from the as-printed oracle only through codes of P~ that
are one step apart:
  * beyond A, within B: the kernel-order oracle's codes differ from the printed form's by single steps only
    (checked), and the printed form recomputed with those codes in place of its own (everything else - m, P~, l
    - as printed) agrees with the GPU row to the bar;
  * beyond B: the hardware exponential is accurate to 1 ulp, not correctly rounded; the codes whose value E
    lies within 2^-21 of a rounding boundary are the only ones it can move; the row must agree, to the bar,
    with the printed form recomputed with one or two of those codes moved by one step.
Anything else fails the test.

The bars carry one more term, SCALE_COEF * |m| (m: the row's running maximum in base 2): the kernel folds the
static scale 448 of P~ into the exponent offset e = m - log2 448, which FP32 resolves to 2^-24 |e| at best and
which the kernel nudges upward by 2^-22 |m| so that the row's largest code cannot overflow; P~ and l are both
scaled by that amount, which cancels in O / l except for where the 8-bit grid falls.  For scores of ordinary
size (|m| < 100) the term is below 3e-5; it matters only for the awkward-value sweeps that scale heads by
large powers of two, where FP32 scores themselves no longer resolve more.  Beyond |m| = DOMAIN_M = 2^12 (natural-log
scores beyond +-2800) that term alone reaches half of the stated bar: such rows are outside the domain the bar A
and the cosine are claimed for, and are held to comparison B only (which carries the same term).
"""
import itertools

import numpy as np

from . import sage_oracle as so

OUT_TOL = 2e-3            # bar A: the tolerance the benchmark spec states for the output
COS_TOL = 0.9999
KERNEL_TOL = 5e-4         # bar B: room for the hardware's arithmetic only
SCALE_COEF = 2.0 ** -22   # per unit of |m|: the resolution of the folded exponent offset
DOMAIN_M = 2.0 ** 12      # rows whose running maximum |m| (base 2) exceeds this are compared with the kernel-order form only
NEAR = 2.0 ** -21         # relative distance to an 8-bit rounding boundary within which the 1-ulp exponential decides
# Results below the smallest normal FP32 number are not resolved: the hardware exponential returns 0 for results
# below 2^-126 (a rescaling factor alpha or a P~ that small) where the oracle's rounding of a float64 value keeps a
# subnormal, so a row whose whole output is that small (its dominant key has an all-zero V row) can differ by
# its entire, subnormal, magnitude.
FLOOR = 2.0 ** -126


def half_ulp16(x, dtype):
    """Half the spacing of the 16-bit output format at |x| (fp16: 10 mantissa bits, bf16: 7)."""
    mant = 10 if dtype == "fp16" else 7
    ax = np.maximum(np.abs(x).astype(np.float64), 2.0 ** -14 if dtype == "fp16" else 2.0 ** -126)
    return 0.5 * np.exp2(np.floor(np.log2(ax)) - mant)


def _row_scale(ref, vbar):
    """The row norm the bars are relative to: ||ref row||_inf; with the smooth-V option the larger of that and the
    norm of the centred part ref - mean(V), which is what the 8-bit P~V product computes before mean(V) is
    added back (when the two cancel, the output's own norm says nothing about the scale of that product)."""
    linf = np.abs(ref).max(axis=1, keepdims=True)
    if vbar is not None:
        linf = np.maximum(linf, np.abs(ref - vbar.astype(np.float64)[None, :]).max(axis=1, keepdims=True))
    return linf


def _abs_record(pro):
    """The head's record with |V^| in place of V^ and no mean to add back: either form of the oracle then returns
    sum_t P^_t |V^_tc| delta_V[c] / l / 448, the magnitude that rounding errors inside the P~V product scale with."""
    a = dict(pro)
    a["v_dec"] = np.abs(pro["v_dec"])
    a["vbar"] = None
    return a


def _allowed(ref, tol, m, dtype, vbar=None, scale=None):
    """scale: row norms [rows, 1] to use instead of the norm of `ref` (bar B)."""
    linf = _row_scale(ref, vbar) if scale is None else scale
    with np.errstate(invalid="ignore"):
        scale = np.where(np.isfinite(m), np.abs(m), 0.0).astype(np.float64)[:, None]
    return (tol + SCALE_COEF * scale) * linf + half_ulp16(ref, dtype) + FLOOR


def _near_boundary(E, fmt, width=NEAR):
    """Positions whose value E is within `width` (relative) of a rounding boundary of the 8-bit format, and the
    codes on either side of it."""
    enc = so._FP8[fmt][2]
    lo = enc((E.astype(np.float64) * (1.0 - width)).astype(np.float32)).view(np.uint8)
    hi = enc((E.astype(np.float64) * (1.0 + width)).astype(np.float32)).view(np.uint8)
    return lo != hi, lo, hi


class OutputCheck:
    """Collects blocks of GPU output rows with the oracle's record of their head, then verifies them (see the
    module text).  One instance per comparison a test makes; `finish()` asserts."""

    def __init__(self, dtype, label="", near=None):
        """near: optional function (pro, row) -> [N_kv] relative widths to use instead of NEAR when looking for the
        codes another correct evaluation could have decided differently (for options whose scores are only
        approximately the oracle's)."""
        self.dtype, self.label, self.near = dtype, label, near
        self.n_rows = self.over_a = self.over_b = self.n_outside = 0
        self.worst_a = self.worst_b = 0.0
        self.dot = self.gg = self.rr = 0.0
        self.unexplained = []
        self._abs = {}          # id(pro) -> _abs_record(pro)

    def _scale_b(self, ref_k64, pro, rows, causal, bkv, chunks):
        """Row norms bar B is relative to (module text)."""
        a = self._abs.get(id(pro))
        if a is None:
            a = self._abs[id(pro)] = _abs_record(pro)
        mag = self._eval("kernel", a, rows, causal, bkv, chunks)[0].astype(np.float64)
        return np.maximum(_row_scale(ref_k64, pro.get("vbar")), np.abs(mag).max(axis=1, keepdims=True))

    @staticmethod
    def _eval(form, pro, rows, causal, bkv, chunks, p_codes=None):
        """Either form of the oracle on `rows`, the key range walked in one piece or in `chunks` merged by
        `merge_key_chunks`.  Returns (FP32 output, state, codes, E or None)."""
        fn = so.FORMS[form]
        extra = dict(return_e=True) if form == "kernel" else dict(p_codes=p_codes)
        if chunks is None:
            r = fn(pro, rows, causal, bkv, "fp32", return_state=True, return_codes=True, **extra)
            return r if form == "kernel" else r + (None,)
        parts = [fn(pro, rows, causal, bkv, "fp32", return_state=True, return_codes=True, blocks=c, **extra) for c in chunks]
        out, st = so.merge_key_chunks(pro, [p[1] for p in parts], form, "fp32")
        codes = parts[0][2].copy()
        E = parts[0][3].copy() if form == "kernel" else None
        for c, p in zip(chunks[1:], parts[1:]):              # every chunk filled its own columns
            codes[:, c[0] * bkv:] = p[2][:, c[0] * bkv:]
            if E is not None:
                E[:, c[0] * bkv:] = p[3][:, c[0] * bkv:]
        return out, st, codes, E

    # ---- one block of rows inside one smoothing block of one head
    def add(self, got16, pro, rows, causal, bkv=so.BKV_ACC, chunks=None):
        """chunks: the key chunks [(j0, j1), ...] the kernel split this tile's key range into (None: one piece)."""
        got = np.asarray(got16, np.float64)
        ref_p, st_p, codes_p, _ = self._eval("printed", pro, rows, causal, bkv, chunks)
        ref_k, st_k, codes_k, E_k = self._eval("kernel", pro, rows, causal, bkv, chunks)
        assert np.isfinite(got).all(), f"{self.label}: non-finite output"
        ref_p64, ref_k64 = ref_p.astype(np.float64), ref_k.astype(np.float64)
        m = st_p["m"]
        vbar = pro.get("vbar")
        ex_a = (np.abs(got - ref_p64) - _allowed(ref_p64, OUT_TOL, m, self.dtype, vbar)).max(axis=1)
        scale_b = self._scale_b(ref_k64, pro, rows, causal, bkv, chunks)
        ex_b = (np.abs(got - ref_k64) - _allowed(ref_k64, KERNEL_TOL, m, self.dtype, vbar, scale_b)).max(axis=1)
        linf = _row_scale(ref_p64, vbar)[:, 0]
        safe = np.where(linf > 0, linf, 1.0)
        safe_b = np.where(scale_b[:, 0] > 0, scale_b[:, 0], 1.0)
        # reported: the largest deviation beyond the rounding to the 16-bit output type, relative to the row scale
        self.worst_a = max(self.worst_a, float(((np.abs(got - ref_p64) - half_ulp16(ref_p64, self.dtype)).max(axis=1) / safe).max()))
        self.worst_b = max(self.worst_b, float(((np.abs(got - ref_k64) - half_ulp16(ref_k64, self.dtype)).max(axis=1) / safe_b).max()))
        self.n_rows += len(got)
        with np.errstate(invalid="ignore"):
            inside = ~(np.abs(m) > DOMAIN_M)
        self.n_outside += int((~inside).sum())
        gi, ri = got[inside], ref_p64[inside]
        self.dot += float((gi * ri).sum()); self.gg += float((gi * gi).sum()); self.rr += float((ri * ri).sum())
        bad_a, bad_b = (ex_a > 0) & inside, ex_b > 0
        self.over_a += int(bad_a.sum()); self.over_b += int(bad_b.sum())
        if not (bad_a.any() or bad_b.any()):
            return
        ridx = np.arange(pro["N"])[rows]
        pv_exact = pro["pv_exact"]
        for i in np.nonzero(bad_a | bad_b)[0]:
            why = "unquantized P~: no codes to explain a difference with" if pv_exact else \
                self._explain(got[i], pro, int(ridx[i]), causal, bkv, codes_p[i], codes_k[i], E_k[i], float(m[i]),
                              beyond_b=bool(bad_b[i]), chunks=chunks, scale_b=scale_b[i:i + 1])
            if why is not None:
                self.unexplained.append(f"row {int(ridx[i])}: {why} (excess A {ex_a[i]:.3e}, B {ex_b[i]:.3e})")

    def _explain(self, got, pro, r, causal, bkv, cp, ck, Ek, m, beyond_b, chunks=None, scale_b=None):
        """None if the row is explained, else the reason it is not."""
        step = ck.view(np.int8).astype(int) - cp.view(np.int8).astype(int) if pro["pv_fmt"] == "int8" \
            else ck.astype(int) - cp.astype(int)
        if np.abs(step).max(initial=0) > 1:
            return f"kernel-order and printed codes differ by {np.abs(step).max()} steps"
        mm = np.array([m], np.float32)

        def agrees(codes, tol):
            sub = self._eval("printed", pro, np.array([r]), causal, bkv, chunks, p_codes=codes[None, :])[0].astype(np.float64)
            scale = scale_b if tol == KERNEL_TOL else None
            return bool((np.abs(got[None, :] - sub) <= _allowed(sub, tol, mm, self.dtype, pro.get("vbar"), scale)).all())

        if not beyond_b:
            return None if agrees(ck, OUT_TOL) else "differs from the printed form by more than the kernel-order codes"
        # beyond the kernel-order bar: only codes decided within 1 ulp of the exponential can differ
        width = NEAR
        if self.near is not None:
            w = np.asarray(self.near(pro, r), np.float64)
            width = np.concatenate([w, np.zeros(len(Ek) - len(w))])[:len(Ek)] + NEAR
        near, lo, hi = _near_boundary(Ek, pro["pv_fmt"], width)
        cand = np.nonzero(near)[0]
        if len(cand) == 0 or len(cand) > 12:
            return f"{len(cand)} codes near a rounding boundary"
        for k in (1, 2):
            for pick in itertools.combinations(cand, k):
                codes = ck.copy()
                for t in pick:
                    codes[t] = hi[t] if ck[t] == lo[t] else lo[t]
                if agrees(codes, KERNEL_TOL):
                    return None
        return f"no one or two of the {len(cand)} near-boundary codes account for it"

    # ---- conveniences
    def add_head(self, got_head, pro, causal, blocks=None, bkv=so.BKV_ACC, splits=1):
        """got_head: [N, d] of one (batch, head); blocks: smoothing blocks to compare (default all); splits: key
        chunks per query tile the kernel used (sage_attn_kv_splits)."""
        N, bq = pro["N"], pro["bq"]
        for i in (range((N + bq - 1) // bq) if blocks is None else blocks):
            rows = slice(i * bq, min((i + 1) * bq, N))
            chunks = so.key_chunks(pro, i * bq, i * bq + bq - 1, causal, splits, bkv) if splits > 1 else None
            self.add(got_head[rows], pro, rows, causal, bkv, chunks)

    def finish(self):
        cos = self.dot / np.sqrt(self.gg * self.rr) if self.gg > 0 and self.rr > 0 else 1.0
        print(f"  {self.label}{self.n_rows} rows: vs printed form max-abs/row-Linf beyond output rounding {self.worst_a:.3e} (bar {OUT_TOL:g}), "
              f"cos {cos:.7f}; vs kernel-order form {self.worst_b:.3e} (bar {KERNEL_TOL:g}); rows beyond the bars "
              f"{self.over_a} / {self.over_b}, unexplained {len(self.unexplained)}"
              + (f"; {self.n_outside} rows with |m| > 2^12 held to the kernel-order form only" if self.n_outside else ""), flush=True)
        assert not self.unexplained, "rows beyond the bar that one-step codes of P~ do not explain:\n  " + \
            "\n  ".join(self.unexplained[:10])
        assert cos >= COS_TOL, f"cosine {cos}"
        return cos


def check_heads(got, data, causal, mode, dtype, label="", want_lse=False, splits=1, **oracle_kw):
    """got: [B, H, N, d] (float32 values of the 16-bit outputs); data: dict with q [B, H, N, d], k, v [B, H_kv, N_kv, d].
    Every head goes through `quantize_head(**oracle_kw)` and every smoothing block through OutputCheck.  Returns
    the per-head oracle records, pros[b][h] (with "lse" of the printed form when want_lse)."""
    B, H = data["q"].shape[:2]
    g = H // data["k"].shape[1]
    chk = OutputCheck(dtype, label)
    pros = []
    for b in range(B):
        pros.append([])
        for h in range(H):
            pro = so.quantize_head(data["q"][b, h], data["k"][b, h // g], data["v"][b, h // g], mode=mode, **oracle_kw)
            chk.add_head(got[b, h], pro, causal, splits=splits)
            if want_lse:
                N, bq = pro["N"], pro["bq"]
                lse = np.zeros(N, np.float32)
                for i in range((N + bq - 1) // bq):
                    rows = slice(i * bq, min((i + 1) * bq, N))
                    chunks = so.key_chunks(pro, i * bq, i * bq + bq - 1, causal, splits) if splits > 1 else None
                    st = OutputCheck._eval("printed", pro, rows, causal, so.BKV_ACC, chunks)[1]
                    lse[rows] = so.row_lse(pro, rows, st)
                pro["lse"] = lse
            pros[-1].append(pro)
    chk.finish()
    return pros
