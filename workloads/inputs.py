"""Seeded synthetic Q, K, V with the shapes and outlier structure of the workloads this
repository is measured on.

Values are drawn in float32 with numpy's default_rng, rounded (nearest-even) to the 16-bit
input type, and magnitudes below 2**-20 are flushed to zero so that column sums of up to
2**17 tokens are exact in float64 in any order.  Arrays are returned as float32 holding
exactly representable 16-bit values, laid out [B, H, N, d] (K, V: [B, H_kv, N, d]).
Every (batch, head) slice is generated from its own seed, so a single head of a large
configuration can be drawn without materialising the rest.
"""
import os
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class WorkloadSpec:
    name: str
    B: int
    H: int
    H_kv: int
    N: int
    d: int
    dtype: str          # "fp16" | "bf16"
    causal: bool
    k_offset_std: float  # per-channel offset of K (shared by all tokens of a head)
    q_offset_std: float  # per-channel offset of Q
    n_outlier_ch: int    # channels of Q and K whose per-channel offset is scaled by outlier_gain
    outlier_gain: float
    token_norm_max: float  # token-wise scale drawn log-uniformly from [1, token_norm_max]
    config_id: int
    v_bias: float = 0.0  # per-channel bias of V: sign random per channel, magnitude in v_bias +- 0.5
    N_kv: int = 0        # keys / values per head; 0 = N

    @property
    def kv_len(self):
        return self.N_kv or self.N

    def with_(self, **kw):
        return replace(self, **kw)


CONFIGS = {
    # tiny case the CPU oracle finishes in seconds
    "tiny": WorkloadSpec("tiny", 1, 2, 2, 256, 64, "fp16", False, 3.0, 1.0, 0, 1.0, 1.0, 1),
    # language-model prefill shape; also the paper's kernel-benchmark shape (B=4, H=32)
    "prefill4k": WorkloadSpec("prefill4k", 4, 32, 32, 4096, 128, "bf16", False, 3.0, 3.0, 4, 10.0, 1.0, 2),
    "causal8k": WorkloadSpec("causal8k", 1, 32, 32, 8192, 128, "bf16", True, 3.0, 3.0, 4, 10.0, 1.0, 3),
    "causal16k": WorkloadSpec("causal16k", 1, 32, 32, 16384, 128, "bf16", True, 3.0, 3.0, 4, 10.0, 1.0, 3),
    "causal32k": WorkloadSpec("causal32k", 1, 32, 32, 32768, 128, "bf16", True, 3.0, 3.0, 4, 10.0, 1.0, 3),
    # the causal 8k case with 256-wide heads (half the heads: the same operation count per head as two 128-wide ones)
    "causal8k_d256": WorkloadSpec("causal8k_d256", 1, 16, 16, 8192, 256, "bf16", True, 3.0, 3.0, 4, 10.0, 1.0, 6),
    # one decode step: a single new query per sequence against a 32k-token cache, grouped KV heads
    "decode32k": WorkloadSpec("decode32k", 4, 32, 8, 1, 128, "bf16", True, 3.0, 3.0, 4, 10.0, 1.0, 7, 0.0, 32768),
    # video-diffusion-like: ragged N, d=64, token norms vary
    "video17k": WorkloadSpec("video17k", 2, 48, 48, 17776, 64, "bf16", False, 4.0, 4.0, 0, 1.0, 8.0, 4),
    # the same with the channel-wise V bias quoted for a video model (Appendix "Smoothing V": 8 to 9)
    "video17k_vbias": WorkloadSpec("video17k_vbias", 2, 48, 48, 17776, 64, "bf16", False, 4.0, 4.0, 0, 1.0, 8.0, 4, 8.5),
    # long-context causal prefill with grouped KV heads (4 query heads per KV head)
    "long128k": WorkloadSpec("long128k", 1, 32, 8, 131072, 128, "bf16", True, 3.0, 3.0, 0, 1.0, 1.0, 5),
}


def spec_of(name):
    """A named configuration, or an ad-hoc shape written b<B>h<H>[k<H_kv>]n<N>[m<N_kv>]d<d><c|f> (c: causal, f: full),
    e.g. b4h32n8192d128c: bf16, the value recipe of `prefill4k` (unit normal, channel offsets, 4 outlier channels)."""
    if name in CONFIGS:
        return CONFIGS[name]
    import re
    m = re.fullmatch(r"b(\d+)h(\d+)(?:k(\d+))?n(\d+)(?:m(\d+))?d(\d+)([cf])", name)
    if not m:
        raise KeyError(f"{name}: not a configuration ({', '.join(CONFIGS)}) and not of the form b4h32n8192d128c")
    B, H, Hkv, N, Nkv, d = (int(x) if x else 0 for x in m.groups()[:6])
    return WorkloadSpec(name, B, H, Hkv or H, N, d, "bf16", m.group(7) == "c", 3.0, 3.0, 4, 10.0, 1.0, 8, 0.0, Nkv)


def round_to_dtype(x, dtype):
    """Round float32 values to the nearest fp16/bf16 value (ties to even), return float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "fp16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = x.view(np.uint32)
        with np.errstate(over="ignore"):
            u = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) & np.uint32(0xFFFF0000)
        return u.view(np.float32).reshape(x.shape)   # finite inputs far from overflow: no wrap-around
    raise ValueError(dtype)


def _finish(x, dtype):
    x = round_to_dtype(x, dtype)
    x[np.abs(x) < 2.0 ** -20] = 0.0
    return x


def _seed(spec, seed, kind, b, h):
    return np.random.SeedSequence([1000 * spec.config_id + seed, kind, b, h])


def _qk_like(spec, rng, offset_std, N):
    d = spec.d
    x = rng.standard_normal((N, d), dtype=np.float32)
    if spec.token_norm_max > 1.0:
        s = np.exp(rng.uniform(0.0, np.log(spec.token_norm_max), size=(N, 1))).astype(np.float32)
        x *= s
    off = (offset_std * rng.standard_normal((1, d))).astype(np.float32)
    if spec.n_outlier_ch > 0:
        # channel-wise outliers are biases shared by all tokens (the structure the paper's
        # smoothing removes): a few channels carry an offset outlier_gain times larger
        ch = rng.choice(d, size=spec.n_outlier_ch, replace=False)
        off[:, ch] *= np.float32(spec.outlier_gain)
    if offset_std > 0:
        x += off
    return x


def make_head(spec, which, b, h, seed=0):
    """One [N, d] slice: which in {"q","k","v"}; h is a query head for q, a KV head for k, v."""
    kind = {"q": 0, "k": 1, "v": 2}[which]
    rng = np.random.default_rng(_seed(spec, seed, kind, b, h))
    if which == "q":
        x = _qk_like(spec, rng, spec.q_offset_std, spec.N)
    elif which == "k":
        x = _qk_like(spec, rng, spec.k_offset_std, spec.kv_len)
    else:
        x = rng.standard_normal((spec.kv_len, spec.d), dtype=np.float32)
        if spec.v_bias > 0:
            sign = np.where(rng.random((1, spec.d)) < 0.5, -1.0, 1.0)
            x += (sign * rng.uniform(spec.v_bias - 0.5, spec.v_bias + 0.5, size=(1, spec.d))).astype(np.float32)
    return _finish(x, spec.dtype)


def make_inputs(spec, seed=0, heads=None):
    """Full tensors (or only the listed query heads `heads`, with their KV heads).

    Returns dict(q=[B,H',N,d], k=[B,Hkv',N,d], v=..., q_heads=[...], kv_heads=[...]).
    """
    if isinstance(spec, str):
        spec = CONFIGS[spec]
    g = spec.H // spec.H_kv
    q_heads = list(range(spec.H)) if heads is None else list(heads)
    kv_heads = sorted({h // g for h in q_heads})
    q = np.empty((spec.B, len(q_heads), spec.N, spec.d), np.float32)
    k = np.empty((spec.B, len(kv_heads), spec.kv_len, spec.d), np.float32)
    v = np.empty_like(k)
    jobs = [(q, "q", b, i, h) for b in range(spec.B) for i, h in enumerate(q_heads)]
    jobs += [(a, w, b, i, h) for a, w in ((k, "k"), (v, "v")) for b in range(spec.B) for i, h in enumerate(kv_heads)]

    def fill(job):
        arr, which, b, i, h = job
        arr[b, i] = make_head(spec, which, b, h, seed)

    if len(jobs) * spec.N * spec.d > (1 << 24):     # slices are independent and seeded one by one
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            list(ex.map(fill, jobs))
    else:
        for job in jobs:
            fill(job)
    return dict(q=q, k=k, v=v, q_heads=q_heads, kv_heads=kv_heads, spec=spec)


def awkward_values(rng, shape, dtype, lim=None):
    """[H, n, d] float32 values exactly representable in the 16-bit type, chosen to be awkward for a quantized
    attention path rather than typical: one of four kinds per call (few distinct values, so that many quotients
    x / delta are exact rounding ties; ordinary noise with channel offsets; heavy tails; small integers), every
    head scaled by its own power of two 2^e with -lim <= e <= lim/2, and, with some probability, an all-zero
    token, an all-zero channel and an all-zero head.  `rng` is a numpy Generator (the caller seeds it)."""
    H, n, d = shape
    kind = rng.integers(4)
    if kind == 0:
        x = rng.integers(-15, 16, size=shape).astype(np.float32) * 0.5
    elif kind == 1:
        x = rng.standard_normal(shape).astype(np.float32) + 3.0 * rng.standard_normal((H, 1, d)).astype(np.float32)
    elif kind == 2:
        x = (rng.standard_normal(shape) * np.exp(2.0 * rng.standard_normal(shape))).astype(np.float32)
    else:
        x = rng.integers(-7, 8, size=shape).astype(np.float32)
    if lim is None:
        lim = 14 if dtype == "fp16" else 30         # keep fp16 inside its range
    x = x * np.exp2(rng.integers(-lim, lim // 2 + 1, size=(H, 1, 1))).astype(np.float32)
    if rng.random() < 0.5:
        x[:, rng.integers(n)] = 0.0
    if rng.random() < 0.5:
        x[:, :, rng.integers(d)] = 0.0
    if rng.random() < 0.2:
        x[rng.integers(H)] = 0.0
    return round_to_dtype(np.clip(x, -6e4, 6e4) if dtype == "fp16" else x, dtype)


def flops(spec):
    """Operation count used for TOPS: 4*B*H*N*N_kv*d; under a causal mask the visible (query, key)
    pairs, N*(2*N_kv - N)/2, i.e. half of N^2 when N_kv = N."""
    pairs = float(spec.N) * spec.kv_len
    if spec.causal:
        pairs = float(spec.N) * (2.0 * spec.kv_len - spec.N) / 2.0
    return 4.0 * spec.B * spec.H * pairs * spec.d


def to_torch(x, dtype, device="cpu"):
    """float32 numpy array of exactly representable values -> torch tensor of the 16-bit type."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x))
    td = {"fp16": torch.float16, "bf16": torch.bfloat16}[dtype]
    return t.to(device=device).to(td)


def from_torch(t):
    return t.detach().to("cpu").float().numpy()
