"""ctypes binding of libsageattn.so: argument marshalling only.

Every function here has the name and meaning of the C entry point it calls (see
include/sage_attn.h).  Tensors are torch tensors on the GPU; their device pointers are passed
through untouched.  There is no fallback: if the library cannot be loaded, every call raises.
"""
import ctypes
import os

import torch

SAGE_MODE_INT4_FP8, SAGE_MODE_INT8_FP8 = 0, 1
SAGE_DT_FP16, SAGE_DT_BF16 = 0, 1
SAGE_FLAG_SMOOTH_V = 1
SAGE_FLAG_NO_SMOOTH_K = 2
SAGE_FLAG_NO_SMOOTH_Q = 4
SAGE_FLAG_FP32_DELTA_S = 8
SAGE_FLAG_FP64_DELTA_S = 16
SAGE_FLAG_DIGIT_DELTA_S = 32
SAGE_GROUPS_LANE, SAGE_GROUPS_BLOCK, SAGE_GROUPS_FINE, SAGE_GROUPS_TOKEN, SAGE_GROUPS_TENSOR = 0, 1, 2, 3, 4
_GROUPS = {"lane": 0, "block": 1, "fine": 2, "token": 3, "tensor": 4, 0: 0, 1: 1, 2: 2, 3: 3, 4: 4}
_GROUP_SIZES = {0: (2, 16), 1: (2, 16), 2: (1, 4), 3: (1, 1), 4: (2, 16)}     # queries, keys per stored scale
SAGE_LAYOUT_HND, SAGE_LAYOUT_NHD = 0, 1
_LAYOUTS = {"HND": 0, "NHD": 1, 0: 0, 1: 1}
_MODES = {"int4_fp8": 0, "int8_fp8": 1, 0: 0, 1: 1}
SAGE_PV_E4M3, SAGE_PV_E5M2, SAGE_PV_INT8 = 0, 1, 2
_PV_FORMATS = {"e4m3": 0, "e5m2": 1, "int8": 2, 0: 0, 1: 1, 2: 2}

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class SageError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: status {status} ({sage_status_string(status)})")


class sage_attn_args(ctypes.Structure):
    _fields_ = [("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("out", ctypes.c_void_p),
                ("B", ctypes.c_int), ("H", ctypes.c_int), ("H_kv", ctypes.c_int),
                ("N", ctypes.c_int), ("d", ctypes.c_int),
                ("causal", ctypes.c_int), ("sm_scale", ctypes.c_float),
                ("mode", ctypes.c_int), ("dtype", ctypes.c_int), ("flags", ctypes.c_int), ("group_map", ctypes.c_int), ("N_kv", ctypes.c_int), ("layout", ctypes.c_int),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("stream", ctypes.c_void_p),
                ("cu_seqlens_q", ctypes.c_void_p), ("cu_seqlens_k", ctypes.c_void_p), ("lse", ctypes.c_void_p),
                ("pv_format", ctypes.c_int),
                ("k_mean_in", ctypes.c_void_p), ("v_scale_in", ctypes.c_void_p), ("kv_splits", ctypes.c_int)]


class sage_quant_out(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("q_codes", "k_codes", "v_codes", "q_scale", "k_scale",
                                              "v_scale", "k_mean", "q_mean", "delta_s", "v_mean")]


def lib_path():
    """The in-tree library; SAGEATTN_LIB may name another build of the same sources."""
    return os.environ.get("SAGEATTN_LIB") or os.path.join(_PKG, "libsageattn.so")


def load_library():
    """Loads libsageattn.so from the package directory (built by paper_2411_10958_amd.build)."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise FileNotFoundError(f"{path} is missing: run `python -m paper_2411_10958_amd.build` "
                                    "(or __graft_entry__.build()) first")
        lib = ctypes.CDLL(path)
        P = ctypes.POINTER
        lib.sage_attn_workspace_bytes.restype = ctypes.c_size_t
        lib.sage_attn_workspace_bytes.argtypes = [P(sage_attn_args)]
        for name in ("sage_attn_fwd_ex", "sage_attn_prologue", "sage_attn_core", "sage_attn_fwd_static"):
            getattr(lib, name).restype = ctypes.c_int
            getattr(lib, name).argtypes = [P(sage_attn_args)]
        lib.sage_attn_fwd.restype = ctypes.c_int
        lib.sage_attn_fwd.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_int] * 5 + [ctypes.c_float, ctypes.c_int]
        lib.sage_attn_kv_splits.restype = ctypes.c_int
        lib.sage_attn_kv_splits.argtypes = [P(sage_attn_args)]
        lib.sage_attn_release.restype = None
        lib.sage_attn_kv_stats.restype = ctypes.c_int
        lib.sage_attn_kv_stats.argtypes = [P(sage_attn_args), ctypes.c_void_p, ctypes.c_void_p]
        lib.sage_attn_kv_stats_update.restype = ctypes.c_int
        lib.sage_attn_kv_stats_update.argtypes = [P(sage_attn_args), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_longlong,
                                                  ctypes.c_void_p, ctypes.c_void_p]
        lib.sage_attn_quant.restype = ctypes.c_int
        lib.sage_attn_quant.argtypes = [P(sage_attn_args), P(sage_quant_out)]
        lib.sage_attn_debug_qk.restype = ctypes.c_int
        lib.sage_attn_debug_qk.argtypes = [P(sage_attn_args)] + [ctypes.c_int] * 4 + [ctypes.c_void_p]
        lib.sage_attn_debug_mfma_fp8.restype = ctypes.c_int
        lib.sage_attn_debug_mfma_fp8.argtypes = [ctypes.c_void_p] * 5
        lib.sage_status_string.restype = ctypes.c_char_p
        lib.sage_status_string.argtypes = [ctypes.c_int]
        _LIB = lib
    return _LIB


def sage_status_string(status):
    return load_library().sage_status_string(int(status)).decode()


def _check(status, where):
    if status != 0:
        raise SageError(status, where)


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return SAGE_DT_BF16
    if t.dtype == torch.float16:
        return SAGE_DT_FP16
    raise TypeError(f"q, k, v must be float16 or bfloat16, got {t.dtype}")


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def make_args(q, k, v, out=None, causal=False, sm_scale=0.0, mode="int4_fp8", workspace=None, stream=None,
              smooth_v=False, group_map="lane", layout="HND", pv_format="e4m3", smooth_k=True, smooth_q=True,
              fp32_delta_s=False, kv_stats=None, kv_splits=0, delta_s=None):
    """delta_s: None (the library picks between the two exact forms of the Delta-S product), "digits", "fp64", or "fp32"
    (same as fp32_delta_s=True).
    Fills a sage_attn_args from torch tensors q [B,H,N,d], k/v [B,H_kv,N_kv,d] (layout "HND") or
    q [B,N,H,d], k/v [B,N_kv,H_kv,d] (layout "NHD"), contiguous, on the GPU.  `workspace` is a uint8 GPU tensor (or None); `stream` a torch.cuda.Stream (None = the
    current one)."""
    for name, t in (("q", q), ("k", k), ("v", v)):
        if not t.is_cuda or not t.is_contiguous() or t.dim() != 4:
            raise ValueError(f"{name} must be a contiguous 4-D GPU tensor")
    if k.shape != v.shape or k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("k and v must share shape; q, k, v must share dtype")
    nhd = _LAYOUTS[layout] == SAGE_LAYOUT_NHD
    B, H, N, d = (q.shape[0], q.shape[2], q.shape[1], q.shape[3]) if nhd else q.shape
    Hkv, Nk = (k.shape[2], k.shape[1]) if nhd else (k.shape[1], k.shape[2])
    if k.shape[0] != B or k.shape[3] != d:
        raise ValueError("k/v shape does not match q")
    if out is not None and (out.shape != q.shape or out.dtype != q.dtype or not out.is_contiguous()):
        raise ValueError("out must look like q")
    a = sage_attn_args()
    a.q, a.k, a.v, a.out = q.data_ptr(), k.data_ptr(), v.data_ptr(), (out.data_ptr() if out is not None else 0)
    a.B, a.H, a.H_kv, a.N, a.d = B, H, Hkv, N, d
    a.causal, a.sm_scale, a.mode, a.dtype = int(bool(causal)), float(sm_scale), _MODES[mode], _dtype_code(q)
    a.flags = ((SAGE_FLAG_SMOOTH_V if smooth_v else 0) | (0 if smooth_k else SAGE_FLAG_NO_SMOOTH_K) |
               (0 if smooth_q else SAGE_FLAG_NO_SMOOTH_Q) | (SAGE_FLAG_FP32_DELTA_S if (fp32_delta_s or delta_s == "fp32") else 0) |
               (SAGE_FLAG_FP64_DELTA_S if delta_s == "fp64" else 0) | (SAGE_FLAG_DIGIT_DELTA_S if delta_s == "digits" else 0))
    a.group_map = _GROUPS[group_map]
    a.N_kv = Nk
    a.layout = _LAYOUTS[layout]
    a.pv_format = _PV_FORMATS[pv_format]
    a.kv_splits = int(kv_splits)
    if kv_stats is not None:       # (k_mean, v_scale) float32 GPU tensors [B, H_kv, d], e.g. from sage_attn_kv_stats
        km, vs = kv_stats
        for name, t in (("k_mean", km), ("v_scale", vs)):
            # (the first extent is the batch size, or the number of sequences of a packed batch)
            if not t.is_cuda or t.dtype != torch.float32 or not t.is_contiguous() or t.dim() != 3 or \
                    tuple(t.shape[1:]) != (Hkv, d):
                raise ValueError(f"kv_stats: {name} must be a contiguous float32 GPU tensor of shape [B, H_kv, d]")
        a.k_mean_in, a.v_scale_in = km.data_ptr(), vs.data_ptr()
    if workspace is not None:
        a.workspace, a.workspace_bytes = workspace.data_ptr(), workspace.numel() * workspace.element_size()
    else:
        a.workspace, a.workspace_bytes = 0, 0
    s = stream if stream is not None else torch.cuda.current_stream(q.device)
    a.stream = s.cuda_stream
    return a


def sage_attn_workspace_bytes(args):
    return int(load_library().sage_attn_workspace_bytes(ctypes.byref(args)))


def sage_attn_kv_splits(args):
    """Key chunks per query tile the attention kernel will use for these arguments."""
    return int(load_library().sage_attn_kv_splits(ctypes.byref(args)))


def _alloc_workspace(args, device):
    need = sage_attn_workspace_bytes(args)
    if need == 0:
        raise SageError(load_library().sage_attn_prologue(ctypes.byref(args)) or -1, "sage_attn_workspace_bytes")
    ws = torch.empty(need, dtype=torch.uint8, device=device)
    args.workspace, args.workspace_bytes = ws.data_ptr(), need
    return ws


def sage_attn_fwd_ex(q, k, v, out=None, causal=False, sm_scale=0.0, mode="int4_fp8", workspace=None, stream=None,
                     smooth_v=False, group_map="lane", layout="HND", cu_seqlens_q=None, cu_seqlens_k=None,
                     max_seqlen_q=None, max_seqlen_k=None, return_lse=False, pv_format="e4m3", smooth_k=True,
                     smooth_q=True, fp32_delta_s=False, kv_stats=None, kv_splits=0, delta_s=None):
    """Whole forward pass.  Returns `out` (allocated if not given).  With cu_seqlens_q the batch is a packed
    variable-length one (see make_varlen_args) and `layout` is ignored.  With return_lse the result is
    (out, lse): lse float32 [B, H, N], or [H, total_q] for a variable-length batch."""
    if out is None:
        out = torch.empty_like(q)
    if cu_seqlens_q is not None:
        a = make_varlen_args(q, k, v, out, cu_seqlens_q, cu_seqlens_k, max_seqlen_q, max_seqlen_k, causal=causal,
                             sm_scale=sm_scale, mode=mode, workspace=workspace, stream=stream, smooth_v=smooth_v,
                             group_map=group_map, pv_format=pv_format, smooth_k=smooth_k, smooth_q=smooth_q,
                             fp32_delta_s=fp32_delta_s, kv_stats=kv_stats, kv_splits=kv_splits, delta_s=delta_s)
    else:
        a = make_args(q, k, v, out, causal, sm_scale, mode, workspace, stream, smooth_v, group_map, layout, pv_format,
                      smooth_k, smooth_q, fp32_delta_s, kv_stats, kv_splits, delta_s)
    lse = None
    if return_lse:
        shape = (a.H, q.shape[0]) if cu_seqlens_q is not None else (a.B, a.H, a.N)
        lse = torch.empty(shape, dtype=torch.float32, device=q.device)
        a.lse = lse.data_ptr()
    keep = _alloc_workspace(a, q.device) if workspace is None else workspace
    if workspace is None and stream is not None:
        keep.record_stream(stream)   # allocated on the current stream, used on another one
    _check(load_library().sage_attn_fwd_ex(ctypes.byref(a)), "sage_attn_fwd_ex")
    del keep  # torch's caching allocator keeps the block alive for work already queued on its streams
    return (out, lse) if return_lse else out


def sage_attn_fwd_static(q, k, v, out, causal=False, sm_scale=0.0, mode="int4_fp8", stream=None, **kw):
    """The forward pass on the library's built-in workspace (no allocation anywhere: `out` is the caller's).
    **kw as make_args."""
    a = make_args(q, k, v, out, causal, sm_scale, mode, None, stream, **kw)
    _check(load_library().sage_attn_fwd_static(ctypes.byref(a)), "sage_attn_fwd_static")
    return out


def make_varlen_args(q, k, v, out, cu_seqlens_q, cu_seqlens_k=None, max_seqlen_q=None, max_seqlen_k=None, **kw):
    """sage_attn_args of a packed variable-length batch: q / out [total_q, H, d], k / v [total_k, H_kv, d],
    cu_seqlens_* int32 GPU tensors [B + 1] (cu_seqlens_k None = the query one), max_seqlen_* the longest
    sequence (taken from the prefix sums, with a device-to-host copy, when not given).  **kw as make_args."""
    for name, t in (("q", q), ("k", k), ("v", v)):
        if not t.is_cuda or not t.is_contiguous() or t.dim() != 3:
            raise ValueError(f"{name} must be a contiguous 3-D GPU tensor")
    for name, t in (("cu_seqlens_q", cu_seqlens_q), ("cu_seqlens_k", cu_seqlens_k)):
        if t is not None and (not t.is_cuda or t.dtype != torch.int32 or t.dim() != 1 or not t.is_contiguous()):
            raise ValueError(f"{name} must be a contiguous 1-D int32 GPU tensor")
    if cu_seqlens_k is not None and cu_seqlens_k.numel() != cu_seqlens_q.numel():
        raise ValueError("cu_seqlens_q and cu_seqlens_k must have the same length")
    B = cu_seqlens_q.numel() - 1
    if B < 1:
        raise ValueError("cu_seqlens_q must hold at least two entries")
    if max_seqlen_q is None:
        max_seqlen_q = int((cu_seqlens_q[1:] - cu_seqlens_q[:-1]).max().item())
    if max_seqlen_k is None:
        ck = cu_seqlens_k if cu_seqlens_k is not None else cu_seqlens_q
        max_seqlen_k = int((ck[1:] - ck[:-1]).max().item())
    # the struct is filled through [1, tokens, heads, d] views; B, N, N_kv are then set for the packed batch
    a = make_args(q.unsqueeze(0), k.unsqueeze(0), v.unsqueeze(0), None if out is None else out.unsqueeze(0),
                  layout="NHD", **kw)
    a.B, a.N, a.N_kv = B, max(int(max_seqlen_q), 1), max(int(max_seqlen_k), 1)
    a.cu_seqlens_q = cu_seqlens_q.data_ptr()
    a.cu_seqlens_k = cu_seqlens_k.data_ptr() if cu_seqlens_k is not None else 0
    return a


def sage_attn_prologue(args):
    _check(load_library().sage_attn_prologue(ctypes.byref(args)), "sage_attn_prologue")


def sage_attn_core(args):
    _check(load_library().sage_attn_core(ctypes.byref(args)), "sage_attn_core")


def sage_attn_fwd(q, k, v, out, causal=False, sm_scale=0.0, mode="int4_fp8"):
    """The plain C signature: bf16, H_kv == H, default stream, library-owned workspace."""
    B, H, N, d = q.shape
    _check(load_library().sage_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, H, N, d, int(bool(causal)),
                                         float(sm_scale), _MODES[mode]), "sage_attn_fwd")
    return out


def sage_attn_kv_stats(k, v, layout="HND", pv_format="e4m3", cu_seqlens_k=None, max_seqlen_k=None, workspace=None,
                       stream=None):
    """mean(K) and delta_V alone (the statistics pass of the preprocessing): returns (k_mean, v_scale), float32
    [B, H_kv, d] each, in the form the `kv_stats` argument of the other calls takes.  With cu_seqlens_k, k and v are
    packed [total_k, H_kv, d] tensors and B is the number of sequences."""
    if cu_seqlens_k is not None:
        a = make_varlen_args(k, k, v, None, cu_seqlens_k, cu_seqlens_k, max_seqlen_k, max_seqlen_k, workspace=workspace,
                             stream=stream, pv_format=pv_format)
    else:
        a = make_args(k, k, v, None, workspace=workspace, stream=stream, layout=layout, pv_format=pv_format)
    keep = _alloc_workspace(a, k.device) if workspace is None else workspace
    km = torch.empty((a.B, a.H_kv, a.d), dtype=torch.float32, device=k.device)
    vs = torch.empty_like(km)
    st = load_library().sage_attn_kv_stats(ctypes.byref(a), ctypes.c_void_p(km.data_ptr()), ctypes.c_void_p(vs.data_ptr()))
    if st != 0:
        raise SageError(st, "sage_attn_kv_stats")
    del keep
    return km, vs


def sage_attn_kv_stats_update(k_new, v_new, state, layout="HND", pv_format="e4m3", workspace=None, stream=None):
    """Running statistics of a growing K / V.  k_new, v_new: the new tokens [B, H_kv, n_new, d]; state: None for the
    first chunk, else what the previous call returned.  Returns (k_mean, v_scale, state): the statistics of everything
    accumulated so far (as `kv_stats` takes them) and the updated state (k_sum float64, v_absmax float32, token count)."""
    a = make_args(k_new, k_new, v_new, None, workspace=workspace, stream=stream, layout=layout, pv_format=pv_format)
    keep = _alloc_workspace(a, k_new.device) if workspace is None else workspace
    shape = (a.B, a.H_kv, a.d)
    if state is None:
        ks = torch.empty(shape, dtype=torch.float64, device=k_new.device)
        vm = torch.empty(shape, dtype=torch.float32, device=k_new.device)
        n_before = 0
    else:
        ks, vm, n_before = state
    km = torch.empty(shape, dtype=torch.float32, device=k_new.device)
    vs = torch.empty_like(km)
    st = load_library().sage_attn_kv_stats_update(ctypes.byref(a), ctypes.c_void_p(ks.data_ptr()), ctypes.c_void_p(vm.data_ptr()),
                                                  ctypes.c_longlong(n_before), ctypes.c_void_p(km.data_ptr()),
                                                  ctypes.c_void_p(vs.data_ptr()))
    if st != 0:
        raise SageError(st, "sage_attn_kv_stats_update")
    del keep
    return km, vs, (ks, vm, n_before + a.N_kv)


def sage_attn_release():
    load_library().sage_attn_release()


def sage_attn_quant(q, k, v, causal=False, sm_scale=0.0, mode="int4_fp8", workspace=None, want=None,
                    smooth_v=False, group_map="lane", pv_format="e4m3", smooth_k=True, smooth_q=True,
                    fp32_delta_s=False, kv_stats=None, delta_s=None):
    """Preprocessing only; returns (dict of torch tensors in plain layouts, args, workspace)."""
    a = make_args(q, k, v, None, causal, sm_scale, mode, workspace, smooth_v=smooth_v, group_map=group_map,
                  pv_format=pv_format, smooth_k=smooth_k, smooth_q=smooth_q, fp32_delta_s=fp32_delta_s,
                  kv_stats=kv_stats, delta_s=delta_s)
    ws = _alloc_workspace(a, q.device) if workspace is None else workspace
    B, H, N, d = q.shape
    Hkv, Nk = k.shape[1], k.shape[2]
    dev = q.device
    int4 = _MODES[mode] == 0
    nqb = (N + 127) // 128
    qg, kg = _GROUP_SIZES[_GROUPS[group_map]]
    bufs = dict(
        q_codes=torch.empty((B, H, N, d), dtype=torch.int8, device=dev),
        k_codes=torch.empty((B, Hkv, Nk, d), dtype=torch.int8, device=dev),
        v_codes=torch.empty((B, Hkv, Nk, d), dtype=torch.uint8, device=dev),
        q_scale=torch.empty((B, H, (N + qg - 1) // qg), dtype=torch.float32, device=dev),
        k_scale=torch.empty((B, Hkv, (Nk + kg - 1) // kg), dtype=torch.float32, device=dev),
        v_scale=torch.empty((B, Hkv, d), dtype=torch.float32, device=dev),
        k_mean=torch.empty((B, Hkv, d), dtype=torch.float32, device=dev),
    )
    if int4:
        bufs["q_mean"] = torch.empty((B, H, nqb, d), dtype=torch.float32, device=dev)
        bufs["delta_s"] = torch.empty((B, H, nqb, Nk), dtype=torch.float32, device=dev)
    if smooth_v:
        bufs["v_mean"] = torch.empty((B, Hkv, d), dtype=torch.float32, device=dev)
    if want is not None:
        bufs = {n: t for n, t in bufs.items() if n in want}
    o = sage_quant_out()
    for n, _ in sage_quant_out._fields_:
        setattr(o, n, bufs[n].data_ptr() if n in bufs else 0)
    _check(load_library().sage_attn_quant(ctypes.byref(a), ctypes.byref(o)), "sage_attn_quant")
    return bufs, a, ws


def sage_attn_debug_qk(args, b, h, q_tile, kv_block, device="cuda"):
    out = torch.empty((128, 64), dtype=torch.int32, device=device)
    _check(load_library().sage_attn_debug_qk(ctypes.byref(args), b, h, q_tile, kv_block, _ptr(out)), "sage_attn_debug_qk")
    return out


def sage_attn_debug_mfma_fp8(a_codes, b_codes, c_in):
    """One v_mfma_f32_32x32x64_f8f6f4: a_codes, b_codes uint8 [64, 32] (E4M3), c_in float32 [64, 16]."""
    d = torch.empty_like(c_in)
    s = torch.cuda.current_stream(c_in.device).cuda_stream
    _check(load_library().sage_attn_debug_mfma_fp8(_ptr(a_codes), _ptr(b_codes), _ptr(c_in), _ptr(d), s),
           "sage_attn_debug_mfma_fp8")
    return d
