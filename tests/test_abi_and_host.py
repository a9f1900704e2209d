"""CPU-side checks of the C-ABI library: it loads without a GPU, exports every function that
include/sage_attn.h declares, sizes workspaces consistently and rejects bad arguments on the
host before anything is launched.  No compute call is made here."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    import paper_2411_10958_amd as pa
    if not os.path.exists(pa.lib_path()):
        pytest.skip("libsageattn.so is not built (run __graft_entry__.build())")
    return pa, pa.load_library()


def _declared_functions():
    with open(os.path.join(ROOT, "include", "sage_attn.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    return sorted(set(re.findall(r"\b(sage_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    pa, lib = _lib()
    names = _declared_functions()
    assert {"sage_attn_fwd", "sage_attn_fwd_ex", "sage_attn_quant", "sage_attn_workspace_bytes",
            "sage_attn_prologue", "sage_attn_core", "sage_attn_debug_qk", "sage_attn_release",
            "sage_status_string"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in sage_attn.h but not exported"


def test_binding_has_the_same_names():
    pa, _ = _lib()
    for n in _declared_functions():
        assert hasattr(pa, n), f"binding lacks {n}"


def _args(pa, **kw):
    from paper_2411_10958_amd.binding import sage_attn_args
    a = sage_attn_args()
    a.B, a.H, a.H_kv, a.N, a.d, a.mode, a.dtype = 4, 32, 32, 4096, 128, 0, 1
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def test_workspace_size_formula():
    pa, _ = _lib()
    a = _args(pa)
    n = pa.sage_attn_workspace_bytes(a)
    BH, N, d = 128, 4096, 128
    codes = BH * N * d * 5 // 2          # 6-bit Q^ and K^ codes, 8-bit V^ codes
    delta_s = BH * (N // 128) * N * 4
    assert codes + delta_s <= n <= codes + delta_s + 16 * 1024 * 1024
    a8 = _args(pa, mode=1)
    n8 = pa.sage_attn_workspace_bytes(a8)                              # no Delta-S, 8-bit Q^ and K^ codes
    assert 3 * BH * N * d <= n8 <= 3 * BH * N * d + 16 * 1024 * 1024
    # ragged N rounds up to whole tiles; grouped KV heads shrink K/V storage
    assert pa.sage_attn_workspace_bytes(_args(pa, N=4097)) > n
    assert pa.sage_attn_workspace_bytes(_args(pa, H_kv=8)) < n
    assert n % 256 == 0
    # the smooth-V option adds only the per-channel partial sums (one per 256 tokens) and means of V
    assert 0 < pa.sage_attn_workspace_bytes(_args(pa, flags=1)) - n <= 128 * 128 * (8 * (N // 256) + 4) + 1024
    # switching a smoothing off changes values, not storage
    assert pa.sage_attn_workspace_bytes(_args(pa, flags=2 | 4)) == n
    assert pa.sage_attn_workspace_bytes(_args(pa, flags=8)) == n          # FP32 Delta-S: same storage


def test_key_split_policy():
    """sage_attn_kv_splits (host logic only): the library splits the key range by itself only when a launch has fewer
    than 256 tiles, into enough chunks for about 512 workgroups, at least 8 key blocks per chunk and at most 64; the
    caller's number is honoured up to the same limits; finer group maps and other P~V data types never split.  Short
    queries on grouped KV heads (2..8 query heads per KV head, all their queries within 128) count one tile per KV head."""
    pa, _ = _lib()
    S = lambda **kw: pa.sage_attn_kv_splits(_args(pa, **kw))
    assert S() == 1                                                   # 4096 tiles: nothing to fill
    assert S(B=1, H=1, H_kv=1) == 8                                       # 32 tiles, 64 key blocks: 8 blocks per chunk at least
    assert S(B=1, H=8, H_kv=8, N=128, N_kv=32768) == 64                      # 8 tiles: 512 / 8 = 64 chunks of 8 blocks
    # a decode step of 128 query heads on 32 KV heads: the 4 heads of a group share a tile, 32 tiles, 512 / 32 chunks
    assert S(B=4, H=32, H_kv=8, N=1, N_kv=32768, causal=1) == 16
    assert S(B=4, H=32, H_kv=8, N=32, N_kv=32768, causal=1) == 16     # 4 heads x 32 queries still fit one tile
    assert S(B=4, H=32, H_kv=8, N=33, N_kv=32768, causal=1) == 4      # ... 33 do not: a tile per query head, 512 / 128
    assert S(B=4, H=32, H_kv=2, N=1, N_kv=32768, causal=1) == 4       # 16 query heads per KV head: not packed
    assert S(B=64, H=32, H_kv=8, N=1, N_kv=4096) == 1                 # 512 packed tiles fill the chip unsplit
    assert S(B=1, H=2, H_kv=2, N=1, N_kv=512) == 1                           # too few key blocks to cut
    assert S(B=2, H=32, N=512) == 1                                   # 256 tiles: not split
    assert S(B=2, H=32, N=512, kv_splits=3) == 1                      # ... and 8 key blocks cannot be cut into 3 chunks of 8
    assert S(kv_splits=4) == 4 and S(kv_splits=64) == 8               # asked for: honoured up to one chunk per 8 blocks
    assert S(B=1, H=1, H_kv=1, kv_splits=1) == 1                            # switched off
    assert S(B=1, H=1, H_kv=1, group_map=2) == 1 and S(B=1, H=1, H_kv=1, pv_format=1) == 1
    assert S(kv_splits=65) == 0 and S(kv_splits=-1) == 0              # invalid arguments


def test_argument_errors_are_found_on_the_host():
    pa, lib = _lib()
    bad = [dict(d=96), dict(d=512), dict(mode=2), dict(dtype=3), dict(flags=64), dict(flags=-1), dict(N=(1 << 24) + 1), dict(N_kv=(1 << 24) + 1), dict(group_map=5), dict(group_map=-1), dict(layout=2), dict(pv_format=3),
           dict(pv_format=1, group_map=2)]
    for kw in bad:
        a = _args(pa, **kw)
        assert pa.sage_attn_workspace_bytes(a) == 0
        assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -2, kw
    assert pa.sage_attn_workspace_bytes(_args(pa, B=600, H=128, H_kv=128)) == 0      # B * H beyond the grid limit
    for kw in [dict(N=0), dict(B=-1), dict(H_kv=5)]:
        a = _args(pa, **kw)
        assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -1, kw
    a = _args(pa, cu_seqlens_q=4096)   # a packed variable-length batch needs the token-major layout
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -2
    a = _args(pa, cu_seqlens_k=4096)   # key prefix sums without query prefix sums
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -1
    a = _args(pa, cu_seqlens_q=4096, layout=1)
    assert pa.sage_attn_workspace_bytes(a) == pa.sage_attn_workspace_bytes(_args(pa, layout=1))
    a = _args(pa)                      # valid shapes but null tensors
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -1
    a.q = a.k = a.v = a.out = 4096     # non-null, but no workspace: rejected before any launch
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -3
    a.k = 4096 + 2                     # tensors must be 16-byte aligned
    assert lib.sage_attn_fwd_ex(ctypes.byref(a)) == -1
    a.k = 4096
    assert lib.sage_attn_quant(ctypes.byref(a), None) == -1
    assert lib.sage_attn_debug_qk(ctypes.byref(a), 0, 0, 0, 0, None) == -1
    assert lib.sage_attn_fwd_ex(None) == -1
    assert pa.sage_status_string(0) == "ok" and "workspace" in pa.sage_status_string(-3)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2411_10958_amd.binding as b
    monkeypatch.setenv("SAGEATTN_LIB", str(tmp_path / "nope.so"))
    monkeypatch.setattr(b, "_LIB", None)
    with pytest.raises(FileNotFoundError):
        b.load_library()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr


def test_header_is_plain_c(tmp_path):
    """include/sage_attn.h is a C header: a C11 compiler takes it with no HIP or C++ in sight."""
    import subprocess
    src = tmp_path / "t.c"
    src.write_text('#include "sage_attn.h"\nint main(void) { sage_attn_args a; (void)a; return sizeof(sage_quant_out) > 0 ? 0 : 1; }\n')
    res = subprocess.run(["gcc", "-std=c11", "-Wall", "-Werror", "-pedantic", "-fsyntax-only", "-I", os.path.join(ROOT, "include"),
                          str(src)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
