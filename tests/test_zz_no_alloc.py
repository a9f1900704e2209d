"""The allocation-free entry point (sage_attn_fwd_static: the workspace is a fixed array inside the library's
device image) against sage_attn_fwd_ex on the same inputs: the same kernels on another workspace address, so
the outputs must be bit-identical - on two calls in a row, the second with a smaller input, which finds the
first call's contents in the shared array."""
import ctypes

import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def _pa():
    import paper_2411_10958_amd as pa
    pa.load_library()
    return pa


def _inputs(N, d, H, Hkv, causal, seed, Nk=None):
    spec = wl.WorkloadSpec(f"s{N}x{d}", 1, H, Hkv, N, d, "bf16", causal, 3.0, 1.5, 2, 10.0, 1.0, 77, 0.0, Nk or 0)
    data = wl.make_inputs(spec, seed)
    dev = torch.device("cuda:0")
    return tuple(wl.to_torch(data[n], spec.dtype, dev) for n in "qkv")


@pytest.mark.parametrize("mode", ["int4_fp8", "int8_fp8"])
def test_static_workspace_entry_point_equals_fwd_ex(mode):
    pa = _pa()
    # larger first; the last two split the key range (partial results in the shared array), the very last with the
    # query heads of a KV head in one tile
    calls = [(1000, 128, 4, 2, True, 0, None), (333, 128, 2, 1, True, 1, None), (200, 64, 2, 2, False, 2, None),
             (40, 128, 2, 2, True, 3, 1500), (3, 128, 8, 2, True, 4, 1200)]
    for N, d, H, Hkv, causal, seed, Nk in calls:
        print(f"static workspace: N={N} N_kv={Nk or N} d={d} H={H}/{Hkv} causal={causal} mode={mode}", flush=True)
        q, k, v = _inputs(N, d, H, Hkv, causal, seed, Nk)
        want, want_lse = pa.sage_attn_fwd_ex(q, k, v, causal=causal, mode=mode, return_lse=True)
        out = torch.full_like(q, 3.0)
        lse = torch.empty_like(want_lse)
        a = pa.make_args(q, k, v, out, causal=causal, mode=mode)
        a.lse = lse.data_ptr()
        assert pa.load_library().sage_attn_fwd_static(ctypes.byref(a)) == 0
        torch.cuda.synchronize()
        assert torch.equal(out, want), "output"
        assert torch.equal(lse, want_lse), "log-sum-exp"
    # the Python wrapper of the same call
    out2 = pa.sage_attn_fwd_static(q, k, v, torch.empty_like(q), causal=causal, mode=mode)
    torch.cuda.synchronize()
    assert torch.equal(out2, want)


def test_static_workspace_limit_is_an_error_not_a_fault():
    pa = _pa()
    lib = pa.load_library()
    # a shape whose workspace exceeds the built-in array: refused on the host, nothing launched (the tensors
    # are small stand-ins: a call that is refused never reads them)
    q = torch.zeros((1, 1, 128, 128), dtype=torch.bfloat16, device="cuda")
    a = pa.make_args(q, q, q, torch.empty_like(q))
    a.B, a.H, a.H_kv, a.N, a.N_kv = 4, 32, 32, 4096, 4096
    assert pa.sage_attn_workspace_bytes(a) > (64 << 20)
    assert lib.sage_attn_fwd_static(ctypes.byref(a)) == -3
    a.d = 96
    assert lib.sage_attn_fwd_static(ctypes.byref(a)) == -2
    assert lib.sage_attn_fwd_static(None) == -1
    torch.cuda.synchronize()
