"""The C ABI from a program that is neither Python nor torch: tests/abi_c/abi_smoke.c (plain C, HIP runtime
for device memory) calls sage_attn_fwd and sage_attn_fwd_ex and checks them against the definition of
attention evaluated on the host.  The program is compiled by paper_2411_10958_amd/build.py."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BIN = os.path.join(ROOT, "tests", "abi_c", "abi_smoke")


@pytest.mark.gpu
def test_plain_c_caller():
    if not os.path.exists(BIN):      # normally built by __graft_entry__.build(); a host-only gcc call otherwise
        from paper_2411_10958_amd import build as _build
        _build.build_abi_smoke(verbose=False)
    print("running the plain-C caller of the ABI", flush=True)
    res = subprocess.run([BIN], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=100)
    print(res.stdout, flush=True)
    assert res.returncode == 0 and "abi smoke ok" in res.stdout
