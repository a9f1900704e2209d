"""The paper's accumulator probe (Sec. 3.4: set A = B = 0, vary C, compare D bitwise) and its
extensions, run on the gfx950 instruction the P~V product uses.  These are the hardware facts
the kernel's accumulation design rests on: the C operand (the cross-block accumulator O) is
added in full FP32, while products inside one instruction are summed with reduced precision
within groups of 8 consecutive k (the block-confined, level-1 part)."""
import numpy as np
import pytest
import torch

from oracle import sage_oracle as so

pytestmark = pytest.mark.gpu


def _run(a, b, c):
    import paper_2411_10958_amd as pa
    dev = torch.device("cuda:0")
    d = pa.sage_attn_debug_mfma_fp8(torch.from_numpy(a).to(dev), torch.from_numpy(b).to(dev),
                                    torch.from_numpy(c).to(dev))
    torch.cuda.synchronize()
    return d.cpu().numpy()


def _pack(A, B):
    """A [32, 64], B [64, 32] E4M3 byte codes -> lane-major operands [64, 32]."""
    a = np.zeros((64, 32), np.uint8); b = np.zeros((64, 32), np.uint8)
    for l in range(64):
        a[l] = A[l % 32, 32 * (l // 32): 32 * (l // 32) + 32]
        b[l] = B[32 * (l // 32): 32 * (l // 32) + 32, l % 32]
    return a, b


def _unpack(d):
    """lane-major result [64, 16] -> matrix [32 rows, 32 columns]."""
    M = np.zeros((32, 32), d.dtype)
    for l in range(64):
        for v in range(16):
            M[8 * (v // 4) + 4 * (l // 32) + v % 4, l % 32] = d[l, v]
    return M


def test_c_operand_passes_through_bit_exactly():
    rng = np.random.default_rng(0)
    bits = rng.integers(0, 2 ** 23, (64, 16), dtype=np.uint32) | np.uint32(0x3F800000)   # 1.xxx, all 23 bits
    c = bits.view(np.float32) * np.exp2(rng.integers(-20, 20, (64, 16))).astype(np.float32)
    z = np.zeros((64, 32), np.uint8)
    d = _run(z, z, c)
    assert np.array_equal(d.view(np.uint32), c.view(np.uint32))      # no FP22-style truncation of C


def test_c_plus_block_sum_is_an_fp32_add():
    # one product per group of 8 k (so the in-group alignment cannot interfere): D = fl32(C + sum)
    rng = np.random.default_rng(1)
    A = np.zeros((32, 64), np.uint8); B = np.zeros((64, 32), np.uint8)
    ks = np.arange(0, 64, 8)
    codes = np.array([c for c in range(1, 0x7F)], np.uint8)
    A[:, ks] = rng.choice(codes, (32, 8)) | (rng.integers(0, 2, (32, 8)).astype(np.uint8) << 7)
    B[ks, :] = rng.choice(codes, (8, 32))
    C = (rng.standard_normal((32, 32)) * np.exp2(rng.integers(0, 18, (32, 32)))).astype(np.float32)
    c_l = np.zeros((64, 16), np.float32)
    for l in range(64):
        for v in range(16):
            c_l[l, v] = C[8 * (v // 4) + 4 * (l // 32) + v % 4, l % 32]
    a, b = _pack(A, B)
    got = _unpack(_run(a, b, c_l)).astype(np.float64)
    exact = so.e4m3_decode(A) @ so.e4m3_decode(B) + C.astype(np.float64)
    mag = np.abs(so.e4m3_decode(A)) @ np.abs(so.e4m3_decode(B)) + np.abs(C.astype(np.float64))
    err = np.abs(got - exact)
    # a few FP32 roundings at the magnitude of the terms; an accumulator with 13 mantissa bits
    # (the FP22 of the paper) would be off by up to 2^-14 of that magnitude
    assert np.all(err <= 4 * np.spacing(mag.astype(np.float32)))
    print("max err / magnitude:", float((err / mag).max()), "(2^-24 =", 2.0 ** -24, ")")
    # the paper's example magnitude: 2^16 + 2^-6 needs 23 bits
    A[:] = 0; B[:] = 0
    A[:, 0] = so.e4m3_encode(np.array([2.0 ** -3]))[0]; B[0, :] = so.e4m3_encode(np.array([2.0 ** -3]))[0]
    a, b = _pack(A, B)
    got = _unpack(_run(a, b, np.full((64, 16), 65536.0, np.float32)))
    assert np.all(got == np.float32(65536.0 + 2.0 ** -6))


def test_products_inside_one_instruction_use_a_narrow_aligned_sum():
    # two products in the same group of 8 k: the smaller survives down to 2^-12 of the larger
    # and is dropped from 2^-14 on; in different groups it survives to FP32 precision.
    def two(k_small, gap):
        A = np.zeros((32, 64), np.uint8); B = np.zeros((64, 32), np.uint8)
        A[:, 0] = so.e4m3_encode(np.array([256.0]))[0]; B[0, :] = so.e4m3_encode(np.array([256.0]))[0]
        es = 16 - gap
        A[:, k_small] = so.e4m3_encode(np.array([2.0 ** (es // 2)]))[0]
        B[k_small, :] = so.e4m3_encode(np.array([2.0 ** (es - es // 2)]))[0]
        a, b = _pack(A, B)
        return float(_unpack(_run(a, b, np.zeros((64, 16), np.float32)))[0, 0]) - 65536.0, 2.0 ** es
    for gap in (8, 10, 12):
        got, want = two(1, gap)
        assert got == want
    for gap in (14, 16, 20):
        got, want = two(1, gap)
        assert got == 0.0                       # lost: the gfx950 counterpart of the FP22 finding
    for gap in (14, 18, 22):
        got, want = two(8, gap)                  # another group of 8: kept
        assert got == want


def test_integer_codes_are_exact():
    rng = np.random.default_rng(2)
    Ai = rng.integers(-7, 8, (32, 64)); Bi = rng.integers(-7, 8, (64, 32))
    Ai[0, :] = 7; Bi[:, 0] = -7                       # extreme row/column
    a, b = _pack(so.e4m3_encode(Ai.astype(np.float64)), so.e4m3_encode(Bi.astype(np.float64)))
    c = np.full((64, 16), 3136.0, np.float32)         # the partial sum of a first 64-channel step
    got = _unpack(_run(a, b, c))
    assert np.array_equal(got, (Ai @ Bi + 3136).astype(np.float32))
