"""Pins for the CPU oracle's 8-bit codes (Eq. 3 with N = 8; no GPU).

Each test ties uref.wq_dequant / wq_linear / quantize_sym_bits to something other than itself: exact rational
arithmetic on tiny inputs, an unpacker written separately with numpy, the already pinned 4-bit functions (an 8-bit
matrix whose codes stay below 16 IS a 4-bit matrix; with power-of-two scales an 8-bit weight is exactly 16 times its
high-nibble weight plus its low-nibble weight), byte order probes, and the closed form and error bound of Eq. 3.
"""
from fractions import Fraction

import numpy as np
import pytest

import workloads as wl
from workloads import Keep


def pack_bytes(codes):
    """[N][K] codes 0..255 -> uint32 [N][K/4], byte j of word w = column 4w + j (written out, not via the oracle)."""
    N, K = codes.shape
    out = np.zeros((N, K // 4), dtype=np.uint32)
    for j in range(4):
        out |= codes[:, j::4].astype(np.uint32) << np.uint32(8 * j)
    return out


def pack_nibbles(codes):
    N, K = codes.shape
    out = np.zeros((N, K // 8), dtype=np.uint32)
    for j in range(8):
        out |= codes[:, j::8].astype(np.uint32) << np.uint32(4 * j)
    return out


def unpack8_numpy(qweight, scales, zeros, group=128):
    N, K4 = qweight.shape
    q = qweight.view(np.uint8).reshape(N, K4 * 4).astype(np.int64)      # little-endian bytes of the words
    z = np.repeat((zeros if zeros is not None else np.full(scales.shape, 128, np.uint8)).astype(np.int64), group, axis=1)
    s = np.repeat(scales.astype(np.float64), group, axis=1)
    return ((q - z).astype(np.float64) * s).astype(np.float16)          # exact product, one RNE rounding


def test_w8_byte_order_and_group_boundaries(uref):
    """A single non-zero byte lands in exactly one column; scale / zero switch at multiples of the group."""
    N, K = 1, 256
    scales = np.array([[0.01, 0.02]], dtype=np.float16)
    zeros = np.array([[0, 130]], dtype=np.uint8)
    for k in (0, 1, 3, 4, 127, 128, 129, 255):
        qweight = np.zeros((N, K // 4), dtype=np.uint32)
        qweight[0, k // 4] = np.uint32(201 << (8 * (k % 4)))
        wd = uref.wq_dequant(8, qweight, scales, zeros).astype(np.float64)[0]
        exp = np.zeros(K)
        exp[128:] = float(np.float16(-130 * float(scales[0, 1])))
        exp[k] = float(np.float16((201 - int(zeros[0, k // 128])) * float(scales[0, k // 128])))
        assert np.array_equal(wd, exp)


def test_w8_dequant_exhaustive_q_z(uref):
    """Every (q, z) in 0..255 squared for several scales (subnormal results, ties, large): the exact rational product
    rounded once, computed with Fractions and numpy's fp64 -> fp16 conversion of the exactly representable product."""
    for s_bits in (0x2000, 0x211f, 0x2400, 0x1c01, 0x0003, 0x3555, 0x5000):
        s16 = np.array([s_bits], dtype=np.uint16).view(np.float16)[0]
        codes = np.tile(np.arange(256, dtype=np.int64), 256).reshape(256, 256)       # row z: q = 0..255
        qweight = pack_bytes(codes)
        scales = np.full((256, 2), s16, dtype=np.float16)
        zeros = np.repeat(np.arange(256, dtype=np.uint8)[:, None], 2, axis=1)
        wd = uref.wq_dequant(8, qweight, scales, zeros)
        q = codes
        z = np.arange(256, dtype=np.int64)[:, None]
        # (q - z) * s is exact in fp64 (9 bits times 11 bits), so fp64 -> fp16 is the single rounding
        with np.errstate(over="ignore"):
            exp = ((q - z).astype(np.float64) * float(s16)).astype(np.float16)
        assert np.array_equal(wd.view(np.uint16), exp.view(np.uint16)), hex(s_bits)
        # three spot checks in exact rationals
        for (zz, qq) in ((0, 255), (255, 0), (77, 200)):
            exact = (qq - zz) * Fraction(float(s16))
            assert float(wd[zz, qq]) == float(np.float16(float(exact)))


@pytest.mark.parametrize("N,K,M", [(4, 128, 1), (6, 256, 3)])
def test_w8_linear_brute_force_fractions(uref, N, K, M):
    rng = np.random.default_rng(300 + K)
    codes = rng.integers(0, 256, size=(N, K))
    qweight = pack_bytes(codes)
    scales = rng.uniform(0.0003, 0.0012, size=(N, K // 128)).astype(np.float16)
    zeros = rng.integers(0, 256, size=(N, K // 128), dtype=np.uint8)
    x = wl.gen_activations(rng, M, K)
    y = uref.wq_linear(8, qweight, scales, zeros, x)
    for r in range(N):
        wrow = []
        for k in range(K):
            exact = (int(codes[r, k]) - int(zeros[r, k // 128])) * Fraction(float(scales[r, k // 128]))
            wrow.append(Fraction(float(np.float16(float(exact)))))
        for m in range(M):
            exact = sum(Fraction(float(x[m, k])) * wrow[k] for k in range(K))
            assert abs(float(exact) - y[m, r]) <= 1e-13 * max(1.0, abs(float(exact)))


KEEPS = [
    Keep(),
    Keep(n_keep=200, k_keep=301),
    Keep(n_keep=4 * 54, row_seg_stride=64, row_seg_keep=54),
    Keep(k_keep=4 * 108, col_seg_stride=128, col_seg_keep=108),
    Keep(n_keep=2 * 82, k_keep=8 * 41, row_seg_stride=128, row_seg_keep=82, col_seg_stride=64, col_seg_keep=41),
]


@pytest.mark.parametrize("keep", KEEPS)
@pytest.mark.parametrize("with_zeros", [True, False])
def test_w8_matches_numpy_unpack_and_matmul(uref, keep, with_zeros):
    from test_oracle_linear_pins import kept_lists
    rng = np.random.default_rng(17)
    N, K = 256, 512
    qweight = rng.integers(0, 2 ** 32, size=(N, K // 4), dtype=np.uint64).astype(np.uint32)
    scales = rng.uniform(0.0003, 0.0012, size=(N, K // 128)).astype(np.float16)
    zeros = rng.integers(0, 256, size=(N, K // 128), dtype=np.uint8) if with_zeros else None
    rows, cols = kept_lists(N, K, keep)
    W = unpack8_numpy(qweight, scales, zeros)[np.ix_(rows, cols)]
    assert np.array_equal(uref.wq_dequant(8, qweight, scales, zeros, keep).view(np.uint16), W.view(np.uint16))
    x = wl.gen_activations(rng, 3, len(cols))
    y = uref.wq_linear(8, qweight, scales, zeros, x, keep)
    ref = x.astype(np.float64) @ W.astype(np.float64).T
    assert np.max(np.abs(y - ref)) <= 1e-11 * max(1.0, np.max(np.abs(ref)))
    # sampled rows are rows of the full result
    pick = np.array([0, len(rows) - 1, len(rows) // 2], dtype=np.int32)
    assert np.array_equal(uref.wq_linear(8, qweight, scales, zeros, x, keep, rows=pick), y[:, pick])


def test_w8_with_small_codes_is_the_w4_matrix(uref):
    """Codes and zero points below 16 stored as bytes: the same matrix as the 4-bit one with those nibbles, whose
    oracle functions have their own pins.  Also through the generic entry with bits = 4."""
    rng = np.random.default_rng(23)
    N, K = 64, 512
    codes = rng.integers(0, 16, size=(N, K))
    scales = rng.uniform(0.005, 0.02, size=(N, K // 128)).astype(np.float16)
    zeros = rng.integers(0, 16, size=(N, K // 128), dtype=np.uint8)
    keep = Keep(n_keep=50, k_keep=400)
    x = wl.gen_activations(rng, 2, 400)
    w4, w8 = pack_nibbles(codes), pack_bytes(codes)
    assert np.array_equal(uref.wq_dequant(8, w8, scales, zeros, keep).view(np.uint16),
                          uref.w4_dequant(w4, scales, zeros, keep).view(np.uint16))
    assert np.array_equal(uref.wq_linear(8, w8, scales, zeros, x, keep), uref.w4_linear(w4, scales, zeros, x, keep))
    assert np.array_equal(uref.wq_linear(4, w4, scales, zeros, x, keep), uref.w4_linear(w4, scales, zeros, x, keep))
    assert np.array_equal(uref.wq_dequant(4, w4, scales, zeros, keep).view(np.uint16),
                          uref.w4_dequant(w4, scales, zeros, keep).view(np.uint16))


def test_w8_is_sixteen_times_high_nibbles_plus_low_nibbles(uref):
    """With power-of-two scales no weight is rounded (|q - z| <= 255 fits fp16), so
    W8(q, z) = 16 * W4(q >> 4, z >> 4) + W4(q & 15, z & 15) exactly, element by element and in the fp64 linear."""
    rng = np.random.default_rng(29)
    N, K = 32, 256
    codes = rng.integers(0, 256, size=(N, K))
    zeros = rng.integers(0, 256, size=(N, K // 128), dtype=np.uint8)
    scales = (2.0 ** rng.integers(-12, -6, size=(N, K // 128))).astype(np.float16)
    w8 = uref.wq_dequant(8, pack_bytes(codes), scales, zeros).astype(np.float64)
    hi = uref.w4_dequant(pack_nibbles(codes >> 4), scales, (zeros >> 4).astype(np.uint8)).astype(np.float64)
    lo = uref.w4_dequant(pack_nibbles(codes & 15), scales, (zeros & 15).astype(np.uint8)).astype(np.float64)
    assert np.array_equal(w8, 16.0 * hi + lo)
    x = wl.gen_activations(rng, 2, K)
    y8 = uref.wq_linear(8, pack_bytes(codes), scales, zeros, x)
    yh = uref.w4_linear(pack_nibbles(codes >> 4), scales, (zeros >> 4).astype(np.uint8), x)
    yl = uref.w4_linear(pack_nibbles(codes & 15), scales, (zeros & 15).astype(np.uint8), x)
    assert np.max(np.abs(y8 - (16.0 * yh + yl))) <= 1e-12 * max(1.0, np.max(np.abs(y8)))


def test_w8_no_zero_points_is_zero_128(uref):
    rng = np.random.default_rng(31)
    N, K = 16, 256
    qweight = rng.integers(0, 2 ** 32, size=(N, K // 4), dtype=np.uint64).astype(np.uint32)
    scales = rng.uniform(0.0003, 0.0012, size=(N, K // 128)).astype(np.float16)
    z128 = np.full((N, K // 128), 128, dtype=np.uint8)
    assert np.array_equal(uref.wq_dequant(8, qweight, scales, None).view(np.uint16),
                          uref.wq_dequant(8, qweight, scales, z128).view(np.uint16))


def test_w8_symmetric_quantiser_equation_and_bound(uref):
    """Eq. 3 with N = 8 on random data: s = max|W| / 127 (stored in fp16), code = clamp(rint(W / s), -128, 127), stored
    + 128; the round trip stays within half a step (plus the fp16 rounding of the weight)."""
    rng = np.random.default_rng(37)
    w = rng.standard_normal((6, 384))
    qw, sc, zr = uref.quantize_sym_bits(8, w)
    assert qw.shape == (6, 96) and np.all(zr == 128)
    mx = np.abs(w.reshape(6, 3, 128)).max(axis=2)
    assert np.array_equal(sc.view(np.uint16), (mx / 127.0).astype(np.float16).view(np.uint16))
    s = np.repeat(sc.astype(np.float64), 128, axis=1)
    codes = qw.view(np.uint8).reshape(6, 384).astype(np.int64) - 128
    assert np.array_equal(codes, np.clip(np.rint(w / s), -128, 127))
    err = np.abs(uref.wq_dequant(8, qw, sc, zr).astype(np.float64) - w)
    assert np.all(err <= 0.5 * s * 1.01 + 1e-3 * np.abs(w))
    # values on the grid survive exactly, and N = 4 through the same function is the 4-bit quantiser
    q = rng.integers(-127, 128, size=(4, 256))
    q[:, ::128] = 127
    s16 = rng.uniform(0.0003, 0.0012, size=(4, 2)).astype(np.float16)
    wg = q * np.repeat(s16.astype(np.float64), 128, axis=1)
    qw2, sc2, zr2 = uref.quantize_sym_bits(8, wg)
    assert np.array_equal(sc2.view(np.uint16), s16.view(np.uint16))
    assert np.array_equal(qw2.view(np.uint8).reshape(4, 256).astype(np.int64) - 128, q)
    w4 = rng.standard_normal((4, 256))
    a, b = uref.quantize_sym_bits(4, w4), uref.quantize_sym(w4)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))
