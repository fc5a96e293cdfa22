"""Pins for the CPU oracle's codes of 3 and 6 bits (Eq. 3 with N = 3, 6; Sec. 3.4 and App. C name these widths; no GPU).

The packing is a row-wise little-endian bit stream (code k in bits [N k, N k + N) of the row's words).  Each test ties
uref.wq_dequant / wq_linear / quantize_sym_bits to something other than itself: Python's arbitrary-precision integers
as the bit stream, numpy's unpackbits as a second unpacker, exact rational arithmetic on tiny inputs, the already
pinned 4-bit functions (a 3-bit code is a 4-bit code below 8; a 6-bit matrix whose codes stay below 16 is a 4-bit
matrix; with power-of-two scales a 6-bit weight is exactly 8 times its high-3-bit weight plus its low-3-bit weight),
single-code probes at word boundaries, and the closed form and error bound of Eq. 3.
"""
from fractions import Fraction

import numpy as np
import pytest

import workloads as wl
from workloads import Keep

WIDTHS = (3, 6)


def pack_stream(codes, bits):
    """[N][K] codes -> uint32 [N][K * bits / 32]: each row as ONE big integer sum(code_k << (bits k)), cut into 32-bit
    words from the low end (written out with Python integers, not via the oracle)."""
    N, K = codes.shape
    nw = K * bits // 32
    out = np.zeros((N, nw), dtype=np.uint32)
    for r in range(N):
        big = 0
        for k in range(K):
            big |= int(codes[r, k]) << (bits * k)
        for w in range(nw):
            out[r, w] = (big >> (32 * w)) & 0xFFFFFFFF
    return out


def pack_nibbles(codes):
    N, K = codes.shape
    out = np.zeros((N, K // 8), dtype=np.uint32)
    for j in range(8):
        out |= codes[:, j::8].astype(np.uint32) << np.uint32(4 * j)
    return out


def unpack_stream_numpy(qweight, bits):
    """Second unpacker: the little-endian bits of the row's bytes, regrouped `bits` at a time."""
    N, nw = qweight.shape
    bitsarr = np.unpackbits(qweight.view(np.uint8).reshape(N, nw * 4), axis=1, bitorder="little")
    K = nw * 32 // bits
    return (bitsarr.reshape(N, K, bits).astype(np.int64) * (1 << np.arange(bits))).sum(axis=2)


def dequant_numpy(qweight, scales, zeros, bits, group=128):
    q = unpack_stream_numpy(qweight, bits)
    z = np.repeat((zeros if zeros is not None else np.full(scales.shape, 1 << (bits - 1), np.uint8)).astype(np.int64), group, axis=1)
    s = np.repeat(scales.astype(np.float64), group, axis=1)
    return ((q - z).astype(np.float64) * s).astype(np.float16)          # exact product, one RNE rounding


@pytest.mark.parametrize("bits", WIDTHS)
def test_single_code_probes_across_word_boundaries(uref, bits):
    """One non-zero code lands in exactly one column, also where it runs over a word boundary (3 bits: columns 10, 21;
    6 bits: columns 5, 10); scale / zero switch at multiples of the group."""
    K = 256
    top = (1 << bits) - 1
    scales = np.array([[0.01, 0.02]], dtype=np.float16)
    zeros = np.array([[0, top - 1]], dtype=np.uint8)
    for k in (0, 1, 5, 10, 11, 20, 21, 22, 31, 32, 42, 53, 127, 128, 129, 138, 255):
        for code in (top, 5 % (top + 1), 1 << (bits - 1)):
            codes = np.zeros((1, K), dtype=np.int64)
            codes[0, k] = code
            wd = uref.wq_dequant(bits, pack_stream(codes, bits), scales, zeros).astype(np.float64)[0]
            exp = np.zeros(K)
            exp[128:] = float(np.float16(-(top - 1) * float(scales[0, 1])))
            exp[k] = float(np.float16((code - int(zeros[0, k // 128])) * float(scales[0, k // 128])))
            assert np.array_equal(wd, exp), (bits, k, code)


@pytest.mark.parametrize("bits", WIDTHS)
def test_the_two_unpackers_and_the_packer_agree(bits):
    """The pins' own tools: big-integer packing and unpackbits unpacking are inverse to each other."""
    rng = np.random.default_rng(5)
    codes = rng.integers(0, 1 << bits, size=(3, 256))
    assert np.array_equal(unpack_stream_numpy(pack_stream(codes, bits), bits), codes)


@pytest.mark.parametrize("bits", WIDTHS)
def test_dequant_exhaustive_q_z(uref, bits):
    """Every (q, z) for several scales (subnormal results, ties, large), every code at every position of a group
    (all alignments against the words): the exact product rounded once."""
    L = 1 << bits
    for s_bits in (0x2000, 0x211f, 0x2400, 0x1c01, 0x0003, 0x3555, 0x5000, 0x7bff):
        s16 = np.array([s_bits], dtype=np.uint16).view(np.float16)[0]
        # row (z, shift): column k holds code (k + shift) % L -> every code meets every bit alignment
        shifts = (0, 1, 3)
        codes = np.stack([(np.arange(128) + sh) % L for _ in range(L) for sh in shifts]).astype(np.int64)
        zcol = np.repeat(np.arange(L, dtype=np.uint8), len(shifts))[:, None]
        scales = np.full((codes.shape[0], 1), s16, dtype=np.float16)
        wd = uref.wq_dequant(bits, pack_stream(codes, bits), scales, zcol)
        with np.errstate(over="ignore"):
            exp = ((codes - zcol.astype(np.int64)).astype(np.float64) * float(s16)).astype(np.float16)
        assert np.array_equal(wd.view(np.uint16), exp.view(np.uint16)), (bits, hex(s_bits))
        for (zz, qq) in ((0, L - 1), (L - 1, 0), (L // 3, L // 2)):
            exact = (qq - zz) * Fraction(float(s16))
            with np.errstate(over="ignore"):
                want = float(np.float16(float(exact)))
            assert float(wd[zz * len(shifts), qq]) == want


@pytest.mark.parametrize("bits", WIDTHS)
@pytest.mark.parametrize("N,K,M", [(4, 128, 1), (5, 256, 3)])
def test_linear_brute_force_fractions(uref, bits, N, K, M):
    rng = np.random.default_rng(300 + K + bits)
    L = 1 << bits
    codes = rng.integers(0, L, size=(N, K))
    qweight = pack_stream(codes, bits)
    scales = rng.uniform(0.08 / L, 0.32 / L, size=(N, K // 128)).astype(np.float16)
    zeros = rng.integers(0, L, size=(N, K // 128), dtype=np.uint8)
    x = wl.gen_activations(rng, M, K)
    y = uref.wq_linear(bits, qweight, scales, zeros, x)
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


@pytest.mark.parametrize("bits", WIDTHS)
@pytest.mark.parametrize("keep", KEEPS)
@pytest.mark.parametrize("with_zeros", [True, False])
def test_matches_numpy_unpack_and_matmul(uref, bits, keep, with_zeros):
    from test_oracle_linear_pins import kept_lists
    rng = np.random.default_rng(17 + bits)
    N, K = 256, 512
    w = wl.gen_linear_bits(rng, N, K, bits)
    qweight, scales = w["qweight"], w["scales"]
    zeros = w["zeros"] if with_zeros else None
    rows, cols = kept_lists(N, K, keep)
    W = dequant_numpy(qweight, scales, zeros, bits)[np.ix_(rows, cols)]
    assert np.array_equal(uref.wq_dequant(bits, qweight, scales, zeros, keep).view(np.uint16), W.view(np.uint16))
    x = wl.gen_activations(rng, 3, len(cols))
    y = uref.wq_linear(bits, qweight, scales, zeros, x, keep)
    ref = x.astype(np.float64) @ W.astype(np.float64).T
    assert np.max(np.abs(y - ref)) <= 1e-11 * max(1.0, np.max(np.abs(ref)))
    pick = np.array([0, len(rows) - 1, len(rows) // 2], dtype=np.int32)
    assert np.array_equal(uref.wq_linear(bits, qweight, scales, zeros, x, keep, rows=pick), y[:, pick])


@pytest.mark.parametrize("bits", WIDTHS)
def test_small_codes_are_the_w4_matrix(uref, bits):
    """Codes and zero points below min(16, 2^bits) stored in `bits` bits: the same matrix as the 4-bit one with those
    nibbles, whose oracle functions have their own pins."""
    rng = np.random.default_rng(23 + bits)
    N, K = 64, 512
    top = min(16, 1 << bits)
    codes = rng.integers(0, top, size=(N, K))
    scales = rng.uniform(0.005, 0.02, size=(N, K // 128)).astype(np.float16)
    zeros = rng.integers(0, top, size=(N, K // 128), dtype=np.uint8)
    keep = Keep(n_keep=50, k_keep=400)
    x = wl.gen_activations(rng, 2, 400)
    w4, wb = pack_nibbles(codes), pack_stream(codes, bits)
    assert np.array_equal(uref.wq_dequant(bits, wb, scales, zeros, keep).view(np.uint16),
                          uref.w4_dequant(w4, scales, zeros, keep).view(np.uint16))
    assert np.array_equal(uref.wq_linear(bits, wb, scales, zeros, x, keep), uref.w4_linear(w4, scales, zeros, x, keep))


def test_w6_is_eight_times_high_codes_plus_low_codes(uref):
    """With power-of-two scales no weight is rounded, so W6(q, z) = 8 * W3(q >> 3, z >> 3) + W3(q & 7, z & 7) exactly,
    element by element and in the fp64 linear: ties the two widths (and their different word alignments) together."""
    rng = np.random.default_rng(29)
    N, K = 32, 256
    codes = rng.integers(0, 64, size=(N, K))
    zeros = rng.integers(0, 64, size=(N, K // 128), dtype=np.uint8)
    scales = (2.0 ** rng.integers(-12, -6, size=(N, K // 128))).astype(np.float16)
    w6 = uref.wq_dequant(6, pack_stream(codes, 6), scales, zeros).astype(np.float64)
    hi = uref.wq_dequant(3, pack_stream(codes >> 3, 3), scales, (zeros >> 3).astype(np.uint8)).astype(np.float64)
    lo = uref.wq_dequant(3, pack_stream(codes & 7, 3), scales, (zeros & 7).astype(np.uint8)).astype(np.float64)
    assert np.array_equal(w6, 8.0 * hi + lo)
    x = wl.gen_activations(rng, 2, K)
    y6 = uref.wq_linear(6, pack_stream(codes, 6), scales, zeros, x)
    yh = uref.wq_linear(3, pack_stream(codes >> 3, 3), scales, (zeros >> 3).astype(np.uint8), x)
    yl = uref.wq_linear(3, pack_stream(codes & 7, 3), scales, (zeros & 7).astype(np.uint8), x)
    assert np.max(np.abs(y6 - (8.0 * yh + yl))) <= 1e-12 * max(1.0, np.max(np.abs(y6)))


@pytest.mark.parametrize("bits", WIDTHS)
def test_no_zero_points_is_the_middle_code(uref, bits):
    rng = np.random.default_rng(31 + bits)
    w = wl.gen_linear_bits(rng, 16, 256, bits)
    mid = np.full((16, 2), 1 << (bits - 1), dtype=np.uint8)
    assert np.array_equal(uref.wq_dequant(bits, w["qweight"], w["scales"], None).view(np.uint16),
                          uref.wq_dequant(bits, w["qweight"], w["scales"], mid).view(np.uint16))


@pytest.mark.parametrize("bits", WIDTHS)
def test_symmetric_quantiser_equation_and_bound(uref, bits):
    """Eq. 3 with N = bits on random data: s = max|W| / (2^(N-1) - 1) (stored in fp16), code = clamp(rint(W / s)),
    stored + 2^(N-1); the round trip stays within half a step (plus the fp16 rounding of the weight)."""
    rng = np.random.default_rng(37 + bits)
    half = 1 << (bits - 1)
    w = rng.standard_normal((6, 384))
    qw, sc, zr = uref.quantize_sym_bits(bits, w)
    assert qw.shape == (6, 384 * bits // 32) and np.all(zr == half)
    mx = np.abs(w.reshape(6, 3, 128)).max(axis=2)
    assert np.array_equal(sc.view(np.uint16), (mx / float(half - 1)).astype(np.float16).view(np.uint16))
    s = np.repeat(sc.astype(np.float64), 128, axis=1)
    codes = unpack_stream_numpy(qw, bits) - half
    assert np.array_equal(codes, np.clip(np.rint(w / s), -half, half - 1))
    err = np.abs(uref.wq_dequant(bits, qw, sc, zr).astype(np.float64) - w)
    assert np.all(err <= 0.5 * s * 1.01 + 1e-3 * np.abs(w))
    # values on the grid survive exactly
    q = rng.integers(-(half - 1), half, size=(4, 256))
    q[:, ::128] = half - 1
    s16 = rng.uniform(0.005, 0.02, size=(4, 2)).astype(np.float16)
    wg = q * np.repeat(s16.astype(np.float64), 128, axis=1)
    qw2, sc2, zr2 = uref.quantize_sym_bits(bits, wg)
    assert np.array_equal(sc2.view(np.uint16), s16.view(np.uint16))
    assert np.array_equal(unpack_stream_numpy(qw2, bits) - half, q)


def test_other_widths_are_refused(uref):
    rng = np.random.default_rng(41)
    w = wl.gen_linear_bits(rng, 4, 128, 3)
    for bits in (0, 1, 2, 5, 7, 16):
        rc = uref.lib().uref_wq_dequant(bits, None, None, None, 4, 128, 128, None, None, 0)
        assert rc == -3
