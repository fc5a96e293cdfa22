"""Pins for the CPU oracle's bfloat16 format (Sec. 4.1 names BF16 as the compute type).  No GPU.

bfloat16 is the upper half of a binary32.  The codec is tied to numpy's binary32 (decode) and to a
brute-force search for the nearest representable value (encode); the dequantised weights to the same
search over an independently unpacked matrix and to hand-computed roundings; the linear to numpy's fp64
matmul; the two formats to each other where both hold every quantity exactly.
"""
import numpy as np
import pytest

import workloads as wl
from workloads import Keep

GROUP = 128


def bf16_values(bits):
    with np.errstate(invalid="ignore"):     # signalling-nan patterns in the exhaustive decode test
        return _bf16_values(bits)


def _bf16_values(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# every finite non-negative bfloat16, ascending: bit patterns 0x0000 .. 0x7f7f are monotone in value
_FINITE = bf16_values(np.arange(0x7f80, dtype=np.uint16))


def nearest_bf16_bits(vals):
    """Nearest bfloat16 by search in the table of all of them; a tie goes to the even bit pattern."""
    vals = np.asarray(vals, dtype=np.float64)
    a = np.abs(vals)
    hi = np.clip(np.searchsorted(_FINITE, a, side="left"), 1, _FINITE.size - 1)
    lo = hi - 1
    dl, dh = a - _FINITE[lo], _FINITE[hi] - a
    pick = np.where(dl < dh, lo, np.where(dh < dl, hi, np.where(lo % 2 == 0, lo, hi)))
    pick = np.where(a == 0, 0, pick)
    return (pick | np.where(np.signbit(vals), 0x8000, 0)).astype(np.uint16)


def unpack_codes(qweight):
    N, K8 = qweight.shape
    sh = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    return ((qweight[:, :, None] >> sh) & np.uint32(15)).reshape(N, K8 * 8).astype(np.int64)


# ---------------------------------------------------------------- codec
def test_bf16_decode_all_bit_patterns(uref):
    bits = np.arange(65536, dtype=np.uint32)
    mine = np.array([uref.bf16_to_double(int(b)) for b in bits])
    ref = bf16_values(bits.astype(np.uint16))
    assert np.array_equal(np.isnan(mine), np.isnan(ref))
    m = ~np.isnan(ref)
    assert np.array_equal(mine[m], ref[m])
    assert np.array_equal(np.signbit(mine[m]), np.signbit(ref[m]))


def test_bf16_encode_inverts_decode(uref):
    for b in range(65536):
        v = uref.bf16_to_double(b)
        if v == v:
            assert uref.double_to_bf16(v) == b, hex(b)


def test_bf16_encode_is_nearest_ties_to_even(uref):
    rng = np.random.default_rng(3)
    vals = [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -40, 1.0 + 2.0 ** -8 - 2.0 ** -40,
            255.5, 256.5, 257.0, 2.0 ** -126, 2.0 ** -133, 2.0 ** -134, 3 * 2.0 ** -134, 2.0 ** -134 * 1.0000001,
            2.0 ** -126 - 2.0 ** -134]
    h = np.arange(0, 0x7f7f, 5)
    vals += list((_FINITE[h] + _FINITE[h + 1]) / 2) + list(-(_FINITE[h] + _FINITE[h + 1]) / 2)   # every 5th midpoint
    vals += list(rng.standard_normal(4000) * 10.0 ** rng.integers(-30, 30, 4000))
    mine = np.array([uref.double_to_bf16(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(mine, nearest_bf16_bits(vals))
    # overflow: the largest finite value is (2 - 2^-7) 2^127; from half an ulp above it on the result is inf
    top = (2.0 - 2.0 ** -7) * 2.0 ** 127
    assert uref.double_to_bf16(top) == 0x7f7f and uref.double_to_bf16(-top) == 0xff7f
    assert uref.double_to_bf16(top + 2.0 ** 118) == 0x7f7f          # below the midpoint
    assert uref.double_to_bf16(top + 2.0 ** 119) == 0x7f80          # the midpoint: ties to even = inf
    assert uref.double_to_bf16(1e300) == 0x7f80 and uref.double_to_bf16(-1e300) == 0xff80
    assert uref.double_to_bf16(float("inf")) == 0x7f80
    assert uref.double_to_bf16(0.0) == 0 and uref.double_to_bf16(-0.0) == 0x8000


# ---------------------------------------------------------------- dequantised weights
def one_group(q_codes, z, scale_bits):
    """A 1 x 128 matrix whose first len(q_codes) codes are given (the rest equal z, weight 0)."""
    codes = np.full(GROUP, z, dtype=np.uint32)
    codes[: len(q_codes)] = q_codes
    qweight = np.zeros((1, GROUP // 8), dtype=np.uint32)
    for k, c in enumerate(codes):
        qweight[0, k // 8] |= np.uint32(int(c) << (4 * (k % 8)))
    return qweight, np.array([[scale_bits]], dtype=np.uint16), np.array([[z]], dtype=np.uint8)


def test_dequant_bf16_hand_computed_roundings(uref):
    """s = 1 + 2^-7 (bits 0x3f81), z = 8.  The products (q - 8) s need more than 8 significant bits:
      7 s = 7.0546875   ulp 2^-5: 225.75 ulps -> 226 -> 7.0625
      5 s = 5.0390625   ulp 2^-5: 161.25 ulps -> 161 -> 5.03125
      3 s = 3.0234375   ulp 2^-6: 193.5  ulps -> tie, even 194 -> 3.03125
     -3 s               -> -3.03125;   1 s = s exactly;   0 -> +0."""
    qweight, scales, zeros = one_group([15, 13, 11, 5, 9, 8], 8, 0x3f81)
    w = uref.w4_dequant(qweight, scales, zeros, fmt="bf16")
    got = bf16_values(w[0, :6])
    assert list(got) == [7.0625, 5.03125, 3.03125, -3.03125, 1.0078125, 0.0]
    assert w[0, 5] == 0      # +0, not -0
    # the same codes in fp16 (s = 1 + 2^-7 is exact there too) round at 11 bits instead: all products exact
    w16 = uref.w4_dequant(qweight, np.array([[1.0 + 2.0 ** -7]], dtype=np.float16), zeros)
    assert list(w16[0, :6].astype(np.float64)) == [7.0546875, 5.0390625, 3.0234375, -3.0234375, 1.0078125, 0.0]


def test_dequant_bf16_exhaustive_q_z_scale(uref):
    """Every (q, z) pair against 128 scales spread over the format: nearest-value search on the exact product."""
    rng = np.random.default_rng(5)
    scale_bits = np.concatenate([rng.integers(0x3800, 0x4000, 120), [0x3f80, 0x3f81, 0x3fff, 0x0080, 0x0001, 0x3c23, 0x7000, 0x0000]])
    for sb in scale_bits.astype(np.uint16):
        s = float(bf16_values([sb])[0])
        for z in range(16):
            qweight, scales, zeros = one_group(list(range(16)), z, sb)
            w = uref.w4_dequant(qweight, scales, zeros, fmt="bf16")[0, :16]
            exact = (np.arange(16) - z).astype(np.float64) * s      # exact in fp64: 5 bits times 8 bits
            exp = nearest_bf16_bits(exact)
            # a zero product keeps the sign of (q - z) * s as fp64 forms it
            assert np.array_equal(w, exp), (hex(sb), z)


KEEPS = [
    Keep(),
    Keep(n_keep=21, k_keep=300),
    Keep(n_keep=27, row_seg_stride=16, row_seg_keep=9, row_seg_limit=48),
    Keep(k_keep=4 * 54, col_seg_stride=64, col_seg_keep=54),
    Keep(n_keep=2 * 12 + 2 * 5 + 4, row_seg_stride=16, row_seg_keep=12, row_seg_limit=32,
         row_seg2_stride=8, row_seg2_keep=5, row_seg2_limit=48, k_keep=200),
]


def kept(N, K, keep):
    r, k = np.arange(N), np.arange(K)
    if keep.row_seg_stride:
        m = np.where(r < keep.row_seg_limit, r % keep.row_seg_stride < keep.row_seg_keep,
                     np.where((keep.row_seg2_stride != 0) & (r < keep.row_seg2_limit),
                              (r - keep.row_seg_limit) % max(keep.row_seg2_stride, 1) < keep.row_seg2_keep, True))
        rows = r[m]
    else:
        rows = r[: keep.n_keep or N]
    cols = k[k % keep.col_seg_stride < keep.col_seg_keep] if keep.col_seg_stride else k[: keep.k_keep or K]
    return rows, cols


@pytest.mark.parametrize("keep", KEEPS, ids=[str(i) for i in range(len(KEEPS))])
@pytest.mark.parametrize("with_zeros", [True, False])
def test_bf16_dequant_and_linear_match_numpy(uref, keep, with_zeros):
    rng = np.random.default_rng(11)
    N, K, M = 52, 256, 3
    w = wl.gen_linear(rng, N, K, fmt="bf16")
    zeros = w["zeros"] if with_zeros else None
    rows, cols = kept(N, K, keep)
    z = w["zeros"].astype(np.int64) if with_zeros else np.full((N, K // GROUP), 8, dtype=np.int64)
    s = bf16_values(w["scales"])
    exact = (unpack_codes(w["qweight"]) - np.repeat(z, GROUP, axis=1)) * np.repeat(s, GROUP, axis=1)
    exp_bits = nearest_bf16_bits(exact)[np.ix_(rows, cols)]
    d = uref.w4_dequant(w["qweight"], w["scales"], zeros, keep, fmt="bf16")
    assert d.dtype == np.uint16 and np.array_equal(d, exp_bits)
    x = wl.gen_activations(rng, M, cols.size, fmt="bf16")
    y = uref.w4_linear(w["qweight"], w["scales"], zeros, x, keep, fmt="bf16")
    ref = bf16_values(x) @ bf16_values(exp_bits).T
    assert y.shape == ref.shape
    assert np.max(np.abs(y - ref)) <= 1e-12 * np.max(np.abs(ref))
    # sampled rows are the same numbers
    pick = [0, rows.size - 1, rows.size // 2]
    ys = uref.w4_linear(w["qweight"], w["scales"], zeros, x, keep, rows=pick, fmt="bf16")
    assert np.array_equal(ys, y[:, pick])


def test_formats_agree_where_both_are_exact(uref):
    """Power-of-two scales and activations with at most 8 significant bits are the same numbers in both
    formats, and (q - z) * 2^e needs 5 bits: dequantised weights and outputs must then be identical."""
    rng = np.random.default_rng(13)
    N, K, M = 24, 384, 2
    qweight = rng.integers(0, 2 ** 32, size=(N, K // 8), dtype=np.uint64).astype(np.uint32)
    zeros = rng.integers(0, 16, size=(N, K // GROUP), dtype=np.uint8)
    s = 2.0 ** rng.integers(-9, -3, size=(N, K // GROUP))
    x = rng.integers(-128, 129, size=(M, K)) / 64.0
    keep = Keep(n_keep=19, k_keep=300)
    x = x[:, :300]
    y16 = uref.w4_linear(qweight, s.astype(np.float16), zeros, np.ascontiguousarray(x.astype(np.float16)), keep)
    yb = uref.w4_linear(qweight, wl.to_bf16_bits(s), zeros, wl.to_bf16_bits(x), keep, fmt="bf16")
    assert np.array_equal(y16, yb)
    d16 = uref.w4_dequant(qweight, s.astype(np.float16), zeros, keep)
    db = uref.w4_dequant(qweight, wl.to_bf16_bits(s), zeros, keep, fmt="bf16")
    assert np.array_equal(d16.astype(np.float64), bf16_values(db))


def test_bf16_embedding_rows_are_dequantised_rows(uref):
    rng = np.random.default_rng(17)
    w = wl.gen_linear(rng, 40, 256, fmt="bf16")
    ids = np.array([3, 39, 0, 3, 17], dtype=np.int32)
    e = uref.w4_embedding(w["qweight"], w["scales"], w["zeros"], ids, fmt="bf16")
    z = w["zeros"].astype(np.int64)
    exact = (unpack_codes(w["qweight"]) - np.repeat(z, GROUP, axis=1)) * np.repeat(bf16_values(w["scales"]), GROUP, axis=1)
    assert np.array_equal(e, nearest_bf16_bits(exact)[ids])


def test_bf16_rope_is_the_fp64_rotation_of_the_decoded_inputs(uref):
    """Only the input format differs: the rotation itself is pinned in the RoPE pins."""
    rng = np.random.default_rng(19)
    spec = wl.RopeSpec(T=5, Hq=4, Hkv=2, H_tab=2, D_full=64, D_keep=40, theta=10000.0, pos_max=500)
    r = wl.gen_rope_inputs(rng, spec, fmt="bf16")
    q, k = uref.pruned_rope(r["q"], r["k"], r["positions"], r["kept_idx"], spec.D_full, spec.theta, fmt="bf16")
    q64 = uref.pruned_rope_f64(bf16_values(r["q"]), r["positions"], r["kept_idx"], spec.D_full, spec.theta)
    k64 = uref.pruned_rope_f64(bf16_values(r["k"]), r["positions"], r["kept_idx"], spec.D_full, spec.theta)
    assert np.array_equal(q, q64) and np.array_equal(k, k64)
    # position 0 leaves the decoded inputs unchanged
    pos0 = np.zeros(spec.T, dtype=np.int32)
    q0, _ = uref.pruned_rope(r["q"], None, pos0, r["kept_idx"], spec.D_full, spec.theta, fmt="bf16")
    assert np.array_equal(q0, bf16_values(r["q"]))


def test_generated_bf16_inputs_are_round_to_nearest(uref):
    """The input generator's float32 -> bfloat16 storage conversion agrees with the oracle's encoder."""
    rng = np.random.default_rng(23)
    a = (rng.standard_normal(3000) * 10.0 ** rng.integers(-6, 6, 3000)).astype(np.float32)
    a = np.concatenate([a, np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 0.0, -0.0], dtype=np.float32)])
    bits = wl.to_bf16_bits(a)
    assert np.array_equal(bits, np.array([uref.double_to_bf16(float(v)) for v in a], dtype=np.uint16))
    assert np.array_equal(wl.bf16_bits_to_f32(bits).astype(np.float64), bf16_values(bits))
