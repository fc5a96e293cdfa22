"""Pins for the CPU oracle's W4 dequant / linear (no GPU).

Each test ties the oracle to something other than itself: numpy's fp16
conversion, exact rational arithmetic on tiny inputs, closed forms, sub-matrix
invariants and numpy's fp64 matmul on an independently unpacked matrix.
"""
from fractions import Fraction

import numpy as np
import pytest

import workloads as wl
from workloads import Keep


# ---------------------------------------------------------------- fp16 codec
def test_half_decode_all_bit_patterns(uref):
    bits = np.arange(65536, dtype=np.uint16)
    mine = np.array([uref.half_to_double(int(b)) for b in bits])
    ref = bits.view(np.float16).astype(np.float64)
    assert np.array_equal(np.isnan(mine), np.isnan(ref))
    m = ~np.isnan(ref)
    assert np.array_equal(mine[m], ref[m])
    assert np.array_equal(np.signbit(mine[m]), np.signbit(ref[m]))


def test_half_encode_matches_numpy_rne(uref):
    rng = np.random.default_rng(1)
    vals = [0.0, -0.0, 1.0, -1.0, 65504.0, 65519.9, 65520.0, 1e6, -1e6, 2.0 ** -24, 2.0 ** -25,
            2.0 ** -25 * 1.0000001, 3 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25,
            1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -11 + 2.0 ** -30, 2047.5, 2048.5, 4094.0, 4095.0]
    # every midpoint between adjacent finite halfs of the positive normal/subnormal range (ties)
    h = np.arange(0, 0x7bff, 37, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    vals += list((lo + hi) / 2) + list(-(lo + hi) / 2)
    vals += list(rng.standard_normal(4000) * 10.0 ** rng.integers(-8, 5, 4000))
    with np.errstate(over="ignore"):
        ref = np.asarray(vals, dtype=np.float64).astype(np.float16).view(np.uint16)
    mine = np.array([uref.double_to_half(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(mine, ref)


# ------------------------------------------------------ independent unpacking
def unpack_numpy(qweight, scales, zeros, group=128):
    """Vectorised dequant written separately from the oracle: fp16 matrix [N][K]."""
    N, K8 = qweight.shape
    sh = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    q = ((qweight[:, :, None] >> sh) & np.uint32(15)).reshape(N, K8 * 8).astype(np.int64)
    z = np.repeat(zeros.astype(np.int64), group, axis=1)
    s = np.repeat(scales.astype(np.float64), group, axis=1)
    return ((q - z).astype(np.float64) * s).astype(np.float16)   # exact product, one RNE rounding


def kept_lists(N, K, keep: Keep):
    r = np.arange(N)
    k = np.arange(K)
    if keep.row_seg_stride:
        first = (r < keep.row_seg_limit) & (r % keep.row_seg_stride < keep.row_seg_keep)
        if keep.row_seg2_stride:
            second = ((r >= keep.row_seg_limit) & (r < keep.row_seg2_limit)
                      & ((r - keep.row_seg_limit) % keep.row_seg2_stride < keep.row_seg2_keep))
            rows = r[first | second | (r >= keep.row_seg2_limit)]
        else:
            rows = r[first | (r >= keep.row_seg_limit)]
    else:
        rows = r[: keep.n_keep or N]
    if keep.col_seg_stride:
        cols = k[k % keep.col_seg_stride < keep.col_seg_keep]
    else:
        cols = k[: keep.k_keep or K]
    return rows, cols


# ------------------------------------------------------ P5 exhaustive dequant
def test_dequant_exhaustive_q_z_scale(uref):
    """All 16x16 (q, z) pairs times every fp16 scale in (0.005, 0.02), plus
    subnormal / tiny / large scales: equals the exact product rounded once by numpy."""
    s_bits = np.arange(np.float16(0.005).view(np.uint16), np.float16(0.02).view(np.uint16) + 1, dtype=np.uint16)
    extra = np.array([0x0001, 0x0003, 0x03ff, 0x0400, 0x0401, 0x1400, 0x3c00, 0x3c01, 0x6bff, 0x7000, 0x8001, 0xbc00],
                     dtype=np.uint16)
    s_all = np.concatenate([s_bits, extra]).view(np.float16)
    G = 256                      # one row per scale; 256 columns = every (q, z)... z is per group
    # layout: group size 16 -> 16 groups per row, group g has zero g and nibbles 0..15
    N, K, group = s_all.size, 256, 16
    qweight = np.zeros((N, K // 8), dtype=np.uint32)
    word_lo = sum(j << (4 * j) for j in range(8))
    word_hi = sum((8 + j) << (4 * j) for j in range(8))
    qweight[:, 0::2] = word_lo
    qweight[:, 1::2] = word_hi
    zeros = np.tile(np.arange(16, dtype=np.uint8), (N, 1))
    scales = np.repeat(s_all[:, None], 16, axis=1).copy()
    got = uref.w4_dequant(qweight, scales, zeros, group=group)
    q = np.tile(np.arange(16), 16)[None, :]
    z = np.repeat(np.arange(16), 16)[None, :]
    with np.errstate(over="ignore"):
        exp = ((q - z).astype(np.float64) * s_all.astype(np.float64)[:, None]).astype(np.float16)
    assert got.shape == (N, G)
    assert np.array_equal(got.view(np.uint16), exp.view(np.uint16))


# ------------------------------------------------------------- P6 brute force
@pytest.mark.parametrize("N,K,group,M", [(8, 8, 8, 1), (8, 128, 128, 2), (16, 256, 128, 3)])
def test_linear_brute_force_fractions(uref, N, K, group, M):
    rng = np.random.default_rng(100 + K)
    nib = rng.integers(0, 16, size=(N, K))
    qweight = np.zeros((N, K // 8), dtype=np.uint32)
    for r in range(N):
        for k in range(K):
            qweight[r, k // 8] |= np.uint32(int(nib[r, k]) << (4 * (k % 8)))
    scales = rng.uniform(0.005, 0.02, size=(N, K // group)).astype(np.float16)
    zeros = rng.integers(0, 16, size=(N, K // group), dtype=np.uint8)
    x = wl.gen_activations(rng, M, K)
    y = uref.w4_linear(qweight, scales, zeros, x, group=group)
    wd = uref.w4_dequant(qweight, scales, zeros, group=group)
    for r in range(N):
        wrow = []
        for k in range(K):
            exact = (int(nib[r, k]) - int(zeros[r, k // group])) * Fraction(float(scales[r, k // group]))
            w16 = np.float16(float(exact))          # exact in fp64, then one RNE rounding
            assert wd[r, k].view(np.uint16) == w16.view(np.uint16)
            wrow.append(Fraction(float(w16)))
        for m in range(M):
            exact = sum(Fraction(float(x[m, k])) * wrow[k] for k in range(K))
            assert abs(float(exact) - y[m, r]) <= 1e-13 * max(1.0, abs(float(exact)))


# ---------------------------------------------------- P7 numpy matmul, pruned
KEEPS = [
    Keep(),
    Keep(n_keep=870),
    Keep(k_keep=870),                                           # not a multiple of 8: nibble-granular tail
    Keep(n_keep=333, k_keep=517),
    Keep(n_keep=16 * 54, row_seg_stride=64, row_seg_keep=54),    # q/k style: half-head segments... stride 64
    Keep(k_keep=8 * 108, col_seg_stride=128, col_seg_keep=108),  # o_proj style
    Keep(n_keep=2 * 300 + 224, row_seg_stride=400, row_seg_keep=300, row_seg_limit=800),   # in_proj style + tail
    Keep(n_keep=8 * 82, k_keep=16 * 41, row_seg_stride=128, row_seg_keep=82, col_seg_stride=64, col_seg_keep=41),
    # Mamba in_proj with head and state dimension pruned: z | x heads of 64 keep 54, B | C groups of 128 keep 109, dt whole
    Keep(n_keep=10 * 54 + 2 * 109 + 128, row_seg_stride=64, row_seg_keep=54, row_seg_limit=640,
         row_seg2_stride=128, row_seg2_keep=109, row_seg2_limit=896),
    # second family running to the last row (no whole-kept tail), first family one segment
    Keep(n_keep=500 + 4 * 100, row_seg_stride=512, row_seg_keep=500, row_seg_limit=512,
         row_seg2_stride=128, row_seg2_keep=100, row_seg2_limit=1024),
]


@pytest.mark.parametrize("keep", KEEPS)
def test_linear_matches_numpy_matmul(uref, keep):
    N = K = 1024
    rng = wl.rng_for(0, stream=7)
    w = wl.gen_linear(rng, N, K)
    rows, cols = kept_lists(N, K, keep)
    assert uref.count_kept(N, K, keep) == (rows.size, cols.size)
    x = wl.gen_activations(rng, 3, cols.size)
    Wd = unpack_numpy(**w)
    got_w = uref.w4_dequant(w["qweight"], w["scales"], w["zeros"], keep)
    assert np.array_equal(got_w.view(np.uint16), Wd[np.ix_(rows, cols)].view(np.uint16))
    y = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    ref = x.astype(np.float64) @ Wd[np.ix_(rows, cols)].astype(np.float64).T
    assert y.shape == ref.shape
    assert np.max(np.abs(y - ref)) <= 1e-11


def test_mamba_in_proj_rows_by_part(uref):
    """The head- and state-pruned in_proj keeps, part by part, what Alg. 5 / Alg. 4 and Sec. 3.4 say: the
    leading channels of every head of z and of x, the leading state channels of the group in B and in C,
    every step-size row -- written here as explicit slices of the full output, not through the rule."""
    spec = wl.mamba2_2p7b_layer_heads_and_state(15)[0]
    H, D, Ds = 80, 64, 128
    Dk, Sk = wl.kept_head_dim(D, 15), wl.kept_dim(Ds, 15)
    assert (Dk, Sk) == (54, 108) and spec.N == 2 * H * D + 2 * Ds + H
    rng = wl.rng_for(3, 77)
    # a narrow stand-in for the 2560 input columns keeps the test fast; the rows are the real ones
    w = wl.gen_linear(rng, spec.N, 256)
    x = wl.gen_activations(rng, 1, 256)
    full = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, None)[0]
    y = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, spec.keep)[0]
    z_part = full[: H * D].reshape(H, D)[:, :Dk].reshape(-1)
    x_part = full[H * D: 2 * H * D].reshape(H, D)[:, :Dk].reshape(-1)
    b_part = full[2 * H * D: 2 * H * D + Ds][:Sk]
    c_part = full[2 * H * D + Ds: 2 * H * D + 2 * Ds][:Sk]
    dt_part = full[2 * H * D + 2 * Ds:]
    assert np.array_equal(y, np.concatenate([z_part, x_part, b_part, c_part, dt_part]))
    assert y.size == spec.n_keep


# ------------------------------------------------------ P1 / P2 invariants
def test_keep_full_is_unpruned_bit_identical(uref):
    rng = wl.rng_for(0, stream=8)
    w = wl.gen_linear(rng, 256, 512)
    x = wl.gen_activations(rng, 2, 512)
    y0 = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, None)
    y1 = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, Keep(n_keep=256, k_keep=512))
    y2 = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x,
                        Keep(n_keep=256, k_keep=512, row_seg_stride=64, row_seg_keep=64, row_seg_limit=256,
                             col_seg_stride=128, col_seg_keep=128))
    assert np.array_equal(y0, y1) and np.array_equal(y0, y2)


def test_truncation_is_submatrix_selection(uref):
    rng = wl.rng_for(0, stream=9)
    N, K = 384, 640
    w = wl.gen_linear(rng, N, K)
    x = wl.gen_activations(rng, 2, K)
    full = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, None)
    # rows: compact output r' is exactly the full output at the stored row
    keep = Keep(n_keep=3 * 100 + 84, row_seg_stride=100, row_seg_keep=100 - 0, row_seg_limit=300)
    keep = Keep(n_keep=3 * 61 + 84, row_seg_stride=100, row_seg_keep=61, row_seg_limit=300)
    rows, _ = kept_lists(N, K, keep)
    y = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    assert np.array_equal(y, full[:, rows])
    # cols: dropping columns == zeroing the matching inputs of the full layer
    for keep in (Keep(k_keep=333), Keep(k_keep=5 * 77, col_seg_stride=128, col_seg_keep=77)):
        _, cols = kept_lists(N, K, keep)
        xz = np.zeros_like(x)
        xz[:, cols] = x[:, cols]
        y = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], np.ascontiguousarray(x[:, cols]), keep)
        yz = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], xz, None)
        assert np.max(np.abs(y - yz)) <= 1e-12   # zeros add exactly; only the order of exact-zero terms differs


def test_sampled_rows_equal_full_rows(uref):
    rng = wl.rng_for(0, stream=10)
    w = wl.gen_linear(rng, 200, 256)
    x = wl.gen_activations(rng, 2, 256)
    keep = Keep(n_keep=150)
    full = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    rows = [0, 149, 7, 7, 64]
    part = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep, rows=rows)
    assert np.array_equal(part, full[:, rows])


# ------------------------------------------------------------ P4 closed forms
def test_constant_matrix_closed_form(uref):
    N, K = 32, 512
    for c, z, s in [(11, 3, 0.0123), (0, 15, 0.02), (8, 8, 0.005), (15, 0, 0.0077)]:
        word = sum(c << (4 * j) for j in range(8))
        qweight = np.full((N, K // 8), word, dtype=np.uint32)
        scales = np.full((N, K // 128), s, dtype=np.float16)
        zeros = np.full((N, K // 128), z, dtype=np.uint8)
        x = np.ones((1, 300), dtype=np.float16)
        y = uref.w4_linear(qweight, scales, zeros, x, Keep(k_keep=300))
        w16 = float(np.float16((c - z) * float(scales[0, 0])))
        assert np.array_equal(y, np.full((1, N), 300 * w16))


def test_one_hot_input_reads_dequantised_column(uref):
    rng = wl.rng_for(0, stream=11)
    N, K = 64, 256
    w = wl.gen_linear(rng, N, K)
    Wd = uref.w4_dequant(w["qweight"], w["scales"], w["zeros"])
    for k in (0, 1, 7, 8, 127, 128, 255):
        x = np.zeros((1, K), dtype=np.float16)
        x[0, k] = 1.0
        y = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x)
        assert np.array_equal(y[0], Wd[:, k].astype(np.float64))


def test_nibble_order_and_group_boundaries(uref):
    """A single non-zero nibble lands in exactly one column; scale/zero switch at multiples of the group."""
    N, K = 1, 256
    scales = np.array([[0.01, 0.02]], dtype=np.float16)
    zeros = np.array([[0, 5]], dtype=np.uint8)
    for k in (0, 3, 7, 8, 127, 128, 200):
        qweight = np.zeros((N, K // 8), dtype=np.uint32)
        qweight[0, k // 8] = np.uint32(9 << (4 * (k % 8)))
        Wd = uref.w4_dequant(qweight, scales, zeros).astype(np.float64)[0]
        exp = np.zeros(K)
        exp[128:] = float(np.float16(-5 * float(scales[0, 1])))
        exp[k] = float(np.float16((9 - int(zeros[0, k // 128])) * float(scales[0, k // 128])))
        assert np.array_equal(Wd, exp)


# ---------------------------------------------------------- P3 quantiser pins
def test_symmetric_quantiser_round_trip(uref):
    """Values on the symmetric 4-bit grid (|q| <= 7 with 7 attained) survive quantise -> dequantise exactly."""
    rng = np.random.default_rng(5)
    N, K = 16, 512
    q = rng.integers(-7, 8, size=(N, K))
    q[:, ::128] = 7 * rng.choice([-1, 1], size=(N, K // 128))       # every group attains the maximum
    s = rng.uniform(0.005, 0.02, size=(N, K // 128)).astype(np.float16)
    w = q * np.repeat(s.astype(np.float64), 128, axis=1)
    qw, sc, zr = uref.quantize_sym(w)
    assert np.array_equal(sc.view(np.uint16), s.view(np.uint16)) and np.all(zr == 8)
    # the stored code is q + 8, read back with the independent unpacker
    sh = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    codes = ((qw[:, :, None] >> sh) & np.uint32(15)).reshape(N, K).astype(np.int64)
    assert np.array_equal(codes - 8, q)
    wd = uref.w4_dequant(qw, sc, zr).astype(np.float64)
    assert np.array_equal(wd, w.astype(np.float16).astype(np.float64))
    # re-quantising the fp16-rounded weights keeps every code (the scale may move by one fp16 ulp,
    # because 7 * s is itself rounded to fp16 on the way)
    qw2, sc2, zr2 = uref.quantize_sym(wd)
    assert np.array_equal(qw2, qw)
    assert np.max(np.abs(sc2.view(np.uint16).astype(int) - sc.view(np.uint16).astype(int))) <= 1


def test_symmetric_quantiser_equation(uref):
    """Eq. 3 itself on random data: clamp(round(W / s)) with s = max|W| / 7, codes within [-8, 7]."""
    rng = np.random.default_rng(6)
    w = rng.standard_normal((4, 256))
    qw, sc, zr = uref.quantize_sym(w)
    s = sc.astype(np.float64)
    mx = np.abs(w.reshape(4, 2, 128)).max(axis=2)
    assert np.array_equal(sc.view(np.uint16), (mx / 7.0).astype(np.float16).view(np.uint16))
    sh = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    codes = ((qw[:, :, None] >> sh) & np.uint32(15)).reshape(4, 256).astype(np.int64) - 8
    exp = np.clip(np.rint(w / np.repeat(s, 128, axis=1)), -8, 7)
    assert np.array_equal(codes, exp)
    err = np.abs(uref.w4_dequant(qw, sc, zr).astype(np.float64) - w)
    assert np.all(err <= 0.5 * np.repeat(s, 128, axis=1) * 1.01 + 1e-3 * np.abs(w))


def test_asymmetric_quantiser_round_trip(uref):
    rng = np.random.default_rng(7)
    N, K = 8, 256
    q = rng.integers(0, 16, size=(N, K))
    q[:, 0::128] = 0
    q[:, 1::128] = 15                                     # full range attained in every group
    z = rng.integers(0, 16, size=(N, K // 128))
    s = rng.uniform(0.005, 0.02, size=(N, K // 128)).astype(np.float16)
    w = (q - np.repeat(z, 128, axis=1)) * np.repeat(s.astype(np.float64), 128, axis=1)
    qw, sc, zr = uref.quantize_asym(w)
    assert np.array_equal(sc.view(np.uint16), s.view(np.uint16))
    assert np.array_equal(zr, z.astype(np.uint8))
    wd = uref.w4_dequant(qw, sc, zr)
    assert np.array_equal(wd.view(np.uint16), w.astype(np.float16).view(np.uint16))


def test_symmetric_is_the_zero_8_case(uref):
    """The asymmetric format with zero = 8 reproduces signed symmetric codes."""
    rng = np.random.default_rng(8)
    w = wl.gen_linear(rng, 8, 128, sym_zero=True)
    Wd = uref.w4_dequant(w["qweight"], w["scales"], w["zeros"]).astype(np.float64)
    sh = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    signed = ((w["qweight"][:, :, None] >> sh) & np.uint32(15)).reshape(8, 128).astype(np.int64) - 8
    assert signed.min() >= -8 and signed.max() <= 7
    exp = (signed * w["scales"].astype(np.float64)).astype(np.float16).astype(np.float64)
    assert np.array_equal(Wd, exp)


def test_no_zero_points_is_the_signed_code_scheme_of_eq3(uref):
    """zeros = None: the stored nibble is Eq. 3's signed code + 8, so the weight is (nibble - 8) * s.
    Checked against the signed codes read back by numpy -- for random nibbles, for the output of the
    symmetric quantiser, and through the linear (numpy matmul on the dense signed matrix), the
    embedding gather and the repack."""
    rng = np.random.default_rng(81)
    N, K = 24, 384
    w = wl.gen_linear(rng, N, K)
    sh = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    signed = ((w["qweight"][:, :, None] >> sh) & np.uint32(15)).reshape(N, K).astype(np.int64) - 8
    s = np.repeat(w["scales"].astype(np.float64), 128, axis=1)
    dense = (signed * s).astype(np.float16)
    got = uref.w4_dequant(w["qweight"], w["scales"], None)
    assert np.array_equal(got.view(np.uint16), dense.view(np.uint16))
    # a stored zero-point array is ignored only when it is absent: random zeros give something else
    assert not np.array_equal(uref.w4_dequant(w["qweight"], w["scales"], w["zeros"]).view(np.uint16), dense.view(np.uint16))
    keep = Keep(n_keep=17, k_keep=300)
    x = wl.gen_activations(rng, 2, 300)
    y = uref.w4_linear(w["qweight"], w["scales"], None, x, keep)
    ref = x.astype(np.float64) @ dense.astype(np.float64)[:17, :300].T
    assert np.allclose(y, ref, rtol=1e-12, atol=1e-12)
    ids = np.array([5, 0, 23], dtype=np.int32)
    assert np.array_equal(uref.w4_embedding(w["qweight"], w["scales"], None, ids).view(np.uint16), dense[ids].view(np.uint16))
    q2, s2, z2, keep2 = uref.w4_repack(w["qweight"], w["scales"], None, keep)
    assert z2 is None
    assert np.array_equal(uref.w4_dequant(q2, s2, None, Keep(*keep2)).view(np.uint16), dense[:17, :300].view(np.uint16))
    # Eq. 3 end to end: quantise real weights, drop the (all 8) zero points, dequantise
    wf = rng.standard_normal((4, 256))
    qw, sc, zr = uref.quantize_sym(wf)
    exp = (np.clip(np.rint(wf / np.repeat(sc.astype(np.float64), 128, axis=1)), -8, 7)
           * np.repeat(sc.astype(np.float64), 128, axis=1)).astype(np.float16)
    # by value: numpy's rint keeps the sign of a zero, an integer code has none
    assert np.array_equal(uref.w4_dequant(qw, sc, None).astype(np.float64), exp.astype(np.float64))


def test_gate_up_silu_is_numpy_matmul_then_silu(uref):
    """h = SiLU(x Wg) * (x Wu) (Eq. 1) against an independently unpacked dense weight, numpy matmul and
    the textbook SiLU written with tanh: x * (1 + tanh(x / 2)) / 2."""
    rng = wl.rng_for(0, 24)
    N, K, T = 96, 256, 3
    keep = wl.Keep(n_keep=81)
    wg, wu = wl.gen_linear(rng, N, K), wl.gen_linear(rng, N, K)
    x = wl.gen_activations(rng, T, K)
    h = uref.gate_up_silu(wg, keep, wu, keep, x)

    def dense(w):
        qw = w["qweight"]
        nib = np.stack([(qw >> np.uint32(4 * j)) & np.uint32(15) for j in range(8)], axis=-1).reshape(qw.shape[0], -1)
        s = np.repeat(w["scales"].astype(np.float64), 128, axis=1)
        z = np.repeat(w["zeros"].astype(np.float64), 128, axis=1)
        return ((nib.astype(np.float64) - z) * s).astype(np.float16).astype(np.float64)

    xf = x.astype(np.float64)
    g, u = (xf @ dense(wg).T)[:, :81], (xf @ dense(wu).T)[:, :81]
    ref = g * (1.0 + np.tanh(g / 2.0)) / 2.0 * u
    assert h.shape == (T, 81)
    assert np.max(np.abs(h - ref)) < 1e-9 * max(1.0, np.max(np.abs(ref)))
    # the gate closes for very negative pre-activations and passes very positive ones unchanged
    big = np.array([[-60.0, 60.0]])
    assert np.allclose(big / (1.0 + np.exp(-big)), [[0.0, 60.0]], atol=1e-20, rtol=1e-15)


def test_embedding_gather_is_row_selection_of_an_independent_unpack(uref):
    """Gathered rows against a numpy unpack of the whole table (nibble j of word w = column 8w + j) rounded
    to fp16 by numpy; repeated and out-of-order ids; and as a one-hot product: row id = e_id^T W."""
    rng = wl.rng_for(0, 25)
    N, K = 50, 384
    w = wl.gen_linear(rng, N, K)
    ids = np.array([7, 0, 49, 7, 13], dtype=np.int32)
    got = uref.w4_embedding(w["qweight"], w["scales"], w["zeros"], ids)
    qw = w["qweight"]
    nib = np.stack([(qw >> np.uint32(4 * j)) & np.uint32(15) for j in range(8)], axis=-1).reshape(N, K)
    s = np.repeat(w["scales"].astype(np.float64), 128, axis=1)
    z = np.repeat(w["zeros"].astype(np.float64), 128, axis=1)
    dense = ((nib.astype(np.float64) - z) * s).astype(np.float16)
    assert got.shape == (5, K)
    assert np.array_equal(got.view(np.uint16), dense[ids].view(np.uint16))
    # the transposed table as a linear: a one-hot "activation" over rows is not expressible (rows are
    # outputs), so check through columns instead: x = e_k picks column k of every row, row by row
    for k in (0, 127, 128, 383):
        x = np.zeros((1, K), dtype=np.float16); x[0, k] = 1.0
        col = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x)[0]
        assert np.array_equal(col[ids], got[:, k].astype(np.float64))
