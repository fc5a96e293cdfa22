"""Pins of the oracle's head-interleaved storage order (uref_w4_interleave, the il_heads argument of
uref_w4_linear_il / uref_w4_dequant_il): a second storage order of the same matrix, so everything is pinned to the
plain order -- the permutation against numpy, the results against the oracle's own plain-order functions (which
carry their own pins), and a brute-force case against exact rationals."""
from fractions import Fraction

import numpy as np
import pytest

import oracle as uref
import workloads as wl
from workloads import Keep


def _half_frac(bits: int) -> Fraction:
    """Exact value of a finite binary16 bit pattern."""
    s, e, m = bits >> 15, (bits >> 10) & 31, bits & 1023
    v = Fraction(m, 1 << 24) if e == 0 else Fraction(1024 + m, 1 << 10) * Fraction(2) ** (e - 15)
    return -v if s else v


@pytest.mark.parametrize("N,K,heads", [(3, 256, 2), (5, 512, 4), (2, 4096, 32), (4, 768, 3), (2, 1024, 4)])
def test_interleave_is_the_word_transpose(N, K, heads):
    rng = wl.rng_for(18, N + K + heads)
    q = rng.integers(0, 2 ** 32, (N, K // 8), dtype=np.uint64).astype(np.uint32)
    got = uref.w4_interleave(q, heads)
    want = q.reshape(N, heads, K // 8 // heads).transpose(0, 2, 1).reshape(N, K // 8)
    assert np.array_equal(got, want)
    # word (d / 8) * heads + h of the result is word h * (D / 8) + d / 8 of the source, spelled out for one entry
    D8 = K // 8 // heads
    h, b = heads - 1, D8 - 1
    assert got[N - 1, b * heads + h] == q[N - 1, h * D8 + b]


@pytest.mark.parametrize("keep", [Keep(), Keep(col_seg_stride=128, col_seg_keep=108), Keep(col_seg_stride=128, col_seg_keep=82),
                                  Keep(n_keep=5, col_seg_stride=128, col_seg_keep=8), Keep(k_keep=300),
                                  Keep(col_seg_stride=256, col_seg_keep=131)])
@pytest.mark.parametrize("heads", [2, 4])
def test_interleaved_matrix_gives_the_plain_results_exactly(keep, heads):
    """The same sums over the same columns in the same order: the fp64 outputs and the dequantised weights of the
    interleaved matrix equal those of the plain one bit for bit, for column rules of every kind."""
    rng = wl.rng_for(18, heads)
    N, K = 7, 512
    w = wl.gen_linear(rng, N, K)
    qi = uref.w4_interleave(w["qweight"], heads)
    assert not np.array_equal(qi, w["qweight"])
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, 3, kk)
    y_plain = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    y_il = uref.w4_linear(qi, w["scales"], w["zeros"], x, keep, il_heads=heads)
    assert np.array_equal(y_plain.view(np.uint64), y_il.view(np.uint64))
    d_plain = uref.w4_dequant(w["qweight"], w["scales"], w["zeros"], keep)
    d_il = uref.w4_dequant(qi, w["scales"], w["zeros"], keep, il_heads=heads)
    assert np.array_equal(d_plain.view(np.uint16), d_il.view(np.uint16))
    # reading the interleaved words as if they were in plain order is a different matrix (the argument matters)
    assert not np.array_equal(uref.w4_dequant(qi, w["scales"], w["zeros"], keep).view(np.uint16), d_plain.view(np.uint16))


def test_interleaved_linear_brute_force_rationals():
    """2 heads of 128 dims, the leading 9 dims of each kept: the sum written out over (head, dim) with the word and
    nibble of every code located by hand, in exact rationals."""
    rng = wl.rng_for(18, 99)
    N, K, H, Dk = 4, 256, 2, 9
    w = wl.gen_linear(rng, N, K)
    qi = uref.w4_interleave(w["qweight"], H)
    keep = Keep(col_seg_stride=128, col_seg_keep=Dk)
    x = wl.gen_activations(rng, 1, H * Dk)
    y = uref.w4_linear(qi, w["scales"], w["zeros"], x, keep, il_heads=H)
    xb = x.view(np.uint16)
    for r in range(N):
        acc = Fraction(0)
        for h in range(H):
            s = _half_frac(int(w["scales"].view(np.uint16)[r, h]))     # a head is one group of 128
            z = int(w["zeros"][r, h])
            for d in range(Dk):
                word = int(qi[r, (d // 8) * H + h])
                q = (word >> (4 * (d % 8))) & 15
                wt = _half_frac(int(np.float16(float((q - z) * s)).view(np.uint16)))   # numpy's nearest-even rounding
                acc += _half_frac(int(xb[0, h * Dk + d])) * wt
        assert abs(float(acc) - y[0, r]) <= 1e-12 * max(1.0, abs(float(acc)))


def test_interleave_argument_checks():
    q = np.zeros((2, 32), dtype=np.uint32)                 # K = 256
    with pytest.raises(AssertionError):
        uref.w4_interleave(q, 3)                           # 256 is not a multiple of 3
    with pytest.raises(AssertionError):
        uref.w4_interleave(q, 64)                          # heads of 4 dims: not whole words


@pytest.mark.parametrize("N,K,heads", [(3, 256, 2), (5, 512, 4), (2, 4096, 32), (4, 768, 3)])
def test_deinterleave_is_the_inverse_word_transpose(N, K, heads):
    """uref_w4_deinterleave against numpy's transpose of the [words per head][heads] view, against the round trip through
    uref_w4_interleave in both orders, and spelled out for one entry."""
    rng = wl.rng_for(18, 7 * N + K + heads)
    q = rng.integers(0, 2 ** 32, (N, K // 8), dtype=np.uint64).astype(np.uint32)
    D8 = K // 8 // heads
    got = uref.w4_deinterleave(q, heads)
    want = q.reshape(N, D8, heads).transpose(0, 2, 1).reshape(N, K // 8)
    assert np.array_equal(got, want)
    assert np.array_equal(uref.w4_deinterleave(uref.w4_interleave(q, heads), heads), q)
    assert np.array_equal(uref.w4_interleave(uref.w4_deinterleave(q, heads), heads), q)
    h, b = heads - 1, D8 - 2 if D8 > 1 else 0
    assert got[N - 1, h * D8 + b] == q[N - 1, b * heads + h]


def test_deinterleaved_matrix_is_the_plain_matrix():
    """Reading the deinterleaved words in plain order gives the weights and the sums of the interleaved matrix read
    with its head count, bit for bit (pruned heads included)."""
    rng = wl.rng_for(18, 99)
    N, K, heads = 6, 512, 4
    keep = Keep(col_seg_stride=128, col_seg_keep=101)
    w = wl.gen_linear(rng, N, K)
    qi = rng.integers(0, 2 ** 32, (N, K // 8), dtype=np.uint64).astype(np.uint32)   # any words: an interleaved matrix
    qp = uref.w4_deinterleave(qi, heads)
    d_il = uref.w4_dequant(qi, w["scales"], w["zeros"], keep, il_heads=heads)
    d_pl = uref.w4_dequant(qp, w["scales"], w["zeros"], keep)
    assert np.array_equal(d_il.view(np.uint16), d_pl.view(np.uint16))
    x = wl.gen_activations(rng, 2, heads * 101)
    y_il = uref.w4_linear(qi, w["scales"], w["zeros"], x, keep, il_heads=heads)
    y_pl = uref.w4_linear(qp, w["scales"], w["zeros"], x, keep)
    assert np.array_equal(y_il.view(np.uint64), y_pl.view(np.uint64))
    with pytest.raises(ValueError):
        uref.w4_deinterleave(qi, 3)                          # 512 is not a multiple of 3
