"""GPU parity of the codes of 3 and 6 bits (Eq. 3 with N = 3, 6; row-wise bit stream) through the C ABI against the CPU
oracle: the dequantised matrix bit for bit, the linear within the element-wise bar of the 4-bit linears, in fp16 and
bfloat16."""
import numpy as np
import pytest

import workloads as wl
from workloads import Keep
from parity_util import NORM_TOL, NORM_TOL_BF16, TOL, TOL_BF16, linear_err, normwise_err

pytestmark = pytest.mark.gpu

WIDTHS = (3, 6)


@pytest.fixture(scope="module")
def env(uref):
    import torch
    import paper_2512_03383_amd as uq
    assert torch.cuda.is_available(), "gpu tests need an MI355X"
    uq.lib()
    uref.set_threads(min(16, uref.max_threads()))
    return uq, torch


def to_dev16(torch, a, fmt):
    if fmt == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host_bits(torch, t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_vals(t):
    return t.float().cpu().numpy().astype(np.float64)


def gen(rng, N, K, bits, fmt, sym=False):
    w = wl.gen_linear_bits(rng, N, K, bits, fmt=fmt)
    if sym:
        w["zeros"] = None
    return w


KEEPS = [
    Keep(),
    Keep(n_keep=870, k_keep=517),
    Keep(n_keep=1, k_keep=1),
    Keep(n_keep=33, k_keep=1000),
    Keep(n_keep=16 * 54, row_seg_stride=64, row_seg_keep=54, row_seg_limit=1024),
    Keep(k_keep=8 * 108, col_seg_stride=128, col_seg_keep=108),
    Keep(n_keep=8 * 82, k_keep=16 * 41, row_seg_stride=128, row_seg_keep=82, row_seg_limit=1024,
         col_seg_stride=64, col_seg_keep=41),
    Keep(n_keep=10 * 54 + 2 * 109 + 128, row_seg_stride=64, row_seg_keep=54, row_seg_limit=640,
         row_seg2_stride=128, row_seg2_keep=109, row_seg2_limit=896),
]


@pytest.mark.parametrize("bits", WIDTHS)
@pytest.mark.parametrize("fmt", ["f16", "bf16"])
@pytest.mark.parametrize("sym", [False, True])
@pytest.mark.parametrize("keep", KEEPS)
def test_dequant_bit_exact(env, uref, keep, sym, fmt, bits):
    uq, torch = env
    w = gen(wl.rng_for(36, bits), 1024, 1024, bits, fmt, sym)
    ref = uref.wq_dequant(bits, w["qweight"], w["scales"], w["zeros"], keep, fmt=fmt)
    got = uq.uniql_w4_dequant(uq.QuantLinear.from_numpy(w, bits=bits), keep)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(torch, got), ref.view(np.uint16))


@pytest.mark.parametrize("bits", WIDTHS)
@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_dequant_every_code_zero_point_and_alignment(env, uref, fmt, bits):
    """Row (z, shift) holds code (k + shift) mod 2^bits at column k under zero point z -- every code at every bit
    alignment of the stream -- with scales that produce subnormal, tie and large results.  The random words of the
    other tests only meet these by chance."""
    uq, torch = env
    L = 1 << bits
    shifts = (0, 1, 3, 5)
    K = 1024
    codes = np.stack([(np.arange(K) + sh) % L for _ in range(L) for sh in shifts]).astype(np.uint64)
    N = codes.shape[0]
    # the row's stream, written with 64-bit integers: code k contributes to word (bits k) / 32 and maybe the next one
    qweight = np.zeros((N, K * bits // 32 + 1), dtype=np.uint64)
    for k in range(K):
        pos = bits * k
        v = codes[:, k] << np.uint64(pos % 32)
        qweight[:, pos // 32] |= v & np.uint64(0xFFFFFFFF)
        qweight[:, pos // 32 + 1] |= v >> np.uint64(32)
    qweight = np.ascontiguousarray(qweight[:, :-1].astype(np.uint32))
    zeros = np.repeat(np.repeat(np.arange(L, dtype=np.uint8), len(shifts))[:, None], 8, axis=1)
    sb = np.array([0x2000, 0x211f, 0x2400, 0x1c01, 0x0003, 0x3555, 0x5000, 0x0400], dtype=np.uint16)
    if fmt == "bf16":
        sb = np.array([0x3a00, 0x3a13, 0x3b80, 0x0081, 0x0003, 0x3eab, 0x4700, 0x0080], dtype=np.uint16)
    scales = np.tile(sb, (N, 1))
    scales = scales.view(np.float16) if fmt == "f16" else scales
    w = {"qweight": qweight, "scales": np.ascontiguousarray(scales), "zeros": zeros}
    ref = uref.wq_dequant(bits, w["qweight"], w["scales"], w["zeros"], fmt=fmt)
    got = uq.uniql_w4_dequant(uq.QuantLinear.from_numpy(w, bits=bits), None)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(torch, got), ref.view(np.uint16))
    # the linear on one-hot activations returns single weights: the kernel's own unpack (merged half-words, funnel
    # shifts) at every position of a unit, bit for bit in fp16 (one product, exact in fp32, rounded once at the output)
    if fmt == "f16":
        qw = uq.QuantLinear.from_numpy(w, bits=bits)
        for k0 in (0, 97, 130):
            x = np.zeros((1, K), dtype=np.float16)
            x[0, k0:k0 + 1] = 1.0
            y = uq.uniql_w4_linear(qw, None, to_dev16(torch, x, fmt))
            torch.cuda.synchronize()
            assert np.array_equal(host_bits(torch, y)[0], ref.view(np.uint16)[:, k0]), (bits, k0)


@pytest.mark.parametrize("bits", WIDTHS)
def test_linear_one_hot_every_column_of_two_units(env, uref, bits):
    """One-hot activations at each of the first 64 columns and the last 32: every pair position of the kernel's unpack
    (including the codes that run over word and half-word boundaries) returns the canonical weight bit for bit."""
    uq, torch = env
    rng = wl.rng_for(36, 100 + bits)
    N, K = 64, 512
    w = gen(rng, N, K, bits, "f16")
    qw = uq.QuantLinear.from_numpy(w, bits=bits)
    ref = uref.wq_dequant(bits, w["qweight"], w["scales"], w["zeros"])
    cols = list(range(64)) + list(range(K - 32, K))
    x = np.zeros((len(cols), K), dtype=np.float16)
    for i, k in enumerate(cols):
        x[i, k] = 1.0
    y = uq.uniql_w4_linear(qw, None, to_dev16(torch, x, "f16"))
    torch.cuda.synchronize()
    got = host_bits(torch, y)
    for i, k in enumerate(cols):
        assert np.array_equal(got[i], ref.view(np.uint16)[:, k]), (bits, k)


@pytest.mark.parametrize("bits", WIDTHS)
@pytest.mark.parametrize("fmt", ["f16", "bf16"])
@pytest.mark.parametrize("M", [1, 2, 5, 16])
@pytest.mark.parametrize("keep", KEEPS)
def test_linear_parity_1024(env, uref, keep, M, fmt, bits):
    uq, torch = env
    rng = wl.rng_for(36, 2 + bits)
    w = gen(rng, 1024, 1024, bits, fmt, sym=(M == 5))
    qw = uq.QuantLinear.from_numpy(w, bits=bits)
    nk, kk = uq.kept_dims(qw, keep)
    x = wl.gen_activations(rng, M, kk, fmt=fmt)
    ref = uref.wq_linear(bits, w["qweight"], w["scales"], w["zeros"], x, keep, fmt=fmt)
    pad = 3 if M in (1, 5) else 0
    tdt = torch.bfloat16 if fmt == "bf16" else torch.float16
    xb = torch.full((M, kk + pad), 77.0, dtype=tdt, device="cuda")
    xb[:, :kk] = to_dev16(torch, x, fmt)
    yb = torch.full((M, nk + pad), -5.0, dtype=tdt, device="cuda")
    uq.uniql_w4_linear(qw, keep, xb[:, :kk], yb[:, :nk])
    torch.cuda.synchronize()
    assert torch.all(yb[:, nk:] == -5.0), "wrote past n_keep"
    y = host_vals(yb[:, :nk])
    assert linear_err(y, ref) <= (TOL_BF16 if fmt == "bf16" else TOL)
    if nk >= 64:
        assert normwise_err(y, ref) <= (NORM_TOL_BF16 if fmt == "bf16" else NORM_TOL)


@pytest.mark.parametrize("bits", WIDTHS)
@pytest.mark.parametrize("N,K,keep", [
    (14336, 4096, Keep(n_keep=12185)),          # Llama-3-8B gate / up at 15 %
    (4096, 14336, Keep(k_keep=12185)),          # down: the last unit partly kept, several steps per row
    (300, 32768, Keep()),                       # the longest row the staging holds
    (7, 128, Keep()),                           # one group, fewer rows than a block has waves
    (5000, 256, Keep(n_keep=4097)),             # more rows than one round of the grid's waves
])
def test_linear_model_shapes(env, uref, N, K, keep, bits):
    uq, torch = env
    rng = wl.rng_for(36, N + K + bits)
    w = gen(rng, N, K, bits, "f16")
    qw = uq.QuantLinear.from_numpy(w, bits=bits)
    nk, kk = uq.kept_dims(qw, keep)
    x = wl.gen_activations(rng, 1, kk)
    rows = np.unique(np.concatenate([[0, 1, nk - 2, nk - 1], rng.integers(0, nk, 128)])).astype(np.int32)
    rows = rows[(rows >= 0) & (rows < nk)]
    ref = uref.wq_linear(bits, w["qweight"], w["scales"], w["zeros"], x, keep, rows=rows)
    y = uq.uniql_w4_linear(qw, keep, to_dev16(torch, x, "f16"))
    y2 = uq.uniql_w4_linear(qw, keep, to_dev16(torch, x, "f16"))
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    got = host_vals(y)[:, rows]
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms)) <= TOL


@pytest.mark.parametrize("bits", WIDTHS)
def test_refusals(env, bits):
    """Rows longer than the staging holds, and the calls that only know 4-bit codes."""
    uq, torch = env
    rng = wl.rng_for(36, 9 + bits)
    w = gen(rng, 8, 32768 + 128, bits, "f16")
    qw = uq.QuantLinear.from_numpy(w, bits=bits)
    x = to_dev16(torch, wl.gen_activations(rng, 1, qw.K), "f16")
    with pytest.raises(uq.UniqlError) as e:
        uq.uniql_w4_linear(qw, None, x)
    assert e.value.code == uq.UNIQL_E_SHAPE
    y = uq.uniql_w4_linear(qw, Keep(k_keep=32768), x[:, :32768])     # the same matrix, pruned to what fits
    torch.cuda.synchronize()
    assert y.shape == (1, 8)
    small = uq.QuantLinear.from_numpy(gen(rng, 256, 512, bits, "f16"), bits=bits)
    xs = to_dev16(torch, wl.gen_activations(rng, 1, 512), "f16")
    with pytest.raises(uq.UniqlError) as e:
        uq.uniql_w4_gate_up_silu([small, small], [None, None], xs[0])
    assert e.value.code == uq.UNIQL_E_SHAPE
    with pytest.raises(uq.UniqlError) as e:
        uq.uniql_w4_embedding(small, torch.zeros(1, dtype=torch.int32, device="cuda"))
    assert e.value.code == uq.UNIQL_E_SHAPE
