"""GPU parity of the 8-bit codes (Eq. 3 with N = 8) through the C ABI against the CPU oracle: the dequantised matrix
bit for bit, the linear within the element-wise bar of the 4-bit linears, in fp16 and bfloat16."""
import numpy as np
import pytest

import workloads as wl
from workloads import Keep
from parity_util import NORM_TOL, NORM_TOL_BF16, TOL, TOL_BF16, linear_err, normwise_err

pytestmark = pytest.mark.gpu


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


def gen8(rng, N, K, fmt, sym=False):
    w = wl.gen_linear8(rng, N, K, fmt=fmt)
    if sym:
        w["zeros"] = None
    return w


KEEPS = [
    Keep(),
    Keep(n_keep=870, k_keep=517),
    Keep(n_keep=1, k_keep=1),
    Keep(n_keep=16 * 54, row_seg_stride=64, row_seg_keep=54, row_seg_limit=1024),
    Keep(k_keep=8 * 108, col_seg_stride=128, col_seg_keep=108),
    Keep(n_keep=8 * 82, k_keep=16 * 41, row_seg_stride=128, row_seg_keep=82, row_seg_limit=1024,
         col_seg_stride=64, col_seg_keep=41),
    Keep(n_keep=10 * 54 + 2 * 109 + 128, row_seg_stride=64, row_seg_keep=54, row_seg_limit=640,
         row_seg2_stride=128, row_seg2_keep=109, row_seg2_limit=896),
]


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
@pytest.mark.parametrize("sym", [False, True])
@pytest.mark.parametrize("keep", KEEPS)
def test_w8_dequant_bit_exact(env, uref, keep, sym, fmt):
    uq, torch = env
    w = gen8(wl.rng_for(30, 1), 1024, 1024, fmt, sym)
    ref = uref.wq_dequant(8, w["qweight"], w["scales"], w["zeros"], keep, fmt=fmt)
    got = uq.uniql_w4_dequant(uq.QuantLinear.from_numpy(w, bits=8), keep)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(torch, got), ref.view(np.uint16))


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_w8_dequant_every_code_and_zero_point(env, uref, fmt):
    """Row z holds the codes 0..255 (four times) under zero point z, with scales that produce subnormal, tie and
    large results."""
    uq, torch = env
    codes = np.tile(np.arange(256, dtype=np.uint32), (256, 4))                      # [256][1024]
    qweight = np.zeros((256, 256), dtype=np.uint32)
    for j in range(4):
        qweight |= codes[:, j::4] << np.uint32(8 * j)
    zeros = np.repeat(np.arange(256, dtype=np.uint8)[:, None], 8, axis=1)
    sb = np.array([0x2000, 0x211f, 0x2400, 0x1c01, 0x0003, 0x3555, 0x5000, 0x0400], dtype=np.uint16)
    if fmt == "bf16":
        sb = np.array([0x3a00, 0x3a13, 0x3b80, 0x0081, 0x0003, 0x3eab, 0x4700, 0x0080], dtype=np.uint16)
    scales = np.tile(sb, (256, 1))
    scales = scales.view(np.float16) if fmt == "f16" else scales
    w = {"qweight": qweight, "scales": np.ascontiguousarray(scales), "zeros": zeros}
    ref = uref.wq_dequant(8, w["qweight"], w["scales"], w["zeros"], fmt=fmt)
    got = uq.uniql_w4_dequant(uq.QuantLinear.from_numpy(w, bits=8), None)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(torch, got), ref.view(np.uint16))


@pytest.mark.parametrize("fmt", ["f16", "bf16"])
@pytest.mark.parametrize("M", [1, 2, 5, 16])
@pytest.mark.parametrize("keep", KEEPS)
def test_w8_linear_parity_1024(env, uref, keep, M, fmt):
    uq, torch = env
    rng = wl.rng_for(30, 2)
    w = gen8(rng, 1024, 1024, fmt, sym=(M == 5))
    qw = uq.QuantLinear.from_numpy(w, bits=8)
    nk, kk = uq.kept_dims(qw, keep)
    x = wl.gen_activations(rng, M, kk, fmt=fmt)
    ref = uref.wq_linear(8, w["qweight"], w["scales"], w["zeros"], x, keep, fmt=fmt)
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


@pytest.mark.parametrize("N,K,keep", [
    (14336, 4096, Keep(n_keep=12185)),          # Llama-3-8B gate / up at 15 %
    (4096, 14336, Keep(k_keep=12185)),          # down: 762 chunks per row, the last one partly kept
    (300, 32768, Keep()),                       # the longest row the staging holds
    (7, 128, Keep()),                           # one group, fewer rows than a block has waves
])
def test_w8_linear_model_shapes(env, uref, N, K, keep):
    uq, torch = env
    rng = wl.rng_for(30, N + K)
    w = gen8(rng, N, K, "f16")
    qw = uq.QuantLinear.from_numpy(w, bits=8)
    nk, kk = uq.kept_dims(qw, keep)
    x = wl.gen_activations(rng, 1, kk)
    rows = np.unique(np.concatenate([[0, 1, nk - 2, nk - 1], rng.integers(0, nk, 128)])).astype(np.int32)
    rows = rows[(rows >= 0) & (rows < nk)]
    ref = uref.wq_linear(8, w["qweight"], w["scales"], w["zeros"], x, keep, rows=rows)
    y = uq.uniql_w4_linear(qw, keep, to_dev16(torch, x, "f16"))
    y2 = uq.uniql_w4_linear(qw, keep, to_dev16(torch, x, "f16"))
    torch.cuda.synchronize()
    assert torch.equal(y, y2)
    got = host_vals(y)[:, rows]
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms)) <= TOL


def test_w8_refusals(env):
    """Rows longer than the staging holds, and the calls that only know 4-bit codes."""
    uq, torch = env
    rng = wl.rng_for(30, 9)
    w = gen8(rng, 8, 32768 + 128, "f16")
    qw = uq.QuantLinear.from_numpy(w, bits=8)
    x = to_dev16(torch, wl.gen_activations(rng, 1, qw.K), "f16")
    with pytest.raises(uq.UniqlError) as e:
        uq.uniql_w4_linear(qw, None, x)
    assert e.value.code == uq.UNIQL_E_SHAPE
    y = uq.uniql_w4_linear(qw, Keep(k_keep=32768), x[:, :32768])     # the same matrix, pruned to what fits
    torch.cuda.synchronize()
    assert y.shape == (1, 8)
    small = uq.QuantLinear.from_numpy(gen8(rng, 256, 512, "f16"), bits=8)
    xs = to_dev16(torch, wl.gen_activations(rng, 1, 512), "f16")
    with pytest.raises(uq.UniqlError) as e:
        uq.uniql_w4_gate_up_silu([small, small], [None, None], xs[0])
    assert e.value.code == uq.UNIQL_E_SHAPE
    with pytest.raises(uq.UniqlError) as e:
        uq.uniql_w4_embedding(small, torch.zeros(1, dtype=torch.int32, device="cuda"))
    assert e.value.code == uq.UNIQL_E_SHAPE
