"""GPU parity of the bfloat16 variant (Sec. 4.1's compute type): the HIP path, through the C ABI, against
the CPU oracle's bfloat16 format.  Dequantised weights and embedding rows bit for bit; linears, fused
launches and rotations within TOL_BF16.

bfloat16 arrays are uint16 bit patterns on the numpy side and torch.bfloat16 on the device.
"""
import numpy as np
import pytest

import workloads as wl
from workloads import Keep
from parity_util import NORM_TOL_BF16, TOL_BF16, linear_err, normwise_err, rope_err

pytestmark = pytest.mark.gpu
FMT = "bf16"


@pytest.fixture(scope="module")
def env(uref):
    import torch
    import paper_2512_03383_amd as uq
    assert torch.cuda.is_available(), "gpu tests need an MI355X"
    uq.lib()
    uref.set_threads(min(16, uref.max_threads()))
    return uq, torch


def dev_bf16(torch, bits):
    """uint16 bit patterns -> bfloat16 tensor on the device."""
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def host_bits(torch, t):
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def host_vals(t):
    return t.float().cpu().numpy().astype(np.float64)


def run_linear(uq, torch, qw, keep, x_bits, pad=0):
    """GPU y as fp64 values; pad > 0 puts x and y in wider buffers (ld > kept dim) filled with sentinels."""
    M, kk = x_bits.shape
    nk, _ = uq.kept_dims(qw, keep)
    if pad:
        xb = torch.full((M, kk + pad), 77.0, dtype=torch.bfloat16, device="cuda")
        xb[:, :kk] = dev_bf16(torch, x_bits)
        yb = torch.full((M, nk + pad), -5.0, dtype=torch.bfloat16, device="cuda")
        uq.uniql_w4_linear(qw, keep, xb[:, :kk], yb[:, :nk])
        torch.cuda.synchronize()
        assert torch.all(yb[:, nk:] == -5.0), "wrote past n_keep"
        return host_vals(yb[:, :nk])
    y = uq.uniql_w4_linear(qw, keep, dev_bf16(torch, x_bits))
    torch.cuda.synchronize()
    return host_vals(y)


def gen(rng, N, K, sym=False):
    w = wl.gen_linear(rng, N, K, fmt=FMT)
    if sym:
        w["zeros"] = None
    return w


def oracle_linear(uref, w, x, keep, rows=None):
    return uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep, rows=rows, fmt=FMT)


# ------------------------------------------------------------------ dequant
def test_dequant_bit_exact_exhaustive(env, uref):
    """Every (q, z) pair with every bfloat16 scale in (0.005, 0.02) and a few extreme (normal) scales;
    then the kernels' own dequantisation, observed through one-hot inputs."""
    uq, torch = env
    lo, hi = (int(v) for v in wl.to_bf16_bits(np.array([0.005, 0.02], dtype=np.float32)))
    extra = [0x0080, 0x0081, 0x3f80, 0x3f81, 0x3fff, 0x4000, 0x7000, 0x1234, 0xbf80, 0xbc23]
    s_all = np.array(list(range(lo, hi + 1)) + extra, dtype=np.uint16)
    N, K = s_all.size, 16 * 128
    word_lo = sum(j << (4 * j) for j in range(8))
    word_hi = sum((8 + j) << (4 * j) for j in range(8))
    qweight = np.zeros((N, K // 8), dtype=np.uint32)
    qweight[:, 0::2] = word_lo
    qweight[:, 1::2] = word_hi
    w = {"qweight": qweight, "scales": np.repeat(s_all[:, None], 16, axis=1).copy(),
         "zeros": np.tile(np.arange(16, dtype=np.uint8), (N, 1))}
    ref = uref.w4_dequant(w["qweight"], w["scales"], w["zeros"], fmt=FMT)
    qw = uq.QuantLinear.from_numpy(w)
    got = host_bits(torch, uq.uniql_w4_dequant(qw))
    assert got.dtype == np.uint16 and np.array_equal(got, ref)       # signs of zeros included
    # through the linear kernels a zero weight is +0 whatever the signs of (q - z) and s
    def canon(bits):
        return np.where((bits & 0x7fff) == 0, 0, bits)
    for M in (1, 8):
        for k in (0, 5, 127, 128 + 9, K - 1):
            x = np.zeros((M, K), dtype=np.uint16)
            x[:, k] = 0x3f80
            y = uq.uniql_w4_linear(qw, None, dev_bf16(torch, x))
            torch.cuda.synchronize()
            assert np.array_equal(canon(host_bits(torch, y)[0]), canon(ref[:, k])), (M, k)


KEEPS = [
    Keep(),
    Keep(n_keep=870),
    Keep(k_keep=870),
    Keep(n_keep=333, k_keep=517),
    Keep(n_keep=1, k_keep=1),
    Keep(n_keep=16 * 54, row_seg_stride=64, row_seg_keep=54, row_seg_limit=1024),
    Keep(k_keep=8 * 108, col_seg_stride=128, col_seg_keep=108),
    Keep(n_keep=8 * 82, k_keep=16 * 41, row_seg_stride=128, row_seg_keep=82, row_seg_limit=1024,
         col_seg_stride=64, col_seg_keep=41),
    Keep(n_keep=10 * 54 + 2 * 109 + 128, row_seg_stride=64, row_seg_keep=54, row_seg_limit=640,
         row_seg2_stride=128, row_seg2_keep=109, row_seg2_limit=896),
]


@pytest.mark.parametrize("keep", KEEPS)
@pytest.mark.parametrize("sym", [False, True])
def test_dequant_bit_exact_pruned(env, uref, keep, sym):
    uq, torch = env
    w = gen(wl.rng_for(20, 30), 1024, 1024, sym)
    ref = uref.w4_dequant(w["qweight"], w["scales"], w["zeros"], keep, fmt=FMT)
    got = host_bits(torch, uq.uniql_w4_dequant(uq.QuantLinear.from_numpy(w), keep))
    assert np.array_equal(got, ref)


@pytest.mark.parametrize("N,K,n,pad", [(50, 384, 5, 0), (1000, 4096, 300, 8), (4096, 14336, 33, 16)])
def test_embedding_gather_bit_exact(env, uref, N, K, n, pad):
    uq, torch = env
    rng = wl.rng_for(20, N + K + n)
    w = gen(rng, N, K, sym=(n == 5))
    ids = rng.integers(0, N, n).astype(np.int32)
    ids[0], ids[-1] = N - 1, 0
    ref = uref.w4_embedding(w["qweight"], w["scales"], w["zeros"], ids, fmt=FMT)
    buf = torch.full((n, K + pad), -3.0, dtype=torch.bfloat16, device="cuda")
    out = uq.uniql_w4_embedding(uq.QuantLinear.from_numpy(w), torch.from_numpy(ids).cuda(), out=buf[:, :K])
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(torch, out), ref)
    if pad:
        assert torch.all(buf[:, K:] == -3.0), "wrote past K"


# ------------------------------------------------------------------- linear
@pytest.mark.parametrize("M", [1, 2, 5, 8, 16, 17, 32, 33, 64, 100])
@pytest.mark.parametrize("keep", KEEPS)
def test_linear_parity_1024(env, uref, keep, M):
    uq, torch = env
    rng = wl.rng_for(20, 31)
    w = gen(rng, 1024, 1024)
    qw = uq.QuantLinear.from_numpy(w)
    nk, kk = uq.kept_dims(qw, keep)
    x = wl.gen_activations(rng, M, kk, fmt=FMT)
    ref = oracle_linear(uref, w, x, keep)
    y = run_linear(uq, torch, qw, keep, x, pad=3 if M in (1, 5, 33) else 0)
    assert linear_err(y, ref) <= TOL_BF16
    if nk >= 64:
        assert normwise_err(y, ref) <= NORM_TOL_BF16


@pytest.mark.parametrize("N,K,keep,M", [
    (48, 128, Keep(), 1),
    (1000, 384, Keep(n_keep=999, k_keep=383), 1),
    (257, 2176, Keep(k_keep=2049), 3),
    (4096, 4096, Keep(k_keep=32 * 108, col_seg_stride=128, col_seg_keep=108), 1),    # o_proj
    (700, 18944, Keep(k_keep=14208), 1),                                          # ten chunks: run-time chunk count
    (300, 1280, Keep(k_keep=64 * 10, col_seg_stride=20, col_seg_keep=10), 2),     # element-wise staging
])
@pytest.mark.parametrize("sym", [False, True])
def test_linear_ragged_shapes(env, uref, N, K, keep, M, sym):
    uq, torch = env
    rng = wl.rng_for(21, N + K)
    w = gen(rng, N, K, sym)
    qw = uq.QuantLinear.from_numpy(w)
    nk, kk = uq.kept_dims(qw, keep)
    x = wl.gen_activations(rng, M, kk, fmt=FMT)
    ref = oracle_linear(uref, w, x, keep)
    y = run_linear(uq, torch, qw, keep, x)
    assert y.shape == ref.shape and linear_err(y, ref) <= TOL_BF16


def _sample_rows(n, rng, count=192):
    rows = np.unique(np.concatenate([[0, 1, n - 2, n - 1], rng.integers(0, n, count)]))
    return rows.astype(np.int32)


@pytest.mark.parametrize("rate", [0, 15])
def test_llama3_8b_decode_layer_full_size(env, uref, rate):
    """The seven linears of the Llama-3-8B shaped layer at full size, M = 1: sampled rows against the oracle."""
    uq, torch = env
    rng = wl.rng_for(22, rate)
    for spec in wl.llama3_8b_layer(rate):
        w = gen(rng, spec.N, spec.K)
        qw = uq.QuantLinear.from_numpy(w)
        x = wl.gen_activations(rng, 1, spec.k_keep, fmt=FMT)
        y = run_linear(uq, torch, qw, spec.keep, x)
        assert y.shape == (1, spec.n_keep)
        rows = _sample_rows(spec.n_keep, rng)
        ref = oracle_linear(uref, w, x, spec.keep, rows=rows)
        rms = np.sqrt(np.mean(ref ** 2))
        err = np.max(np.abs(y[:, rows] - ref) / np.maximum(np.abs(ref), 1e-2 * rms))
        assert err <= TOL_BF16, (spec.name, err)


@pytest.mark.parametrize("N,K,keep", [
    (2048, 128, Keep()),                                   # the row threshold of short rows, one group per row
    (9001, 1024, Keep(k_keep=1001)),                       # ragged rows, column prefix with a tail of one
    (12000, 2304, Keep(n_keep=8193, k_keep=2055)),         # two chunks
    (8300, 6144, Keep(k_keep=6100)),                       # three chunks: activations read from LDS per tile
    (8200, 14336, Keep(k_keep=12185)),                     # six
    (8200, 16384, Keep(k_keep=16383)),                     # eight chunks
    (2304, 1024, Keep(col_seg_stride=128, col_seg_keep=108)),              # column segments: a partly kept unit per segment
    (2100, 2048, Keep(col_seg_stride=64, col_seg_keep=37)),                # odd keep
    (2200, 6144, Keep(col_seg_stride=128, col_seg_keep=82)),               # three chunks
    (4096, 1024, Keep(n_keep=3456, row_seg_stride=128, row_seg_keep=108, row_seg_limit=4096)),   # row segments
    (2048, 10240, Keep()),                                 # the row threshold of long rows
])
@pytest.mark.parametrize("sym", [False, True])
def test_streaming_gemv_shapes(env, uref, N, K, keep, sym):
    """Tall matrices (the persistent streaming kernel): every row against the oracle."""
    uq, torch = env
    rng = wl.rng_for(23, N + K)
    w = gen(rng, N, K, sym)
    qw = uq.QuantLinear.from_numpy(w)
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, 1, kk, fmt=FMT)
    y = run_linear(uq, torch, qw, keep, x, pad=3)
    ref = oracle_linear(uref, w, x, keep)
    assert y.shape == ref.shape and linear_err(y, ref) <= TOL_BF16


@pytest.mark.parametrize("N,K,keep", [
    (256, 512, Keep()),                                    # the block-per-rows kernel
    (1024, 1024, Keep(n_keep=870, k_keep=515)),
    (4096, 128, Keep()),                                   # the row threshold of the streaming launch
    (6000, 6144, Keep(n_keep=4500, k_keep=6001)),          # three chunks
    (14336, 4096, Keep(n_keep=12185)),                     # Llama-3-8B gate / up at 15 %
])
@pytest.mark.parametrize("sym", [False, True])
def test_gate_up_silu(env, uref, N, K, keep, sym):
    uq, torch = env
    rng = wl.rng_for(24, N + K)
    wg, wu = gen(rng, N, K, sym), gen(rng, N, K, sym)
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, 1, kk, fmt=FMT)
    h = uq.uniql_w4_gate_up_silu([uq.QuantLinear.from_numpy(wg), uq.QuantLinear.from_numpy(wu)], [keep, keep],
                                 dev_bf16(torch, x[0]))
    torch.cuda.synchronize()
    assert h.shape == (nk,) and h.dtype == torch.bfloat16
    rows = np.arange(nk, dtype=np.int32) if nk <= 6000 else _sample_rows(nk, rng, 512)
    g = oracle_linear(uref, wg, x, keep, rows=rows)
    u = oracle_linear(uref, wu, x, keep, rows=rows)
    ref = g / (1.0 + np.exp(-g)) * u
    got = host_vals(h)[rows].reshape(1, -1)
    rms = np.sqrt(np.mean(ref ** 2))
    assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms)) <= TOL_BF16


@pytest.mark.parametrize("N,K,keep,M", [
    (14208 + 37, 3584, Keep(n_keep=14208), 8),             # Qwen2.5-7B gate / up at 25 %
    (10300, 4096, Keep(n_keep=10241, k_keep=4089), 13),    # ragged rows and columns, sixteen token slots
])
def test_gate_up_silu_decode_batches(env, uref, N, K, keep, M):
    """The gated MLP's hidden vectors of a decode batch in bfloat16, one launch: sampled rows of every token."""
    uq, torch = env
    rng = wl.rng_for(24, 500 + N + M)
    wg, wu = gen(rng, N, K), gen(rng, N, K)
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, M, kk, fmt=FMT)
    h = uq.uniql_w4_gate_up_silu_batch([uq.QuantLinear.from_numpy(wg), uq.QuantLinear.from_numpy(wu)], [keep, keep],
                                       dev_bf16(torch, x))
    torch.cuda.synchronize()
    assert h.shape == (M, nk) and h.dtype == torch.bfloat16
    rows = _sample_rows(nk, rng, 256)
    g = oracle_linear(uref, wg, x, keep, rows=rows)
    u = oracle_linear(uref, wu, x, keep, rows=rows)
    ref = g / (1.0 + np.exp(-g)) * u
    got = host_vals(h)[:, rows]
    rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
    assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms)) <= TOL_BF16


@pytest.mark.parametrize("model", ["llama3_8b_p15", "qwen25_7b_p25"])
@pytest.mark.parametrize("sym", [False, True])
def test_fused_qkv_rope(env, uref, model, sym):
    """q = RoPE(x Wq), k = RoPE(x Wk), v = x Wv in one launch, against the oracle's fp64 composition."""
    uq, torch = env
    if model == "llama3_8b_p15":
        specs, rope = {s.name: s for s in wl.llama3_8b_layer(15)}, wl.llama3_8b_rope(15, T=1)
    else:
        specs, rope = {s.name: s for s in wl.qwen25_7b_layer(25)}, wl.qwen25_7b_rope(25, T=1)
    rng = wl.rng_for(25, len(model))
    names = ["q_proj", "k_proj", "v_proj"]
    ws = [gen(rng, specs[n].N, specs[n].K, sym) for n in names]
    qws = [uq.QuantLinear.from_numpy(w) for w in ws]
    keeps = [specs[n].keep for n in names]
    x = wl.gen_activations(rng, 1, specs["q_proj"].k_keep, fmt=FMT)
    r = wl.gen_rope_inputs(rng, rope)
    pos, idx = r["positions"][:1].copy(), r["kept_idx"]
    q, k, v = uq.uniql_w4_qkv_rope(qws, keeps, dev_bf16(torch, x[0]), torch.from_numpy(pos).cuda(),
                                   torch.from_numpy(idx).cuda(), rope.Hq, rope.Hkv, rope.D_full, rope.D_keep, rope.theta)
    torch.cuda.synchronize()
    assert q.dtype == torch.bfloat16
    rq, rk, rv = uref.qkv_rope(ws[0], keeps[0], ws[1], keeps[1], ws[2], keeps[2], x, pos, idx, rope.Hq, rope.Hkv,
                               rope.D_full, rope.D_keep, rope.theta, fmt=FMT)
    # Qwen's rows (28 groups) take the one launch as well; in either case the bar is that of a linear
    for got, ref in ((q, rq), (k, rk), (v, rv)):
        assert linear_err(host_vals(got).reshape(1, -1), ref.reshape(1, -1)) <= TOL_BF16


@pytest.mark.parametrize("N,K,keep,M", [
    (2048, 128, Keep(), 2),
    (14208 + 37, 3584, Keep(n_keep=14208), 8),             # Qwen2.5-7B gate / up at 25 %, eight tokens
    (3584, 18944, Keep(k_keep=14208), 16),                 # its down_proj, sixteen tokens
    (4100, 6144, Keep(k_keep=6016), 4),
    (4096, 4096, Keep(k_keep=32 * 108, col_seg_stride=128, col_seg_keep=108), 8),   # o_proj, column segments
    (14208 + 37, 3584, Keep(n_keep=14208), 32),            # the configurations of 17..32 and 33..64 tokens, tall and short
    (14208 + 37, 3584, Keep(n_keep=14208), 64),
    (3584, 18944, Keep(k_keep=14208), 32),
    (3584, 18944, Keep(k_keep=14208), 64),
    (14208 + 37, 3584, Keep(n_keep=14208), 16),            # activations staged once per block: sixteen, three and
    (10300, 4096, Keep(n_keep=10241, k_keep=4089), 3),     # thirteen tokens, ragged rows and columns
    (20600, 1024, Keep(n_keep=20481, k_keep=1017), 13),
])
def test_decode_batches(env, uref, N, K, keep, M):
    uq, torch = env
    rng = wl.rng_for(26, N + K + M)
    w = gen(rng, N, K)
    qw = uq.QuantLinear.from_numpy(w)
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, M, kk, fmt=FMT)
    y = run_linear(uq, torch, qw, keep, x)
    rows = _sample_rows(nk, rng, 256)
    ref = oracle_linear(uref, w, x, keep, rows=rows)
    rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
    assert np.max(np.abs(y[:, rows] - ref) / np.maximum(np.abs(ref), 1e-2 * rms)) <= TOL_BF16


@pytest.mark.parametrize("M", [256, 1024, 4096])
def test_prefill_gemm_sampled(env, uref, M):
    """Prefill-sized dequant-GEMM at the gate/up and down shapes, 15 % pruning: sampled (token, row) pairs."""
    uq, torch = env
    rng = wl.rng_for(27, M)
    for spec in wl.prefill_linears(15):
        w = gen(rng, spec.N, spec.K)
        qw = uq.QuantLinear.from_numpy(w)
        x = wl.gen_activations(rng, M, spec.k_keep, fmt=FMT)
        y = uq.uniql_w4_linear(qw, spec.keep, dev_bf16(torch, x))
        torch.cuda.synchronize()
        toks = np.unique(np.concatenate([[0, 255, M - 256, M - 1], rng.integers(0, M, 6)]))
        rows = _sample_rows(spec.n_keep, rng, 64)
        ref = oracle_linear(uref, w, np.ascontiguousarray(x[toks]), spec.keep, rows=rows)
        rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
        got = host_vals(y[torch.from_numpy(toks).cuda()][:, torch.from_numpy(rows.astype(np.int64)).cuda()])
        err = np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms))
        assert err <= TOL_BF16, (spec.name, err)


def test_prefill_persistent_tiles_ragged(env, uref):
    """256 x 256 tiles on the persistent grid with ragged rows, tokens and a column tail: sampled (token, row) pairs
    that include the edges of the first and last tiles."""
    uq, torch = env
    rng = wl.rng_for(28, 1)
    N, K, keep, M = 12300, 1152, Keep(n_keep=12200, k_keep=1100), 1000
    w = gen(rng, N, K)
    qw = uq.QuantLinear.from_numpy(w)
    x = wl.gen_activations(rng, M, 1100, fmt=FMT)
    y = uq.uniql_w4_linear(qw, keep, dev_bf16(torch, x))
    torch.cuda.synchronize()
    toks = np.unique(np.concatenate([[0, 255, 256, 767, 768, M - 1], rng.integers(0, M, 6)]))
    rows = np.unique(np.concatenate([_sample_rows(12200, rng, 64), [255, 256, 12031, 12032, 12199]])).astype(np.int32)
    ref = oracle_linear(uref, w, np.ascontiguousarray(x[toks]), keep, rows=rows)
    rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
    got = host_vals(y[torch.from_numpy(toks).cuda()][:, torch.from_numpy(rows.astype(np.int64)).cuda()])
    assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms)) <= TOL_BF16


def test_prefill_tiles_ragged(env, uref):
    """Token and row counts that leave partial tiles in the 128 x 256 and the smaller tilings; every output."""
    uq, torch = env
    rng = wl.rng_for(28, 0)
    for N, K, keep, M in [(520, 640, Keep(n_keep=515, k_keep=600), 130), (300, 256, Keep(), 65),
                          (1024, 512, Keep(k_keep=4 * 100, col_seg_stride=128, col_seg_keep=100), 200)]:
        w = gen(rng, N, K)
        qw = uq.QuantLinear.from_numpy(w)
        nk, kk = uref.count_kept(N, K, keep)
        x = wl.gen_activations(rng, M, kk, fmt=FMT)
        y = run_linear(uq, torch, qw, keep, x)
        ref = oracle_linear(uref, w, x, keep)
        assert linear_err(y, ref) <= TOL_BF16, (N, K, M)


def test_multi_call_and_mixed_formats(env, uref):
    """Three bfloat16 linears in one multi call equal the single calls bit for bit; a call that mixes an fp16
    and a bfloat16 matrix runs them one by one."""
    uq, torch = env
    rng = wl.rng_for(29, 0)
    specs = {s.name: s for s in wl.llama3_8b_layer(15)}
    names = ["q_proj", "k_proj", "v_proj"]
    ws = [gen(rng, specs[n].N, specs[n].K) for n in names]
    qws = [uq.QuantLinear.from_numpy(w) for w in ws]
    keeps = [specs[n].keep for n in names]
    x = dev_bf16(torch, wl.gen_activations(rng, 1, 4096, fmt=FMT))
    ys = [torch.empty((1, specs[n].n_keep), dtype=torch.bfloat16, device="cuda") for n in names]
    uq.uniql_w4_linear_multi(qws, keeps, [x] * 3, ys)
    torch.cuda.synchronize()
    for qw, kp, y in zip(qws, keeps, ys):
        assert torch.equal(uq.uniql_w4_linear(qw, kp, x), y)
    w16 = wl.gen_linear(rng, 512, 4096)
    q16 = uq.QuantLinear.from_numpy(w16)
    x16 = torch.from_numpy(wl.gen_activations(rng, 1, 4096)).cuda()
    y16 = torch.empty((1, 512), dtype=torch.float16, device="cuda")
    yb = torch.empty((1, specs["k_proj"].n_keep), dtype=torch.bfloat16, device="cuda")
    uq.uniql_w4_linear_multi([q16, qws[1]], [None, keeps[1]], [x16, x], [y16, yb])
    torch.cuda.synchronize()
    assert torch.equal(yb, ys[1]) and torch.equal(y16, uq.uniql_w4_linear(q16, None, x16))


@pytest.mark.parametrize("M", [3, 8, 16, 32])
def test_multi_call_decode_batches_share_a_launch(env, uref, M):
    """q / k / v of a decode batch in bfloat16 through one launch of the decode-batch kernel: the bits of single calls
    and the oracle within the bfloat16 bar; the same tokens with an fp16 member mixed in go one by one."""
    uq, torch = env
    rng = wl.rng_for(29, 40 + M)
    specs = {s.name: s for s in wl.llama3_8b_layer(15)}
    names = ["q_proj", "k_proj", "v_proj"]
    ws = [gen(rng, specs[n].N, specs[n].K) for n in names]
    qws = [uq.QuantLinear.from_numpy(w) for w in ws]
    keeps = [specs[n].keep for n in names]
    xh = wl.gen_activations(rng, M, 4096, fmt=FMT)
    x = dev_bf16(torch, xh)
    ys = [torch.empty((M, specs[n].n_keep), dtype=torch.bfloat16, device="cuda") for n in names]
    uq.uniql_w4_linear_multi(qws, keeps, [x] * 3, ys)
    torch.cuda.synchronize()
    for w, qw, kp, y in zip(ws, qws, keeps, ys):
        assert torch.equal(uq.uniql_w4_linear(qw, kp, x), y)
        ref = oracle_linear(uref, w, xh, kp)
        assert linear_err(y.float().cpu().numpy().astype(np.float64), ref) <= TOL_BF16
    w16 = wl.gen_linear(rng, 512, 4096)
    q16 = uq.QuantLinear.from_numpy(w16)
    x16 = torch.from_numpy(wl.gen_activations(rng, M, 4096)).cuda()
    y16 = torch.empty((M, 512), dtype=torch.float16, device="cuda")
    yb = torch.empty((M, specs["k_proj"].n_keep), dtype=torch.bfloat16, device="cuda")
    uq.uniql_w4_linear_multi([q16, qws[1]], [None, keeps[1]], [x16, x], [y16, yb])
    torch.cuda.synchronize()
    assert torch.equal(yb, ys[1]) and torch.equal(y16, uq.uniql_w4_linear(q16, None, x16))


def test_repack_carries_bf16_scales(env, uref):
    """The compact copy moves scales as they are stored: the repacked matrix gives the same bits."""
    uq, torch = env
    rng = wl.rng_for(30, 0)
    keep = Keep(n_keep=700, k_keep=1500)
    w = gen(rng, 1000, 2048)
    qw = uq.QuantLinear.from_numpy(w)
    out, keep2 = uq.uniql_w4_repack(qw, keep)
    torch.cuda.synchronize()
    q2, s2, z2, ko = uref.w4_repack(w["qweight"], w["scales"], w["zeros"], keep)
    assert np.array_equal(out.qweight.cpu().numpy().view(np.uint32), q2)
    assert np.array_equal(host_bits(torch, out.scales), s2) and np.array_equal(out.zeros.cpu().numpy(), z2)
    x = dev_bf16(torch, wl.gen_activations(rng, 1, 1500, fmt=FMT))
    assert torch.equal(uq.uniql_w4_linear(qw, keep, x), uq.uniql_w4_linear(out, keep2, x))


# --------------------------------------------------------------------- RoPE
def run_rope(uq, torch, r, spec):
    q = dev_bf16(torch, r["q"])
    k = dev_bf16(torch, r["k"]) if r["k"] is not None else None
    uq.uniql_pruned_rope(q, k, torch.from_numpy(r["positions"]).cuda(), torch.from_numpy(r["kept_idx"]).cuda(),
                         spec.D_full, spec.theta)
    torch.cuda.synchronize()
    return host_vals(q), (host_vals(k) if k is not None else None)


@pytest.mark.parametrize("spec", [
    wl.small_rope(),
    wl.llama3_8b_rope(15), wl.qwen25_7b_rope(25, T=16), wl.llama3_8b_rope(15, T=37),
    wl.RopeSpec(T=3, Hq=4, Hkv=4, H_tab=4, D_full=64, D_keep=2, theta=1e4, pos_max=100),
    wl.RopeSpec(T=5, Hq=6, Hkv=2, H_tab=1, D_full=256, D_keep=202, theta=1e6, pos_max=32768),   # odd pair count
    wl.RopeSpec(T=300, Hq=2, Hkv=0, H_tab=2, D_full=1024, D_keep=700, theta=1e4, pos_max=32768),
    wl.prefill_rope(15, T=4096),
], ids=lambda s: f"T{s.T}_H{s.Hq}-{s.Hkv}-{s.H_tab}_D{s.D_full}-{s.D_keep}")
def test_rope_parity(env, uref, spec):
    uq, torch = env
    r = wl.gen_rope_inputs(wl.rng_for(31, 40), spec, fmt=FMT)
    qo, ko = uref.pruned_rope(r["q"], r["k"], r["positions"], r["kept_idx"], spec.D_full, spec.theta, fmt=FMT)
    gq, gk = run_rope(uq, torch, r, spec)
    assert rope_err(gq, qo) <= TOL_BF16
    if ko is not None:
        assert rope_err(gk, ko) <= TOL_BF16
