"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle."""
import numpy as np
import pytest

import workloads as wl
from workloads import Keep
from parity_util import NORM_TOL, TOL, linear_err, normwise_err, rope_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env(uref):
    import torch
    import paper_2512_03383_amd as uq
    assert torch.cuda.is_available(), "gpu tests need an MI355X"
    uq.lib()
    uref.set_threads(min(16, uref.max_threads()))
    return uq, torch


def to_dev(torch, a):
    return torch.from_numpy(a).cuda()


def run_linear(uq, torch, w, qw, keep, x, pad=0):
    """GPU y as numpy fp16; pad > 0 puts x and y in wider buffers (ld > kept dim) filled with sentinels."""
    M, kk = x.shape
    nk, _ = uq.kept_dims(qw, keep)
    if pad:
        xb = torch.full((M, kk + pad), 77.0, dtype=torch.float16, device="cuda")
        xb[:, :kk] = to_dev(torch, x)
        yb = torch.full((M, nk + pad), -5.0, dtype=torch.float16, device="cuda")
        uq.uniql_w4_linear(qw, keep, xb[:, :kk], yb[:, :nk])
        torch.cuda.synchronize()
        assert torch.all(yb[:, nk:] == -5.0), "wrote past n_keep"
        return yb[:, :nk].cpu().numpy()
    y = uq.uniql_w4_linear(qw, keep, to_dev(torch, x))
    torch.cuda.synchronize()
    return y.cpu().numpy()


# ------------------------------------------------------------------ dequant
def test_dequant_bit_exact_exhaustive(env, uref):
    """Every (q, z) pair with every fp16 scale in (0.005, 0.02) and a few extreme scales."""
    uq, torch = env
    s_bits = np.arange(np.float16(0.005).view(np.uint16), np.float16(0.02).view(np.uint16) + 1, dtype=np.uint16)
    extra = np.array([0x0001, 0x0003, 0x03ff, 0x0400, 0x0401, 0x1400, 0x3c00, 0x3c01, 0x6bff, 0x7000, 0x8001, 0xbc00],
                     dtype=np.uint16)
    s_all = np.concatenate([s_bits, extra]).view(np.float16)
    N, K = s_all.size, 16 * 128
    word_lo = sum(j << (4 * j) for j in range(8))
    word_hi = sum((8 + j) << (4 * j) for j in range(8))
    qweight = np.zeros((N, K // 8), dtype=np.uint32)
    qweight[:, 0::2] = word_lo
    qweight[:, 1::2] = word_hi
    w = {"qweight": qweight, "scales": np.repeat(s_all[:, None], 16, axis=1).copy(),
         "zeros": np.tile(np.arange(16, dtype=np.uint8), (N, 1))}
    ref = uref.w4_dequant(w["qweight"], w["scales"], w["zeros"])
    qw = uq.QuantLinear.from_numpy(w)
    got = uq.uniql_w4_dequant(qw).cpu().numpy()
    # Scales are non-negative by construction (Eq. 3); for the two negative test scales the sign of
    # an exact zero (q == z) is left unspecified, everything else is compared bit for bit.
    neg = s_all < 0

    def canon(a):
        a = a.copy()
        a[neg] = np.where(a[neg] == 0, np.float16(0), a[neg])
        return a.view(np.uint16)

    assert np.array_equal(canon(got), canon(ref))
    # the kernels' packed-fp16 dequantisation, observed through one-hot inputs: y[:, k] is column k
    # (rows whose scale overflows fp16 hold infinities, and inf * 0 is NaN in any dot product: left out)
    fin = np.isfinite(ref.astype(np.float64)).all(axis=1)
    for M in (1, 8):
        for k in (0, 5, 127, 128 + 9, K - 1):
            x = np.zeros((M, K), dtype=np.float16)
            x[:, k] = 1.0
            y = run_linear(uq, torch, w, qw, None, x)
            assert np.array_equal(canon(y[0][:, None])[fin, 0], canon(ref[:, k:k + 1])[fin, 0]), (M, k)


KEEPS = [
    Keep(),
    Keep(n_keep=870),
    Keep(k_keep=870),
    Keep(n_keep=333, k_keep=517),
    Keep(n_keep=1, k_keep=1),
    Keep(n_keep=16 * 54, row_seg_stride=64, row_seg_keep=54, row_seg_limit=1024),
    Keep(k_keep=8 * 108, col_seg_stride=128, col_seg_keep=108),
    Keep(n_keep=2 * 300 + 224, row_seg_stride=400, row_seg_keep=300, row_seg_limit=800),
    Keep(n_keep=8 * 82, k_keep=16 * 41, row_seg_stride=128, row_seg_keep=82, row_seg_limit=1024,
         col_seg_stride=64, col_seg_keep=41),
    # two families of row segments and a whole-kept tail (Mamba in_proj with head and state dimension pruned)
    Keep(n_keep=10 * 54 + 2 * 109 + 128, row_seg_stride=64, row_seg_keep=54, row_seg_limit=640,
         row_seg2_stride=128, row_seg2_keep=109, row_seg2_limit=896),
    Keep(n_keep=500 + 4 * 100, k_keep=700, row_seg_stride=512, row_seg_keep=500, row_seg_limit=512,
         row_seg2_stride=128, row_seg2_keep=100, row_seg2_limit=1024),
]


@pytest.mark.parametrize("keep", KEEPS)
def test_dequant_bit_exact_pruned(env, uref, keep):
    uq, torch = env
    w = wl.gen_linear(wl.rng_for(0, 30), 1024, 1024)
    ref = uref.w4_dequant(w["qweight"], w["scales"], w["zeros"], keep)
    got = uq.uniql_w4_dequant(uq.QuantLinear.from_numpy(w), keep).cpu().numpy()
    assert np.array_equal(got.view(np.uint16), ref.view(np.uint16))


# ------------------------------------------------------------------- linear
def test_small_case_config0(env, uref):
    """1024x1024, first 870 output rows, M = 1 (the small benchmark configuration)."""
    uq, torch = env
    spec = wl.small_case()
    rng = wl.rng_for(0)
    w = wl.gen_linear(rng, spec.N, spec.K)
    x = wl.gen_activations(rng, 1, spec.k_keep)
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, spec.keep)
    y = run_linear(uq, torch, w, uq.QuantLinear.from_numpy(w), spec.keep, x)
    assert y.shape == (1, 870)
    assert linear_err(y, ref) <= TOL


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 16, 17, 32, 33, 64, 100])
@pytest.mark.parametrize("keep", KEEPS)
def test_linear_parity_1024(env, uref, keep, M):
    uq, torch = env
    rng = wl.rng_for(0, 31)
    w = wl.gen_linear(rng, 1024, 1024)
    qw = uq.QuantLinear.from_numpy(w)
    nk, kk = uq.kept_dims(qw, keep)
    x = wl.gen_activations(rng, M, kk)
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    y = run_linear(uq, torch, w, qw, keep, x, pad=3 if M in (1, 5, 33) else 0)
    assert linear_err(y, ref) <= TOL
    if nk >= 64:      # the norm-wise figure needs enough outputs to average over
        assert normwise_err(y, ref) <= NORM_TOL


@pytest.mark.parametrize("sym", [False, True])
@pytest.mark.parametrize("M", [2, 7, 12, 20, 32])
@pytest.mark.parametrize("N,K,keep", [
    (999, 1152, Keep()),                               # 9 groups and an odd number of rows: the arrays end in the middle of a 32-bit word
    (1000, 1408, Keep(n_keep=777, k_keep=1283)),       # 11 groups, the last kept group short, tail columns
    (333, 2944, Keep(k_keep=2817)),                    # 23 groups over eight waves: three groups per wave, the last wave short
    (4000, 1024, Keep()),                              # exactly 8 groups, K not split
    (2500, 3200, Keep(k_keep=25 * 100, col_seg_stride=128, col_seg_keep=100)),    # column segments, 25 groups
    (640, 1920, Keep(k_keep=15 * 77, col_seg_stride=128, col_seg_keep=77)),       # an odd number of kept columns per segment
    (515, 896, Keep()),                                # 7 groups: fewer than the decode-batch kernel takes
    (9700, 1024, Keep(n_keep=9650)),                   # more than 600 row tiles: above 8 tokens the slab kernel
])
def test_decode_batch_shapes(env, uref, N, K, keep, M, sym):
    """2 .. 32 tokens on shapes that put the ends of the arrays, of the rows and of the K split in every position
    (every row against the oracle: the last stored row reads the arrays' last bytes)."""
    uq, torch = env
    rng = wl.rng_for(21, N + K + M)
    w = wl.gen_linear(rng, N, K, sym_zero=sym)
    qw = uq.QuantLinear.from_numpy(w) if not sym else uq.QuantLinear.from_numpy({"qweight": w["qweight"], "scales": w["scales"], "zeros": None})
    nk, kk = uq.kept_dims(qw, keep)
    x = wl.gen_activations(rng, M, kk)
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    y = run_linear(uq, torch, w, qw, keep, x, pad=5 if M in (7, 20) else 0)
    assert linear_err(y, ref) <= TOL
    assert normwise_err(y, ref) <= NORM_TOL


@pytest.mark.parametrize("N,K,keep", [
    (48, 128, Keep()),                      # a single group, fewer rows than one block handles
    (7, 256, Keep(k_keep=129)),             # one column into the second group
    (130, 2176, Keep(n_keep=129, k_keep=2049)),   # one column past a 2048-column chunk
    (64, 18944, Keep(k_keep=14208)),        # longest benchmark K (Qwen MLP down)
    (300, 4096, Keep()),
])
@pytest.mark.parametrize("M", [1, 4, 7])
def test_linear_parity_ragged_shapes(env, uref, N, K, keep, M):
    uq, torch = env
    rng = wl.rng_for(0, 32)
    w = wl.gen_linear(rng, N, K)
    qw = uq.QuantLinear.from_numpy(w)
    nk, kk = uq.kept_dims(qw, keep)
    x = wl.gen_activations(rng, M, kk)
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    y = run_linear(uq, torch, w, qw, keep, x)
    assert linear_err(y, ref) <= TOL


def test_symmetric_zero8_and_extreme_values(env, uref):
    """zero = 8 everywhere (the symmetric scheme), large activations, zero activations."""
    uq, torch = env
    rng = wl.rng_for(0, 33)
    w = wl.gen_linear(rng, 256, 512, sym_zero=True)
    qw = uq.QuantLinear.from_numpy(w)
    for M in (1, 6):
        x = (wl.gen_activations(rng, M, 512).astype(np.float32) * 50).astype(np.float16)
        ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x)
        assert linear_err(run_linear(uq, torch, w, qw, None, x), ref) <= TOL
        x0 = np.zeros((M, 512), dtype=np.float16)
        assert np.all(run_linear(uq, torch, w, qw, None, x0) == 0)


def test_keep_changes_between_calls_and_determinism(env, uref):
    """The pruning rate is a run-time argument: alternate keeps on the same weights; identical bits on repeats;
    row truncation returns exactly the matching outputs of the unpruned call."""
    uq, torch = env
    rng = wl.rng_for(0, 34)
    w = wl.gen_linear(rng, 1024, 1024)
    qw = uq.QuantLinear.from_numpy(w)
    x = wl.gen_activations(rng, 1, 1024)
    xd = to_dev(torch, x)
    full = uq.uniql_w4_linear(qw, None, xd).cpu().numpy()
    seen = {}
    for rep in range(3):
        for n in (1024, 870, 665, 870, 1024):
            y = uq.uniql_w4_linear(qw, Keep(n_keep=n), xd).cpu().numpy()
            assert np.array_equal(y.view(np.uint16), full[:, :n].view(np.uint16))
            seen.setdefault(n, y)
            assert np.array_equal(seen[n].view(np.uint16), y.view(np.uint16))
    for kk in (870, 665):
        ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], np.ascontiguousarray(x[:, :kk]), Keep(k_keep=kk))
        y = uq.uniql_w4_linear(qw, Keep(k_keep=kk), xd[:, :kk].contiguous()).cpu().numpy()
        assert linear_err(y, ref) <= TOL


def _sample_rows(n, rng, count=192):
    rows = np.unique(np.concatenate([[0, 1, n - 2, n - 1], rng.integers(0, n, count)]))
    return rows.astype(np.int32)


@pytest.mark.parametrize("rate", [0, 15, 35])
def test_llama3_8b_decode_layer_full_size(env, uref, rate):
    """All seven linears of the Llama-3-8B shaped layer at full size, M = 1: EVERY kept row against the oracle
    (element-wise and norm-wise bars), and bitwise repeatability."""
    uq, torch = env
    rng = wl.rng_for(1, rate)
    for spec in wl.llama3_8b_layer(rate):
        w = wl.gen_linear(rng, spec.N, spec.K)
        qw = uq.QuantLinear.from_numpy(w)
        x = wl.gen_activations(rng, 1, spec.k_keep)
        y = run_linear(uq, torch, w, qw, spec.keep, x)
        assert y.shape == (1, spec.n_keep)
        ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, spec.keep)
        assert ref.shape == y.shape
        err = linear_err(y, ref)
        assert err <= TOL, (spec.name, err)
        assert normwise_err(y, ref) <= NORM_TOL, (spec.name, normwise_err(y, ref))
        y2 = run_linear(uq, torch, w, qw, spec.keep, x)
        assert np.array_equal(y.view(np.uint16), y2.view(np.uint16))


@pytest.mark.parametrize("M", [1, 8, 16, 17, 32, 33, 64, 65, 128])
def test_qwen25_7b_shapes(env, uref, M):
    """Every decode-batch configuration (up to 16, 32 and 64 tokens; tall and short matrices; column segments in
    o_proj) and the small prefill tiles, at the model's sizes: sampled rows of every token."""
    uq, torch = env
    rng = wl.rng_for(2, M)
    for spec in wl.qwen25_7b_layer(25):
        if spec.name in ("up_proj", "v_proj"):
            continue
        w = wl.gen_linear(rng, spec.N, spec.K)
        qw = uq.QuantLinear.from_numpy(w)
        x = wl.gen_activations(rng, M, spec.k_keep)
        y = run_linear(uq, torch, w, qw, spec.keep, x)
        rows = _sample_rows(spec.n_keep, rng, 96)
        ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, spec.keep, rows=rows)
        rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
        err = np.max(np.abs(y[:, rows].astype(np.float64) - ref) / np.maximum(np.abs(ref), 1e-2 * rms))
        assert err <= TOL, (spec.name, err)


@pytest.mark.parametrize("M", [2, 8, 12, 16])
def test_qwen25_7b_decode_batch_in_one_call(env, uref, M):
    """q + k + v and gate + up of a Qwen2.5-7B decode batch through uniql_w4_linear_multi at the model's sizes (one
    launch of the decode-batch kernel per call; gate / up with the activations staged once per block): sampled rows of
    every token against the oracle, and the bits of single calls."""
    uq, torch = env
    rng = wl.rng_for(2, 300 + M)
    specs = {s.name: s for s in wl.qwen25_7b_layer(25)}
    for names in (("q_proj", "k_proj", "v_proj"), ("gate_proj", "up_proj")):
        ws = [wl.gen_linear(rng, specs[n].N, specs[n].K) for n in names]
        qws = [uq.QuantLinear.from_numpy(w) for w in ws]
        keeps = [specs[n].keep for n in names]
        x = wl.gen_activations(rng, M, specs[names[0]].k_keep)
        xd = to_dev(torch, x)
        ys = [torch.full((M, specs[n].n_keep), 9.0, dtype=torch.float16, device="cuda") for n in names]
        uq.uniql_w4_linear_multi(qws, keeps, [xd] * len(names), ys)
        torch.cuda.synchronize()
        for n, w, qw, kp, y in zip(names, ws, qws, keeps, ys):
            assert torch.equal(uq.uniql_w4_linear(qw, kp, xd), y), n
            rows = _sample_rows(specs[n].n_keep, rng, 64)
            ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, kp, rows=rows)
            rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
            got = y.cpu().numpy().astype(np.float64)[:, rows]
            assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms)) <= TOL, n


def test_mamba2_shapes(env, uref):
    uq, torch = env
    rng = wl.rng_for(3)
    for spec in wl.mamba2_2p7b_layer(15):
        w = wl.gen_linear(rng, spec.N, spec.K)
        qw = uq.QuantLinear.from_numpy(w)
        x = wl.gen_activations(rng, 1, spec.k_keep)
        y = run_linear(uq, torch, w, qw, spec.keep, x)
        rows = _sample_rows(spec.n_keep, rng, 128)
        if spec.name == "in_proj":      # include the segment boundaries and the whole tail
            rows = np.unique(np.concatenate([rows, [4351, 4352, 8703, 8704, 9039]])).astype(np.int32)
        ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, spec.keep, rows=rows)
        rms = np.sqrt(np.mean(ref ** 2))
        err = np.max(np.abs(y[:, rows].astype(np.float64) - ref) / np.maximum(np.abs(ref), 1e-2 * rms))
        assert err <= TOL, (spec.name, err)


@pytest.mark.parametrize("M", [1, 8])
def test_mamba2_head_and_state_dimension_pruned(env, uref, M):
    """in_proj with the 80 heads of z and x cut to 54 of 64 channels and the B and C parts to 108 of 128
    state channels (second family of row segments), out_proj with the matching per-head columns."""
    uq, torch = env
    rng = wl.rng_for(3, 5)
    for spec in wl.mamba2_2p7b_layer_heads_and_state(15):
        w = wl.gen_linear(rng, spec.N, spec.K)
        qw = uq.QuantLinear.from_numpy(w)
        assert uq.kept_dims(qw, spec.keep) == uref.count_kept(spec.N, spec.K, spec.keep) == (spec.n_keep, spec.k_keep)
        x = wl.gen_activations(rng, M, spec.k_keep)
        y = run_linear(uq, torch, w, qw, spec.keep, x)
        rows = _sample_rows(spec.n_keep, rng, 128)
        if spec.name == "in_proj":      # every zone boundary: z | x | B | C | dt in compact rows
            zx, s = 2 * 80 * 54, 108
            edges = [53, 54, zx - 1, zx, zx + s - 1, zx + s, zx + 2 * s - 1, zx + 2 * s, spec.n_keep - 1]
            rows = np.unique(np.concatenate([rows, edges])).astype(np.int32)
        ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, spec.keep, rows=rows)
        assert linear_err(y[:, rows], ref) <= TOL, spec.name
        if M == 1:
            d = uq.uniql_w4_dequant(qw, spec.keep)
            torch.cuda.synchronize()
            assert np.array_equal(d.cpu().numpy().view(np.uint16),
                                  uref.w4_dequant(w["qweight"], w["scales"], w["zeros"], spec.keep).view(np.uint16))


@pytest.mark.parametrize("seed", range(12))
def test_linear_random_two_segment_families(env, uref, seed):
    """Seeded random two-family row rules (either family may be empty, the tail may be empty) at
    token counts that reach the GEMV with one, two and four rows per wave and the MFMA kernels."""
    uq, torch = env
    rng = wl.rng_for(12, seed)
    s1 = int(rng.choice([8, 24, 64, 100])); k1 = int(rng.integers(1, s1 + 1)); n1 = int(rng.integers(0, 40))
    s2 = int(rng.choice([8, 16, 128])); k2 = int(rng.integers(1, s2 + 1)); n2 = int(rng.integers(0, 6))
    tail = int(rng.integers(0, 90))
    N = max(1, n1 * s1 + n2 * s2 + tail)
    if n1 * s1 + n2 * s2 + tail == 0:
        tail = 1
    keep = Keep(n_keep=n1 * k1 + n2 * k2 + tail, row_seg_stride=s1, row_seg_keep=k1, row_seg_limit=n1 * s1,
                row_seg2_stride=s2, row_seg2_keep=k2, row_seg2_limit=n1 * s1 + n2 * s2)
    K = 128 * int(rng.choice([1, 4, 8, 20]))
    M = int(rng.choice([1, 1, 1, 5, 16, 70]))
    w = wl.gen_linear(rng, N, K)
    qw = uq.QuantLinear.from_numpy(w)
    x = wl.gen_activations(rng, M, K)
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    y = run_linear(uq, torch, w, qw, keep, x)
    assert y.shape == ref.shape and linear_err(y, ref) <= TOL, (N, K, M, keep)


@pytest.mark.parametrize("M", [256, 1024, 4096])
def test_prefill_gemm_sampled(env, uref, M):
    """Prefill-sized dequant-GEMM at the gate/up and down shapes, 15 % pruning, up to the 4096 tokens every prefill
    figure is quoted on: sampled (token, row) pairs that include the first and last token / row of the matrix and
    the edges of the first and last 128 x 256 tiles."""
    uq, torch = env
    rng = wl.rng_for(4, M)
    for spec in wl.prefill_linears(15):
        w = wl.gen_linear(rng, spec.N, spec.K)
        qw = uq.QuantLinear.from_numpy(w)
        x = wl.gen_activations(rng, M, spec.k_keep)
        y = run_linear(uq, torch, w, qw, spec.keep, x)
        toks = np.unique(np.concatenate([[0, 127, 128, 255, M - 257, M - 256, M - 129, M - 128, M - 1], rng.integers(0, M, 6)]))
        rows = np.unique(np.concatenate([_sample_rows(spec.n_keep, rng, 64),
                                         [255, 256, spec.n_keep - spec.n_keep % 256 - 1, spec.n_keep - spec.n_keep % 256]]))
        rows = rows[(rows >= 0) & (rows < spec.n_keep)].astype(np.int32)
        ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], np.ascontiguousarray(x[toks]), spec.keep, rows=rows)
        rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
        got = y[np.ix_(toks, rows)].astype(np.float64)
        err = np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms))
        assert err <= TOL, (spec.name, err)
        assert normwise_err(y[np.ix_(toks, rows)], ref) <= NORM_TOL, spec.name


def test_prefill_persistent_kernel_without_zero_points_and_strided(env, uref):
    """The 256 x 256 persistent prefill kernel on a matrix without zero points, x and y with row strides larger than
    their widths (odd ones), sampled against the oracle; nothing is written between the rows of y."""
    uq, torch = env
    rng = wl.rng_for(4, 777)
    N, K, M = 12288, 1024, 1030
    keep = Keep(n_keep=12285, k_keep=1003)
    w = wl.gen_linear(rng, N, K)
    w["zeros"] = None
    qw = uq.QuantLinear.from_numpy(w)
    x = wl.gen_activations(rng, M, 1003)
    xd = torch.zeros((M, 1003 + 19), dtype=torch.float16, device="cuda")
    xd[:, :1003] = to_dev(torch, x)
    yd = torch.full((M, 12285 + 7), 3.0, dtype=torch.float16, device="cuda")
    uq.uniql_w4_linear(qw, keep, xd[:, :1003], yd[:, :12285])
    y = yd.cpu().numpy()
    assert np.all(y[:, 12285:] == 3.0)
    toks = np.unique(np.concatenate([[0, 255, 256, 1023, 1024, M - 1], rng.integers(0, M, 6)]))
    rows = np.unique(np.concatenate([_sample_rows(12285, rng, 96), [255, 256, 12031, 12032, 12283, 12284]])).astype(np.int32)
    ref = uref.w4_linear(w["qweight"], w["scales"], None, np.ascontiguousarray(x[toks]), keep, rows=rows)
    rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
    got = y[np.ix_(toks, rows)].astype(np.float64)
    assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms)) <= TOL


def test_lm_head_sized_gemv_sampled(env, uref):
    """The output-head shape (128256 x 4096, unpruned), M = 1: sampled rows against the oracle."""
    uq, torch = env
    spec = wl.lm_head_llama3()
    rng = wl.rng_for(5, 1)
    w = wl.gen_linear(rng, spec.N, spec.K)
    x = wl.gen_activations(rng, 1, spec.K)
    y = run_linear(uq, torch, w, uq.QuantLinear.from_numpy(w), spec.keep, x)
    rows = _sample_rows(spec.N, rng, 256)
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, spec.keep, rows=rows)
    rms = np.sqrt(np.mean(ref ** 2))
    err = np.max(np.abs(y[:, rows].astype(np.float64) - ref) / np.maximum(np.abs(ref), 1e-2 * rms))
    assert err <= TOL, err


@pytest.mark.parametrize("N,K,keep,M", [
    (6144, 2176, Keep(n_keep=6100, k_keep=2049), 1000),    # ragged rows, tokens and K tail; one column into a group
    (6144, 1152, Keep(k_keep=1100), 1024),                 # 9 groups per row: the last set of scales starts early
    (6400, 1024, Keep(n_keep=6200, row_seg_stride=128, row_seg_keep=124, row_seg_limit=6400), 1024),   # row segments
    (3072, 1280, Keep(k_keep=1279), 500),                  # 64 x 128 tiles with K split over two waves
    (6144, 1024, Keep(k_keep=1000), 500),                  # 64 x 256 tiles
    (512, 2048, Keep(), 130),
    (12300, 1152, Keep(n_keep=12200, k_keep=1100), 1000),  # 256 x 256 tiles on the persistent grid: ragged rows, tokens, K tail
    (12288, 1024, Keep(k_keep=1017), 4096),                # ... three tiles per block, a column tail of one
    (4096, 2176, Keep(k_keep=2049), 4000),                 # ... one tile per block, the last token tile ragged
    (12800, 1024, Keep(n_keep=12400, row_seg_stride=128, row_seg_keep=124, row_seg_limit=12800), 1024),   # ... row segments
])
def test_prefill_tiles_ragged(env, uref, N, K, keep, M):
    """The prefill tile configurations (128 x 256 hand-scheduled kernel when the grid fills the chip, smaller
    tiles otherwise) on shapes with ragged row / token / column tails: sampled (token, row) pairs."""
    uq, torch = env
    rng = wl.rng_for(4, N + K + M)
    w = wl.gen_linear(rng, N, K)
    qw = uq.QuantLinear.from_numpy(w)
    nk, kk = uq.kept_dims(qw, keep)
    x = wl.gen_activations(rng, M, kk)
    y = run_linear(uq, torch, w, qw, keep, x)
    toks = np.unique(np.concatenate([[0, 63, 64, 127, 128, min(255, M - 1), min(256, M - 1), M - M % 256 - 1, M - 1], rng.integers(0, M, 6)]))
    rows = _sample_rows(nk, rng, 96)
    rows = np.unique(np.concatenate([rows, [255, 256, min(nk - 1, 4095), nk - nk % 256 - 1, nk - 1]])).astype(np.int32)
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], np.ascontiguousarray(x[toks]), keep, rows=rows)
    rms = np.sqrt(np.mean(ref ** 2, axis=-1, keepdims=True))
    got = y[np.ix_(toks, rows)].astype(np.float64)
    err = np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms))
    assert err <= TOL, err


def _random_keep(rng, N, K):
    """A random valid keep rule for an N x K matrix: prefixes or uniform segments on either side."""
    kw = {}
    mode = rng.integers(0, 4)
    if mode == 1:
        kw["n_keep"] = int(rng.integers(1, N + 1))
    elif mode >= 2 and N >= 8:
        stride = int(rng.choice([d for d in (8, 16, 32, 64, 128) if d <= N]))
        limit = (int(rng.integers(1, N // stride + 1))) * stride
        kw.update(row_seg_stride=stride, row_seg_keep=int(rng.integers(1, stride + 1)), row_seg_limit=limit)
    mode = rng.integers(0, 4)
    if mode == 1:
        kw["k_keep"] = int(rng.integers(1, K + 1))
    elif mode >= 2:
        stride = int(rng.choice([d for d in (8, 16, 32, 64, 128, 256) if K % d == 0]))
        kw.update(col_seg_stride=stride, col_seg_keep=int(rng.integers(1, stride + 1)))
    return Keep(**kw)


@pytest.mark.parametrize("seed", range(24))
def test_linear_random_shapes(env, uref, seed):
    """Seeded random shapes, keep rules and token counts through every kernel selection (GEMV, K-split
    decode batches, all prefill tiles), each against the full oracle output."""
    uq, torch = env
    rng = wl.rng_for(6, seed)
    K = 128 * int(rng.choice([1, 2, 3, 4, 7, 8, 9, 12, 16, 17, 24, 32]))
    N = int(rng.choice([1, 5, 16, 17, 48, 100, 256, 300, 513, 700]))
    M = int(rng.choice([1, 1, 2, 7, 16, 17, 33, 64, 65, 130, 257]))
    keep = _random_keep(rng, N, K)
    w = wl.gen_linear(rng, N, K)
    qw = uq.QuantLinear.from_numpy(w)
    nk, kk = uq.kept_dims(qw, keep)
    x = wl.gen_activations(rng, M, kk)
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    y = run_linear(uq, torch, w, qw, keep, x, pad=int(rng.integers(0, 4)))
    assert y.shape == (M, nk)
    assert linear_err(y, ref) <= TOL, (N, K, M, keep)


# --------------------------------------------------------------------- RoPE
def run_rope(uq, torch, r, spec):
    q = to_dev(torch, r["q"])
    k = to_dev(torch, r["k"]) if r["k"] is not None else None
    uq.uniql_pruned_rope(q, k, to_dev(torch, r["positions"]), to_dev(torch, r["kept_idx"]), spec.D_full, spec.theta)
    torch.cuda.synchronize()
    return q.cpu().numpy(), (k.cpu().numpy() if k is not None else None)


@pytest.mark.parametrize("spec", [
    wl.small_rope(),
    wl.llama3_8b_rope(0), wl.llama3_8b_rope(15), wl.llama3_8b_rope(35),
    wl.qwen25_7b_rope(25, T=16),
    wl.llama3_8b_rope(15, T=37),
    wl.RopeSpec(T=3, Hq=4, Hkv=4, H_tab=4, D_full=64, D_keep=2, theta=1e4, pos_max=100),
    wl.RopeSpec(T=5, Hq=6, Hkv=2, H_tab=1, D_full=256, D_keep=200, theta=1e6, pos_max=32768),
    wl.RopeSpec(T=2, Hq=2, Hkv=0, H_tab=2, D_full=1024, D_keep=700, theta=1e4, pos_max=32768),
], ids=lambda s: f"T{s.T}_H{s.Hq}-{s.Hkv}-{s.H_tab}_D{s.D_full}-{s.D_keep}")
def test_rope_parity(env, uref, spec):
    uq, torch = env
    r = wl.gen_rope_inputs(wl.rng_for(1, 40), spec)
    qo, ko = uref.pruned_rope(r["q"], r["k"], r["positions"], r["kept_idx"], spec.D_full, spec.theta)
    gq, gk = run_rope(uq, torch, r, spec)
    assert rope_err(gq, qo) <= TOL
    if ko is not None:
        assert rope_err(gk, ko) <= TOL
    # pair norms survive up to fp16 rounding
    hk = spec.D_keep // 2
    n_in = r["q"].astype(np.float64)[..., :hk] ** 2 + r["q"].astype(np.float64)[..., hk:] ** 2
    n_out = gq.astype(np.float64)[..., :hk] ** 2 + gq.astype(np.float64)[..., hk:] ** 2
    assert np.max(np.abs(n_in - n_out) / np.maximum(n_in, 1e-3)) < 4e-3


@pytest.mark.parametrize("seed", range(16))
def test_rope_random_shapes(env, uref, seed):
    """Seeded random head counts, table rows, head dimensions (odd and even pair counts), token counts that
    span one item per thread, one batch and several batches, with and without K."""
    uq, torch = env
    rng = wl.rng_for(7, seed)
    H_tab = int(rng.choice([1, 2, 4, 8]))
    Hkv = H_tab * int(rng.choice([0, 1, 2]))
    Hq = H_tab * int(rng.choice([1, 2, 4, 7]))
    D_full = int(rng.choice([8, 32, 64, 128, 256]))
    D_keep = 2 * int(rng.integers(1, D_full // 2 + 1))
    T = int(rng.choice([1, 2, 3, 9, 40, 97, 300]))
    spec = wl.RopeSpec(T=T, Hq=Hq, Hkv=Hkv, H_tab=H_tab, D_full=D_full, D_keep=D_keep,
                       theta=float(rng.choice([1.0e4, 5.0e5, 1.0e6])), pos_max=int(rng.choice([64, 4096, 131072])))
    r = wl.gen_rope_inputs(rng, spec)
    qo, ko = uref.pruned_rope(r["q"], r["k"], r["positions"], r["kept_idx"], spec.D_full, spec.theta)
    gq, gk = run_rope(uq, torch, r, spec)
    assert rope_err(gq, qo) <= TOL, spec
    if ko is not None:
        assert rope_err(gk, ko) <= TOL, spec


def test_rope_prefill_full_size(env, uref):
    """[4096 tokens, 32 Q + 8 KV heads, 108 of 128 dims], positions 0..4095: every element against the oracle."""
    uq, torch = env
    spec = wl.prefill_rope(15, T=4096)
    r = wl.gen_rope_inputs(wl.rng_for(4, 41), spec)
    qo, ko = uref.pruned_rope(r["q"], r["k"], r["positions"], r["kept_idx"], spec.D_full, spec.theta)
    gq, gk = run_rope(uq, torch, r, spec)
    assert rope_err(gq, qo) <= TOL and rope_err(gk, ko) <= TOL
    gq2, gk2 = run_rope(uq, torch, r, spec)
    assert np.array_equal(gq.view(np.uint16), gq2.view(np.uint16))


def test_rope_position_zero_and_identity_table(env, uref):
    uq, torch = env
    spec = wl.RopeSpec(T=4, Hq=8, Hkv=2, H_tab=2, D_full=128, D_keep=128, theta=5e5, pos_max=1)
    r = wl.gen_rope_inputs(wl.rng_for(1, 42), spec)
    gq, gk = run_rope(uq, torch, r, spec)          # all positions are 0: the identity
    assert np.array_equal(gq.view(np.uint16), r["q"].view(np.uint16))
    assert np.array_equal(gk.view(np.uint16), r["k"].view(np.uint16))


# ------------------------------------------------------- several linears per call
@pytest.mark.parametrize("rate", [0, 15, 35])
def test_multi_call_matches_single_calls(env, uref, rate):
    """q/k/v and gate/up of the Llama-3-8B shaped layer through uniql_w4_linear_multi (one launch at
    M = 1): bit-identical to separate calls, and within tolerance of the oracle on sampled rows."""
    uq, torch = env
    rng = wl.rng_for(1, 50 + rate)
    specs = {s.name: s for s in wl.llama3_8b_layer(rate)}
    for names in (("q_proj", "k_proj", "v_proj"), ("gate_proj", "up_proj")):
        ws = [wl.gen_linear(rng, specs[n].N, specs[n].K) for n in names]
        qws = [uq.QuantLinear.from_numpy(w) for w in ws]
        x = wl.gen_activations(rng, 1, specs[names[0]].k_keep)
        xd = to_dev(torch, x)
        ys = [torch.full((1, specs[n].n_keep), 3.0, dtype=torch.float16, device="cuda") for n in names]
        uq.uniql_w4_linear_multi(qws, [specs[n].keep for n in names], [xd] * len(names), ys)
        torch.cuda.synchronize()
        for n, w, qw, y in zip(names, ws, qws, ys):
            single = uq.uniql_w4_linear(qw, specs[n].keep, xd).cpu().numpy()
            got = y.cpu().numpy()
            assert np.array_equal(got.view(np.uint16), single.view(np.uint16)), n
            rows = _sample_rows(specs[n].n_keep, rng, 64)
            ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, specs[n].keep, rows=rows)
            rms = np.sqrt(np.mean(ref ** 2))
            err = np.max(np.abs(got[:, rows].astype(np.float64) - ref) / np.maximum(np.abs(ref), 1e-2 * rms))
            assert err <= TOL, (n, err)


def test_multi_call_mixed_shapes_and_tokens(env, uref):
    """Entries that cannot share a launch (different row lengths, or M > 1) still give the single-call results."""
    uq, torch = env
    rng = wl.rng_for(0, 60)
    shapes = [(300, 1024, Keep(n_keep=257)), (64, 4096, Keep(k_keep=3000)), (128, 256, Keep())]
    for M in (1, 3):
        ws = [wl.gen_linear(rng, N, K) for N, K, _ in shapes]
        qws = [uq.QuantLinear.from_numpy(w) for w in ws]
        xs = [to_dev(torch, wl.gen_activations(rng, M, uq.kept_dims(qw, kp)[1])) for qw, (_, _, kp) in zip(qws, shapes)]
        ys = [torch.zeros((M, uq.kept_dims(qw, kp)[0]), dtype=torch.float16, device="cuda") for qw, (_, _, kp) in zip(qws, shapes)]
        uq.uniql_w4_linear_multi(qws, [kp for _, _, kp in shapes], xs, ys)
        for qw, (_, _, kp), x, y in zip(qws, shapes, xs, ys):
            single = uq.uniql_w4_linear(qw, kp, x)
            assert torch.equal(single, y)


@pytest.mark.parametrize("M", [2, 4, 7, 8, 16, 31])
def test_multi_call_decode_batches_share_a_launch(env, uref, M):
    """q / k / v (row segments, GQA sizes) and gate / up (row prefix) of a decode batch through uniql_w4_linear_multi:
    2..32 tokens with column prefixes go out as ONE launch of the decode-batch kernel; the bits of separate calls, the
    oracle on sampled rows, padding of strided outputs untouched.  A member the kernel does not take (fewer than 8
    groups per row) sends the whole call down the one-by-one path with the same results."""
    uq, torch = env
    rng = wl.rng_for(0, 70 + M)
    hidden = 2048
    sets = [
        [(2048, hidden, Keep(n_keep=16 * 108, k_keep=1741, row_seg_stride=64, row_seg_keep=54, row_seg_limit=2048)),
         (512, hidden, Keep(n_keep=4 * 108, k_keep=1741, row_seg_stride=64, row_seg_keep=54, row_seg_limit=512)),
         (512, hidden, Keep(n_keep=4 * 108, k_keep=1741, row_seg_stride=128, row_seg_keep=108, row_seg_limit=512))],
        [(5632, hidden, Keep(n_keep=4787)), (5632, hidden, Keep(n_keep=4787))],
        [(300, 1024, Keep(n_keep=257)), (64, 4096, Keep(k_keep=3001)), (128, 256, Keep()), (48, 1024, Keep(k_keep=9))],
    ]
    for shapes in sets:
        ws = [wl.gen_linear(rng, N, K) for N, K, _ in shapes]
        qws = [uq.QuantLinear.from_numpy(w) for w in ws]
        dims = [uq.kept_dims(qw, kp) for qw, (_, _, kp) in zip(qws, shapes)]
        xs_h = [wl.gen_activations(rng, M, kk) for _, kk in dims]
        xs = [to_dev(torch, x) for x in xs_h]
        ybufs = [torch.full((M, nk + 5), -7.0, dtype=torch.float16, device="cuda") for nk, _ in dims]
        ys = [yb[:, :nk] for yb, (nk, _) in zip(ybufs, dims)]
        uq.uniql_w4_linear_multi(qws, [kp for _, _, kp in shapes], xs, ys)
        torch.cuda.synchronize()
        for w, qw, (_, _, kp), x, xh, yb, (nk, kk) in zip(ws, qws, shapes, xs, xs_h, ybufs, dims):
            assert torch.all(yb[:, nk:] == -7.0)
            single = uq.uniql_w4_linear(qw, kp, x)
            assert torch.equal(single, yb[:, :nk])
            rows = _sample_rows(nk, rng, 48)
            ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], xh, kp, rows=rows)
            got = yb[:, :nk].cpu().numpy().astype(np.float64)[:, rows]
            rms = np.sqrt(np.mean(ref ** 2))
            assert np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-2 * rms)) <= TOL


# ------------------------------------------------- fused q / k / v projections + rotary embedding
def _qkv_case(uq, torch, uref, specs, rope, rng):
    """One token through uniql_w4_qkv_rope against the oracle's y = RoPE(x W).  The rotation preserves
    norms, so q and k are judged with the metric of the linears (floor 1e-2 * rms of the tensor)."""
    names = ("q_proj", "k_proj", "v_proj")
    ws = [wl.gen_linear(rng, specs[n].N, specs[n].K) for n in names]
    qws = [uq.QuantLinear.from_numpy(w) for w in ws]
    keeps = [specs[n].keep for n in names]
    x = wl.gen_activations(rng, 1, specs["q_proj"].k_keep)
    r = wl.gen_rope_inputs(rng, rope)
    pos, idx = r["positions"][:1].copy(), r["kept_idx"]
    xd = to_dev(torch, x[0])
    q, k, v = uq.uniql_w4_qkv_rope(qws, keeps, xd, to_dev(torch, pos), to_dev(torch, idx), rope.Hq, rope.Hkv,
                                   rope.D_full, rope.D_keep, rope.theta)
    torch.cuda.synchronize()
    rq, rk, rv = uref.qkv_rope(ws[0], keeps[0], ws[1], keeps[1], ws[2], keeps[2], x, pos, idx, rope.Hq, rope.Hkv,
                               rope.D_full, rope.D_keep, rope.theta)
    # One launch (rotation of the fp32 sums) needs rows of a multiple of four groups and at most 16384
    # columns; otherwise the entry point runs the separate kernels, which round q and k to fp16 before
    # rotating: an extra error of up to 2^-11 of each member of the pair, so the floor is the pair's norm.
    one_launch = (specs["q_proj"].K // 128) % 4 == 0 and specs["q_proj"].k_keep <= 16384

    def qk_err(got, ref):
        if one_launch:
            return linear_err(got.cpu().numpy().reshape(1, -1), ref.reshape(1, -1))
        hk = rope.D_keep // 2
        pn = np.sqrt(ref[..., :hk] ** 2 + ref[..., hk:] ** 2)
        pn = np.concatenate([pn, pn], axis=-1)
        den = np.maximum(np.maximum(np.abs(ref), pn), 1e-2 * np.sqrt(np.mean(ref ** 2)))
        return float(np.max(np.abs(got.cpu().numpy().astype(np.float64).reshape(ref.shape) - ref) / den))

    errs = (qk_err(q, rq), qk_err(k, rk), linear_err(v.cpu().numpy().reshape(1, -1), rv.reshape(1, -1)))
    # a second call returns the same bits
    q2, k2, v2 = uq.uniql_w4_qkv_rope(qws, keeps, xd, to_dev(torch, pos), to_dev(torch, idx), rope.Hq, rope.Hkv,
                                      rope.D_full, rope.D_keep, rope.theta)
    assert torch.equal(q, q2) and torch.equal(k, k2) and torch.equal(v, v2)
    # The separate calls round q and k to fp16 before rotating them, an error of up to 2^-11 of each
    # member of a pair, so they are compared with the fused result relative to the pair's norm.
    ys = [torch.empty((1, specs[n].n_keep), dtype=torch.float16, device="cuda") for n in names]
    uq.uniql_w4_linear_multi(qws, keeps, [xd.view(1, -1)] * 3, ys)
    qs, ks = ys[0].view(1, rope.Hq, rope.D_keep), ys[1].view(1, rope.Hkv, rope.D_keep)
    uq.uniql_pruned_rope(qs, ks, to_dev(torch, pos), to_dev(torch, idx), rope.D_full, rope.theta)
    torch.cuda.synchronize()
    assert torch.equal(ys[2].view(-1), v)
    sep = []
    for fused_t, sep_t, ref in ((q, qs, rq), (k, ks, rk)):
        hk = rope.D_keep // 2
        pn = np.sqrt(ref[..., :hk] ** 2 + ref[..., hk:] ** 2)
        pn = np.concatenate([pn, pn], axis=-1)
        floor = 1e-2 * np.sqrt(np.mean(ref ** 2))
        d = np.abs(fused_t.cpu().numpy().astype(np.float64).reshape(ref.shape) - sep_t.cpu().numpy().astype(np.float64).reshape(ref.shape))
        sep.append(float(np.max(d / np.maximum(pn, floor))))
    return errs, tuple(sep)


@pytest.mark.parametrize("rate", [0, 15, 35])
def test_fused_qkv_rope_llama3_8b(env, uref, rate):
    uq, torch = env
    specs = {s.name: s for s in wl.llama3_8b_layer(rate)}
    errs, sep = _qkv_case(uq, torch, uref, specs, wl.llama3_8b_rope(rate, T=1), wl.rng_for(1, 70 + rate))
    assert max(errs) <= TOL and max(sep) <= 2e-3, (errs, sep)


def test_fused_qkv_rope_qwen25_7b(env, uref):
    uq, torch = env
    specs = {s.name: s for s in wl.qwen25_7b_layer(25)}
    errs, sep = _qkv_case(uq, torch, uref, specs, wl.qwen25_7b_rope(25, T=1), wl.rng_for(2, 71))
    assert max(errs) <= TOL and max(sep) <= 2e-3, (errs, sep)


@pytest.mark.parametrize("hidden", [256, 512, 2176])
def test_fused_qkv_rope_small_blocks(env, uref, hidden):
    """Small attention blocks: 512 columns run fused; 256 (two groups per row) and 2176 (17 groups) take the
    path of separate launches inside the same entry point."""
    uq, torch = env
    Hq, Hkv, D, Dk = 6, 2, 64, 50
    hk = Dk // 2
    specs = {
        "q_proj": wl.LinearSpec("q_proj", K=hidden, N=Hq * D, keep=Keep(n_keep=Hq * Dk, row_seg_stride=D // 2, row_seg_keep=hk, row_seg_limit=Hq * D)),
        "k_proj": wl.LinearSpec("k_proj", K=hidden, N=Hkv * D, keep=Keep(n_keep=Hkv * Dk, row_seg_stride=D // 2, row_seg_keep=hk, row_seg_limit=Hkv * D)),
        "v_proj": wl.LinearSpec("v_proj", K=hidden, N=Hkv * D, keep=Keep(n_keep=Hkv * Dk, row_seg_stride=D, row_seg_keep=Dk, row_seg_limit=Hkv * D)),
    }
    rope = wl.RopeSpec(T=1, Hq=Hq, Hkv=Hkv, H_tab=Hkv, D_full=D, D_keep=Dk, theta=1.0e4, pos_max=4096)
    errs, sep = _qkv_case(uq, torch, uref, specs, rope, wl.rng_for(0, 72 + hidden))
    assert max(errs) <= TOL and max(sep) <= 2e-3, (errs, sep)


@pytest.mark.parametrize("case", ["whole_head_segments", "three_tiles_per_row", "one_tile_per_row", "shared_table_row"])
def test_fused_qkv_rope_walk_shapes(env, uref, case):
    """Attention blocks large enough for the persistent walk (a wave owns the two rows of a rotation pair), in the row
    rules it takes: the leading rows of every head, the leading pairs of either half of every head, a row prefix; one
    to three tiles per row; several heads and all heads per row of the kept-pair table."""
    uq, torch = env
    if case == "whole_head_segments":     # q and k keep the leading D_keep rows of every head (x1 block, then x2 block)
        Hq, Hkv, H_tab, D, Dk, hidden = 24, 8, 8, 128, 100, 2048
        seg = lambda H: Keep(n_keep=H * Dk, row_seg_stride=D, row_seg_keep=Dk, row_seg_limit=H * D)
        keeps = (seg(Hq), seg(Hkv), seg(Hkv))
    elif case == "three_tiles_per_row":   # 6144 columns, of which a prefix is kept
        Hq, Hkv, H_tab, D, Dk, hidden = 16, 4, 4, 128, 128, 6144
        keeps = (Keep(k_keep=5000), Keep(k_keep=5000), Keep(k_keep=5000))
    elif case == "one_tile_per_row":
        Hq, Hkv, H_tab, D, Dk, hidden = 40, 8, 8, 64, 52, 1024
        half = lambda H: Keep(n_keep=H * Dk, row_seg_stride=D // 2, row_seg_keep=Dk // 2, row_seg_limit=H * D)
        keeps = (half(Hq), half(Hkv), Keep(n_keep=Hkv * Dk, row_seg_stride=D, row_seg_keep=Dk, row_seg_limit=Hkv * D))
    else:                                  # one table row for all heads, v a row prefix
        Hq, Hkv, H_tab, D, Dk, hidden = 28, 4, 1, 128, 96, 3584
        half = lambda H: Keep(n_keep=H * Dk, row_seg_stride=D // 2, row_seg_keep=Dk // 2, row_seg_limit=H * D)
        keeps = (half(Hq), half(Hkv), Keep(n_keep=Hkv * Dk))
    specs = {
        "q_proj": wl.LinearSpec("q_proj", K=hidden, N=Hq * D, keep=keeps[0]),
        "k_proj": wl.LinearSpec("k_proj", K=hidden, N=Hkv * D, keep=keeps[1]),
        "v_proj": wl.LinearSpec("v_proj", K=hidden, N=Hkv * D, keep=keeps[2]),
    }
    rope = wl.RopeSpec(T=1, Hq=Hq, Hkv=Hkv, H_tab=H_tab, D_full=D, D_keep=Dk, theta=5.0e5, pos_max=100000)
    errs, sep = _qkv_case(uq, torch, uref, specs, rope, wl.rng_for(0, 90 + len(case)))
    assert max(errs) <= TOL and max(sep) <= 2e-3, (errs, sep)


# ------------------------------------------------- gated MLP hidden vector: SiLU(x W_gate) * (x W_up)
@pytest.mark.parametrize("N,K,keep", [
    (14336, 4096, Keep(n_keep=12185)),     # Llama-3-8B gate / up at 15 %: four rows per wave
    (14336, 4096, Keep(n_keep=9318)),      # 35 %
    (18944, 3584, Keep(n_keep=14208)),     # Qwen2.5-7B at 25 %
    (4000, 1024, Keep(n_keep=3333)),       # two rows per wave
    (1030, 512, Keep()),                   # one row per wave, ragged last block
    (300, 2048, Keep(n_keep=7, k_keep=1500)),   # column prefix as well
    (512, 1024, Keep(k_keep=8 * 108, col_seg_stride=128, col_seg_keep=108)),   # column segments
])
def test_gate_up_silu(env, uref, N, K, keep):
    uq, torch = env
    rng = wl.rng_for(8, N + K)
    wg, wu = wl.gen_linear(rng, N, K), wl.gen_linear(rng, N, K)
    qg, qu = uq.QuantLinear.from_numpy(wg), uq.QuantLinear.from_numpy(wu)
    nk, kk = uq.kept_dims(qg, keep)
    x = wl.gen_activations(rng, 1, kk)
    h = uq.uniql_w4_gate_up_silu([qg, qu], [keep, keep], to_dev(torch, x[0]))
    h2 = uq.uniql_w4_gate_up_silu([qg, qu], [keep, keep], to_dev(torch, x[0]))
    torch.cuda.synchronize()
    assert torch.equal(h, h2)
    ref = uref.gate_up_silu(wg, keep, wu, keep, x)
    assert h.shape == (nk,)
    assert linear_err(h.cpu().numpy().reshape(1, -1), ref) <= TOL


def test_gate_up_silu_refuses_what_it_cannot_fuse(env, uref):
    uq, torch = env
    rng = wl.rng_for(8, 1)
    # 35 groups per row in three tiles: a quad's three groups would straddle the end of a row
    w = wl.gen_linear(rng, 64, 35 * 128)
    q = uq.QuantLinear.from_numpy(w)
    with pytest.raises(Exception):
        uq.uniql_w4_gate_up_silu([q, q], [None, None], torch.zeros(35 * 128, dtype=torch.float16, device="cuda"))
    # two groups per row (most quads of a tile lie past the row's end) is served, and right
    wg, wu = wl.gen_linear(rng, 64, 256), wl.gen_linear(rng, 64, 256)
    x = wl.gen_activations(rng, 1, 256)
    h = uq.uniql_w4_gate_up_silu([uq.QuantLinear.from_numpy(wg), uq.QuantLinear.from_numpy(wu)], [None, None], to_dev(torch, x[0]))
    ref = uref.gate_up_silu(wg, Keep(), wu, Keep(), x)
    assert linear_err(h.cpu().numpy().reshape(1, -1), ref) <= TOL


# ------------------------------------------------- head-interleaved words (o_proj: pruned head dims are never fetched)
@pytest.mark.parametrize("N,heads,d_keep,sym", [
    (4096, 32, 108, False),      # Llama-3-8B o_proj at 15 %
    (4096, 32, 82, False),       # ... at 35 %: 11 blocks of 8 dims, the last one partly kept
    (4096, 32, 128, True),       # unpruned, no zero points
    (300, 4, 54, False),         # few rows, a quarter tile of words
    (1000, 64, 96, False),       # K = 8192: three tiles
    (77, 8, 1, False),           # one dim per head
    (2050, 16, 127, True),
])
def test_head_interleaved_o_proj(env, uref, N, heads, d_keep, sym):
    """uniql_w4_interleave bit for bit against the oracle's permutation; the dequantised kept sub-matrix of the
    interleaved matrix bit for bit against the oracle (and equal to the plain matrix's); the one-token linear on it,
    every row, against the oracle on the same interleaved words."""
    uq, torch = env
    rng = wl.rng_for(19, N + heads + d_keep)
    K = heads * 128
    w = wl.gen_linear(rng, N, K)
    if sym:
        w["zeros"] = None
    keep = Keep() if d_keep == 128 else Keep(col_seg_stride=128, col_seg_keep=d_keep)
    qw = uq.QuantLinear.from_numpy(w)
    qi = uq.uniql_w4_interleave(qw, heads)
    torch.cuda.synchronize()
    words = qi.qweight.cpu().numpy().view(np.uint32)
    assert np.array_equal(words, uref.w4_interleave(w["qweight"], heads))
    d_gpu = uq.uniql_w4_dequant(qi, keep).cpu().numpy()
    d_ref = uref.w4_dequant(words, w["scales"], w["zeros"], keep, il_heads=heads)
    assert np.array_equal(d_gpu.view(np.uint16), d_ref.view(np.uint16))
    assert np.array_equal(d_gpu.view(np.uint16), uq.uniql_w4_dequant(qw, keep).cpu().numpy().view(np.uint16))
    x = wl.gen_activations(rng, 1, heads * d_keep)
    y = uq.uniql_w4_linear(qi, keep, to_dev(torch, x)).cpu().numpy()
    ref = uref.w4_linear(words, w["scales"], w["zeros"], x, keep, il_heads=heads)
    assert y.shape == ref.shape and linear_err(y, ref) <= TOL
    assert normwise_err(y, ref) <= NORM_TOL
    y2 = uq.uniql_w4_linear(qi, keep, to_dev(torch, x)).cpu().numpy()
    assert np.array_equal(y.view(np.uint16), y2.view(np.uint16))


@pytest.mark.parametrize("N,heads,d_keep,M", [(4096, 32, 108, 2), (4096, 32, 108, 8), (300, 4, 54, 64), (1000, 64, 128, 5)])
def test_head_interleaved_decode_batches(env, uref, N, heads, d_keep, M):
    """2..64 tokens on head-interleaved words (the one-token kernel, a token per grid row), strided x and y: every output
    against the oracle on the same words, and each token's row bit-identical to the one-token call."""
    uq, torch = env
    rng = wl.rng_for(19, N + heads + d_keep + M)
    K = heads * 128
    w = wl.gen_linear(rng, N, K)
    keep = Keep() if d_keep == 128 else Keep(col_seg_stride=128, col_seg_keep=d_keep)
    qi = uq.uniql_w4_interleave(uq.QuantLinear.from_numpy(w), heads)
    words = qi.qweight.cpu().numpy().view(np.uint32)
    kk = heads * d_keep
    x = wl.gen_activations(rng, M, kk)
    xd = torch.zeros((M, kk + 24), dtype=torch.float16, device="cuda")
    xd[:, :kk] = to_dev(torch, x)
    yd = torch.full((M, N + 8), 7.0, dtype=torch.float16, device="cuda")
    uq.uniql_w4_linear(qi, keep, xd[:, :kk], yd[:, :N])
    y = yd.cpu().numpy()
    assert np.all(y[:, N:] == 7.0)                                    # nothing written past a row's outputs
    ref = uref.w4_linear(words, w["scales"], w["zeros"], x, keep, il_heads=heads)
    assert linear_err(y[:, :N], ref) <= TOL and normwise_err(y[:, :N], ref) <= NORM_TOL
    for m in (0, M - 1):
        y1 = uq.uniql_w4_linear(qi, keep, to_dev(torch, x[m:m + 1])).cpu().numpy()
        assert np.array_equal(y1.view(np.uint16), np.ascontiguousarray(y[m:m + 1, :N]).view(np.uint16))


@pytest.mark.parametrize("N,heads", [(4096, 32), (77, 8), (5, 3), (1000, 64)])
def test_deinterleave_bit_exact(env, uref, N, heads):
    """uniql_w4_deinterleave against the oracle's permutation, and the round trip through uniql_w4_interleave; the
    result is the plain matrix: a prompt-sized linear on it equals the oracle on the interleaved words."""
    uq, torch = env
    rng = wl.rng_for(19, 3 * N + heads)
    K = heads * 128
    w = wl.gen_linear(rng, N, K)
    qw = uq.QuantLinear.from_numpy(w)
    qi = uq.uniql_w4_interleave(qw, heads)
    back = uq.uniql_w4_deinterleave(qi)
    torch.cuda.synchronize()
    words_il = qi.qweight.cpu().numpy().view(np.uint32)
    words = back.qweight.cpu().numpy().view(np.uint32)
    assert back.col_interleave == 0
    assert np.array_equal(words, uref.w4_deinterleave(words_il, heads))
    assert np.array_equal(words, w["qweight"])
    if N >= 64:
        keep = Keep(col_seg_stride=128, col_seg_keep=108)
        M = 70
        x = wl.gen_activations(rng, M, heads * 108)
        y = uq.uniql_w4_linear(back, keep, to_dev(torch, x)).cpu().numpy()
        rows = np.unique(rng.integers(0, N, 48)).astype(np.int32)
        ref = uref.w4_linear(words_il, w["scales"], w["zeros"], x, keep, rows=rows, il_heads=heads)
        assert linear_err(y[:, rows], ref) <= TOL


def test_head_interleaved_refusals(env):
    uq, torch = env
    rng = wl.rng_for(19, 1)
    qw = uq.QuantLinear.from_numpy(wl.gen_linear(rng, 64, 1024))
    qi = uq.uniql_w4_interleave(qw, 8)
    x2 = torch.zeros((2, 1024), dtype=torch.float16, device="cuda")
    with pytest.raises(uq.UniqlError):       # at most 64 tokens on interleaved words
        uq.uniql_w4_linear(qi, None, torch.zeros((65, 1024), dtype=torch.float16, device="cuda"))
    with pytest.raises(uq.UniqlError):       # a matrix in column order has nothing to undo
        uq.uniql_w4_deinterleave(qw)
    with pytest.raises(uq.UniqlError):       # kept columns must be the leading dims of every head
        uq.uniql_w4_linear(qi, Keep(k_keep=512), x2[:1, :512].contiguous())
    with pytest.raises(uq.UniqlError):       # an interleaved matrix is not interleaved again
        uq.uniql_w4_interleave(qi, 8)
    with pytest.raises(uq.UniqlError):       # 1024 columns are not 7 heads
        uq.uniql_w4_interleave(qw, 7)
    with pytest.raises(uq.UniqlError):       # 12 heads do not divide 256
        uq.uniql_w4_linear(uq.uniql_w4_interleave(uq.QuantLinear.from_numpy(wl.gen_linear(rng, 8, 1536)), 12), None,
                           torch.zeros((1, 1536), dtype=torch.float16, device="cuda"))


# ------------------------------------------------- the whole gated MLP of one token (Eq. 1)
def _mlp_specs(layer):
    sp = {s.name: s for s in layer}
    return sp["gate_proj"], sp["up_proj"], sp["down_proj"]


@pytest.mark.parametrize("case", ["llama_p0", "llama_p15", "llama_p35", "qwen_p25", "small"])
def test_mlp_one_launch(env, uref, case):
    """uniql_w4_mlp: the hidden vector it leaves in the workspace against the oracle's SiLU(x Wg) * (x Wu) and bit for
    bit against uniql_w4_gate_up_silu; y against the oracle's down projection OF THAT hidden vector (every row) and
    bit for bit against uniql_w4_linear on it.  Two calls in a row on one workspace, the second at another rate."""
    uq, torch = env
    if case == "small":      # shapes the single persistent launch does not serve: two launches through the workspace
        specs = [wl.LinearSpec("gate_proj", 1024, 2048, Keep(n_keep=1700)), wl.LinearSpec("up_proj", 1024, 2048, Keep(n_keep=1700)),
                 wl.LinearSpec("down_proj", 2048, 1024, Keep(k_keep=1700))]
        others = []
    else:
        model, rate = case.split("_p")
        layer_of = wl.llama3_8b_layer if model == "llama" else wl.qwen25_7b_layer
        specs = _mlp_specs(layer_of(int(rate)))
        others = [_mlp_specs(layer_of(35 if model == "llama" else 25))]
    rng = wl.rng_for(16, sum(map(ord, case)))
    ws = [wl.gen_linear(rng, s.N, s.K) for s in specs]
    qws = [uq.QuantLinear.from_numpy(w) for w in ws]
    work = uq.mlp_workspace(specs[0].N)          # large enough for any rate
    for sp3 in [specs] + others:
        g, u, d = sp3
        x = wl.gen_activations(rng, 1, g.k_keep)
        xd = to_dev(torch, x[0])
        y = uq.uniql_w4_mlp(qws, [g.keep, u.keep, d.keep], xd, work)
        torch.cuda.synchronize()
        assert uq.uniql_w4_mlp_status(work) == 0
        h = uq.mlp_hidden(work, g.n_keep, torch.float16).clone()
        h_ref = uref.gate_up_silu(ws[0], g.keep, ws[1], u.keep, x)
        assert linear_err(h.cpu().numpy().reshape(1, -1), h_ref) <= TOL
        h_sep = uq.uniql_w4_gate_up_silu(qws[:2], [g.keep, u.keep], xd)
        assert torch.equal(h, h_sep)
        hn = h.cpu().numpy().reshape(1, -1)
        y_ref = uref.w4_linear(ws[2]["qweight"], ws[2]["scales"], ws[2]["zeros"], hn, d.keep)
        yn = y.cpu().numpy().reshape(1, -1)
        assert yn.shape == y_ref.shape and linear_err(yn, y_ref) <= TOL
        assert normwise_err(yn, y_ref) <= NORM_TOL
        y_sep = uq.uniql_w4_linear(qws[2], d.keep, h.reshape(1, -1))
        assert torch.equal(y.reshape(1, -1), y_sep)
        y2 = uq.uniql_w4_mlp(qws, [g.keep, u.keep, d.keep], xd, work)
        assert torch.equal(y, y2)


def test_mlp_refuses_mismatched_hidden_dimension(env):
    uq, torch = env
    rng = wl.rng_for(16, 1)
    qg = uq.QuantLinear.from_numpy(wl.gen_linear(rng, 512, 256))
    qd = uq.QuantLinear.from_numpy(wl.gen_linear(rng, 256, 512))
    work = uq.mlp_workspace(512)
    x = torch.zeros(256, dtype=torch.float16, device="cuda")
    with pytest.raises(uq.UniqlError):       # down keeps 400 input columns, gate / up keep 500 rows
        uq.uniql_w4_mlp([qg, qg, qd], [Keep(n_keep=500), Keep(n_keep=500), Keep(k_keep=400)], x, work)
    with pytest.raises(uq.UniqlError):       # workspace too small
        uq.uniql_w4_mlp([qg, qg, qd], [None, None, None], x, work[:1024])


# ------------------------------------------------- 4-bit embedding rows gathered by token id
@pytest.mark.parametrize("N,K,n,pad", [(50, 384, 5, 0), (1000, 4096, 300, 8), (3000, 2176, 1, 0), (4096, 14336, 33, 16)])
def test_embedding_gather_bit_exact(env, uref, N, K, n, pad):
    uq, torch = env
    rng = wl.rng_for(9, N + K + n)
    w = wl.gen_linear(rng, N, K)
    ids = rng.integers(0, N, n).astype(np.int32)
    ids[0], ids[-1] = N - 1, 0
    ref = uref.w4_embedding(w["qweight"], w["scales"], w["zeros"], ids)
    buf = torch.full((n, K + pad), -3.0, dtype=torch.float16, device="cuda")
    out = uq.uniql_w4_embedding(uq.QuantLinear.from_numpy(w), to_dev(torch, ids), out=buf[:, :K])
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    # sign of an exact zero under a negative scale is unspecified (scales are positive here anyway)
    assert np.array_equal(got.view(np.uint16), ref.view(np.uint16))
    if pad:
        assert torch.all(buf[:, K:] == -3.0), "wrote past K"


# ------------------------------------------------- on-device repack of the kept channels
def _repack_cases():
    ll = {s.name: s for s in wl.llama3_8b_layer(15)}
    mb = {s.name: s for s in wl.mamba2_2p7b_layer(15)}
    c0 = wl.small_case()
    return [("config0", c0.N, c0.K, c0.keep),
            ("llama_q_proj", ll["q_proj"].N, ll["q_proj"].K, ll["q_proj"].keep),
            ("llama_o_proj", ll["o_proj"].N, ll["o_proj"].K, ll["o_proj"].keep),
            ("llama_gate_proj", ll["gate_proj"].N, ll["gate_proj"].K, ll["gate_proj"].keep),
            ("llama_down_proj", ll["down_proj"].N, ll["down_proj"].K, ll["down_proj"].keep),
            ("mamba_in_proj", mb["in_proj"].N, mb["in_proj"].K, mb["in_proj"].keep),
            ("unpruned_ragged_rows", 77, 384, Keep()),
            ("col_segments_of_groups", 100, 2048, Keep(k_keep=4 * 200, col_seg_stride=512, col_seg_keep=200)),
            ("rows_and_col_prefix", 333, 1152, Keep(n_keep=250, k_keep=515)),
            ("col_prefix_tiny", 9, 512, Keep(k_keep=3))]


@pytest.mark.parametrize("name,N,K,keep", _repack_cases(), ids=[c[0] for c in _repack_cases()])
def test_repack_bit_exact_and_equivalent(env, uref, name, N, K, keep):
    """The compact matrix equals the oracle's bit for bit, and the GEMV on it (with the descriptor of the
    plan) returns what the GEMV returns on the source with the original descriptor."""
    uq, torch = env
    rng = wl.rng_for(10, N + K)
    w = wl.gen_linear(rng, N, K)
    q2, s2, z2, keep2 = uref.w4_repack(w["qweight"], w["scales"], w["zeros"], keep)
    src = uq.QuantLinear.from_numpy(w)
    out, ko = uq.uniql_w4_repack(src, keep)
    torch.cuda.synchronize()
    assert np.array_equal(out.qweight.cpu().numpy().view(np.uint32), q2)
    assert np.array_equal(out.scales.cpu().numpy().view(np.uint16), s2.view(np.uint16))
    assert np.array_equal(out.zeros.cpu().numpy(), z2)
    nk, kk = uref.count_kept(N, K, keep)
    assert uq.kept_dims(out, ko) == (nk, kk)
    x = wl.gen_activations(rng, 1, kk)
    y_src = run_linear(uq, torch, w, src, keep, x)
    y_cmp = run_linear(uq, torch, None, out, ko, x)
    rows = _sample_rows(nk, rng)
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep, rows=rows)
    assert linear_err(y_cmp[:, rows], ref) <= TOL
    # same numbers summed in the same order: a chunk count that shrinks only drops zero terms
    assert np.array_equal(y_src.view(np.uint16), y_cmp.view(np.uint16))


# ------------------------------------------------- matrices without zero points (Eq. 3's symmetric scheme)
def _drop_zeros(w):
    return {"qweight": w["qweight"], "scales": w["scales"], "zeros": None}


@pytest.mark.parametrize("N,K,keep,M", [
    (1024, 1024, Keep(n_keep=870), 1),                    # one row per wave, wide scale loads
    (14336, 4096, Keep(n_keep=12185), 1),                 # two rows per wave
    (20000, 2048, Keep(), 1),                             # four rows per wave, per-tile scale loads
    (640, 1280, Keep(k_keep=1000), 1),                    # ten groups per row: run-time chunk loop
    (4096, 4096, Keep(k_keep=32 * 108, col_seg_stride=128, col_seg_keep=108), 1),
    (3584, 4096, Keep(n_keep=3000, k_keep=4003), 8),      # K split over waves, tail columns in fp32
    (512, 1024, Keep(k_keep=8 * 108, col_seg_stride=128, col_seg_keep=108), 16),
    (1000, 2048, Keep(k_keep=1999), 48),
    (14336, 4096, Keep(n_keep=12185), 1024),              # hand-scheduled prefill kernel
    (4096, 14336, Keep(k_keep=12185), 333),               # prefill kernel, column prefix, ragged tokens
])
def test_linear_without_zero_points(env, uref, N, K, keep, M):
    """zeros = NULL: parity with the oracle's symmetric reading, and the same bits as the same call
    with an explicit array of 8s."""
    uq, torch = env
    rng = wl.rng_for(11, N + K + M)
    w = wl.gen_linear(rng, N, K, sym_zero=True)
    q_sym, q_z8 = uq.QuantLinear.from_numpy(_drop_zeros(w)), uq.QuantLinear.from_numpy(w)
    assert q_sym.zeros is None
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, M, kk)
    y = run_linear(uq, torch, w, q_sym, keep, x)
    y8 = run_linear(uq, torch, w, q_z8, keep, x)
    assert np.array_equal(y.view(np.uint16), y8.view(np.uint16))
    rows = _sample_rows(nk, rng, 96 if M > 64 else 192)
    toks = np.unique(np.concatenate([[0, M - 1], rng.integers(0, M, 6)]))
    ref = uref.w4_linear(w["qweight"], w["scales"], None, np.ascontiguousarray(x[toks]), keep, rows=rows)
    assert linear_err(y[np.ix_(toks, rows)], ref) <= TOL


def test_fused_launches_dequant_embedding_repack_without_zero_points(env, uref):
    uq, torch = env
    rng = wl.rng_for(11, 5)
    # gate + up + SiLU
    N, K, keep = 14336, 4096, Keep(n_keep=12185)
    wg, wu = _drop_zeros(wl.gen_linear(rng, N, K)), _drop_zeros(wl.gen_linear(rng, N, K))
    x = wl.gen_activations(rng, 1, K)
    h = uq.uniql_w4_gate_up_silu([uq.QuantLinear.from_numpy(wg), uq.QuantLinear.from_numpy(wu)], [keep, keep], to_dev(torch, x[0]))
    torch.cuda.synchronize()
    assert linear_err(h.cpu().numpy().reshape(1, -1), uref.gate_up_silu(wg, keep, wu, keep, x)) <= TOL
    # q / k / v + RoPE on a small attention block
    specs = {s.name: s for s in wl.attention_mlp_layer(512, 1024, 8, 2, 64, 15)}
    rope = wl.RopeSpec(T=1, Hq=8, Hkv=2, H_tab=2, D_full=64, D_keep=specs["q_proj"].n_keep // 8, theta=10000.0, pos_max=4096)
    ws = {n: _drop_zeros(wl.gen_linear(rng, specs[n].N, specs[n].K)) for n in ("q_proj", "k_proj", "v_proj")}
    r = wl.gen_rope_inputs(rng, rope)
    xq = wl.gen_activations(rng, 1, 512)
    q, k, v = uq.uniql_w4_qkv_rope([uq.QuantLinear.from_numpy(ws[n]) for n in ("q_proj", "k_proj", "v_proj")],
                                   [specs[n].keep for n in ("q_proj", "k_proj", "v_proj")], to_dev(torch, xq[0]),
                                   to_dev(torch, r["positions"]), to_dev(torch, r["kept_idx"]), 8, 2, 64, rope.D_keep, rope.theta)
    torch.cuda.synchronize()
    rq, rk, rv = uref.qkv_rope(ws["q_proj"], specs["q_proj"].keep, ws["k_proj"], specs["k_proj"].keep, ws["v_proj"],
                               specs["v_proj"].keep, xq, r["positions"], r["kept_idx"], 8, 2, 64, rope.D_keep, rope.theta)
    assert linear_err(q.cpu().numpy().reshape(1, -1), rq.reshape(1, -1)) <= TOL
    assert linear_err(k.cpu().numpy().reshape(1, -1), rk.reshape(1, -1)) <= TOL
    assert linear_err(v.cpu().numpy().reshape(1, -1), rv) <= TOL
    # dequant export, embedding gather, repack: bit-exact
    w = _drop_zeros(wl.gen_linear(rng, 300, 1152))
    qw = uq.QuantLinear.from_numpy(w)
    kp = Keep(n_keep=250, k_keep=515)
    got = uq.uniql_w4_dequant(qw, kp)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().view(np.uint16), uref.w4_dequant(w["qweight"], w["scales"], None, kp).view(np.uint16))
    ids = np.array([0, 299, 17, 17], dtype=np.int32)
    emb = uq.uniql_w4_embedding(qw, to_dev(torch, ids))
    torch.cuda.synchronize()
    assert np.array_equal(emb.cpu().numpy().view(np.uint16), uref.w4_embedding(w["qweight"], w["scales"], None, ids).view(np.uint16))
    out, ko = uq.uniql_w4_repack(qw, kp)
    torch.cuda.synchronize()
    q2, s2, z2, keep2 = uref.w4_repack(w["qweight"], w["scales"], None, kp)
    assert out.zeros is None and z2 is None
    assert np.array_equal(out.qweight.cpu().numpy().view(np.uint32), q2)
    assert np.array_equal(out.scales.cpu().numpy().view(np.uint16), s2.view(np.uint16))


# ------------------------------------------------- persistent streaming GEMV (tall row-prefix x column-prefix matrices)
@pytest.mark.parametrize("N,K,keep", [
    (2048, 128, Keep()),                                   # one chunk, a single group per row, exactly the row threshold
    (2047, 1024, Keep()),                                  # one row below it: the block-per-rows kernel
    (2560, 5120, Keep(k_keep=4352)),                       # Mamba2 out_proj: three chunks
    (8192, 10240, Keep()),                                 # five chunks, tall
    (2048, 10240, Keep()),                                 # exactly the row threshold of long rows
    (2047, 10240, Keep()),                                 # one row below it: the block-per-rows kernel
    (4096, 1024, Keep(n_keep=3456, row_seg_stride=128, row_seg_keep=108, row_seg_limit=4096)),   # row segments (q_proj's rule) on the walk
    (2432, 2048, Keep(n_keep=2052, row_seg_stride=64, row_seg_keep=54, row_seg_limit=2432, k_keep=2001)),   # ... just above its threshold, with a column tail
    (9001, 1024, Keep(k_keep=1001)),                       # ragged rows, column prefix with a tail of one
    (12000, 2304, Keep(n_keep=8193, k_keep=2055)),         # two chunks, 18 groups per row, tail of seven
    (8200, 4096, Keep(n_keep=8197, k_keep=8)),             # the narrowest prefix the vector staging takes
    (8300, 6144, Keep(k_keep=6100)),                       # three chunks: activations read from LDS per tile
    (8192, 8192, Keep(n_keep=8191)),                       # four chunks
    (8448, 10240, Keep(k_keep=9999)),                      # five
    (8200, 14336, Keep(k_keep=12185)),                     # six (a tall down_proj)
    (8200, 16384, Keep(k_keep=16383)),                     # eight chunks, the longest row the kernel takes
])
@pytest.mark.parametrize("sym", [False, True])
def test_streaming_gemv_shapes(env, uref, N, K, keep, sym):
    uq, torch = env
    rng = wl.rng_for(13, N + K)
    w = wl.gen_linear(rng, N, K)
    if sym:
        w["zeros"] = None
    qw = uq.QuantLinear.from_numpy(w)
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, 1, kk)
    y = run_linear(uq, torch, w, qw, keep, x, pad=3)
    # every row against the oracle: the walk must reach each one exactly once
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    assert y.shape == ref.shape and linear_err(y, ref) <= TOL


@pytest.mark.parametrize("N,K,keep", [
    (2304, 1024, Keep(col_seg_stride=128, col_seg_keep=108)),              # o_proj's rule: a partly kept unit per segment
    (2304, 1024, Keep(col_seg_stride=128, col_seg_keep=1)),                # one column per segment
    (2100, 2048, Keep(col_seg_stride=64, col_seg_keep=37)),                # odd keep, two segments per group
    (2048, 4096, Keep(col_seg_stride=8, col_seg_keep=5)),                  # a segment is one unit; the row threshold
    (2047, 4096, Keep(col_seg_stride=8, col_seg_keep=5)),                  # one row below it: the block-per-rows kernel
    (2500, 4096, Keep(n_keep=2049, col_seg_stride=256, col_seg_keep=255)), # row prefix x column segments
    (2200, 6144, Keep(col_seg_stride=128, col_seg_keep=82)),               # three chunks
    (3584, 3584, Keep(col_seg_stride=128, col_seg_keep=96)),               # Qwen2.5-7B o_proj at 25 %
    (2100, 16384, Keep(col_seg_stride=1024, col_seg_keep=1000)),           # eight chunks
    (2100, 1024, Keep(col_seg_stride=128, col_seg_keep=128)),              # segments kept whole
])
@pytest.mark.parametrize("sym", [False, True])
def test_streaming_gemv_column_segments(env, uref, N, K, keep, sym):
    """One token on matrices whose kept columns are the leading ones of every segment (stride a multiple of 8), from
    the row count the persistent walk takes: every row against the oracle, and the same bits on a second call."""
    uq, torch = env
    rng = wl.rng_for(13, 7 * N + K + keep.col_seg_keep)
    w = wl.gen_linear(rng, N, K)
    if sym:
        w["zeros"] = None
    qw = uq.QuantLinear.from_numpy(w)
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, 1, kk)
    y = run_linear(uq, torch, w, qw, keep, x, pad=5)
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    assert y.shape == ref.shape and linear_err(y, ref) <= TOL
    assert normwise_err(y, ref) <= NORM_TOL
    y2 = run_linear(uq, torch, w, qw, keep, x, pad=5)
    assert np.array_equal(y.view(np.uint16), y2.view(np.uint16))


@pytest.mark.parametrize("N,K,keep", [
    (4096, 128, Keep()),                                   # exactly the row threshold of the fused launch, one chunk
    (5000, 2048, Keep(n_keep=4097, k_keep=2047)),
    (6000, 6144, Keep(n_keep=4500, k_keep=6001)),          # three chunks
    (4200, 8192, Keep(k_keep=8191)),                       # four chunks, the longest row of the fused walk
])
@pytest.mark.parametrize("sym", [False, True])
def test_streaming_gate_up_silu_shapes(env, uref, N, K, keep, sym):
    uq, torch = env
    rng = wl.rng_for(14, N + K)
    wg, wu = wl.gen_linear(rng, N, K), wl.gen_linear(rng, N, K)
    if sym:
        wg["zeros"] = wu["zeros"] = None
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, 1, kk)
    h = uq.uniql_w4_gate_up_silu([uq.QuantLinear.from_numpy(wg), uq.QuantLinear.from_numpy(wu)], [keep, keep], to_dev(torch, x[0]))
    torch.cuda.synchronize()
    ref = uref.gate_up_silu(wg, keep, wu, keep, x)      # every row
    assert h.shape == (nk,)
    assert linear_err(h.cpu().numpy().reshape(1, -1), ref) <= TOL


@pytest.mark.parametrize("N,K,keep,M", [
    (14208 + 37, 3584, Keep(n_keep=14208), 8),             # Qwen2.5-7B gate / up at 25 %
    (14336, 4096, Keep(n_keep=12185), 16),                 # Llama-3-8B gate / up at 15 %, every token slot
    (10300, 4096, Keep(n_keep=10241, k_keep=4089), 3),     # ragged rows (the last tile holds one row) and columns, four token slots
    (20600, 1024, Keep(n_keep=20481, k_keep=1017), 13),    # K not split: every wave owns its tile
    (12800, 1024, Keep(n_keep=100 * 108, row_seg_stride=128, row_seg_keep=108, row_seg_limit=12800), 2),   # row segments
])
@pytest.mark.parametrize("sym", [False, True])
def test_gate_up_silu_decode_batches(env, uref, N, K, keep, M, sym):
    """h = SiLU(x Wg) * (x Wu) for 2..16 tokens in one launch: every output against the oracle, strided x and h with
    the padding untouched, the same bits on a second call; one token through the same entry is the one-token call."""
    uq, torch = env
    rng = wl.rng_for(16, N + K + M)
    wg, wu = wl.gen_linear(rng, N, K), wl.gen_linear(rng, N, K)
    if sym:
        wg["zeros"] = None          # one member without zero points: each wave reads its own matrix's
    qg, qu = uq.QuantLinear.from_numpy(wg), uq.QuantLinear.from_numpy(wu)
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, M, kk)
    xb = torch.full((M, kk + 3), 55.0, dtype=torch.float16, device="cuda")
    xb[:, :kk] = to_dev(torch, x)
    hb = torch.full((M, nk + 5), -3.0, dtype=torch.float16, device="cuda")
    uq.uniql_w4_gate_up_silu_batch([qg, qu], [keep, keep], xb[:, :kk], hb[:, :nk])
    torch.cuda.synchronize()
    assert torch.all(hb[:, nk:] == -3.0)
    ref = uref.gate_up_silu(wg, keep, wu, keep, x)
    h = hb[:, :nk].cpu().numpy()
    assert linear_err(h, ref) <= TOL
    h2 = uq.uniql_w4_gate_up_silu_batch([qg, qu], [keep, keep], xb[:, :kk])
    torch.cuda.synchronize()
    assert torch.equal(h2, hb[:, :nk])
    if not sym and N == 14336:
        h1 = uq.uniql_w4_gate_up_silu_batch([qg, qu], [keep, keep], xb[:1, :kk])
        assert torch.equal(h1[0], uq.uniql_w4_gate_up_silu([qg, qu], [keep, keep], xb[0, :kk].contiguous()))


def test_gate_up_silu_decode_batches_refusals(env):
    """Shapes whose activations a block cannot hold (or too few rows for a K range over at most two waves) and token
    counts beyond 16 are refused: there is no scratch memory to fall back on."""
    uq, torch = env
    rng = wl.rng_for(16, 1)
    def call(N, K, keep, M):
        w = uq.QuantLinear.from_numpy(wl.gen_linear(rng, N, K))
        nk, kk = uq.kept_dims(w, keep)
        x = to_dev(torch, wl.gen_activations(rng, M, kk))
        return uq.uniql_w4_gate_up_silu_batch([w, w], [keep, keep], x)
    for N, K, keep, M in ((4096, 2048, Keep(), 4),                 # 256 row tiles of 16 groups: K over four waves
                          (10400, 4224, Keep(), 4),                # 33 groups
                          (10400, 1024, Keep(), 17),               # more tokens than the image holds
                          (10400, 1024, Keep(k_keep=8 * 108, col_seg_stride=128, col_seg_keep=108), 4)):   # column segments
        with pytest.raises(uq.UniqlError) as e:
            call(N, K, keep, M)
        assert e.value.code == uq.UNIQL_E_SHAPE
    assert call(10400, 1024, Keep(), 16).shape == (16, 10400)
    assert call(4096, 1024, Keep(), 4).shape == (4, 4096)          # few rows of 8 groups: K over two waves, served


@pytest.mark.parametrize("N,K,keep,M", [
    (2048, 128, Keep(), 2),                                # one chunk, the row threshold, two tokens
    (3000, 1024, Keep(n_keep=2500, k_keep=1000), 3),       # padded to four tokens; kept width a multiple of 8
    (14208 + 37, 3584, Keep(n_keep=14208), 8),             # Qwen2.5-7B gate / up at 25 %, eight tokens
    (9000, 4096, Keep(), 5),                               # padded to eight tokens
    (4100, 6144, Keep(k_keep=6016), 4),                    # three chunks
    (2500, 8192, Keep(n_keep=2049, k_keep=8184), 8),       # four chunks, 128 KB of activations
    (2100, 8192, Keep(), 7),
    # activations staged once per block (640 row tiles and more, at most 32 groups, up to 16 tokens):
    (10300, 4096, Keep(n_keep=10241, k_keep=4089), 3),     # 32 groups, one kept column past the last whole block of 8, four token slots
    (20600, 1024, Keep(n_keep=20481, k_keep=1017), 13),    # K not split (1281 row tiles), 16 token slots, ragged rows and columns
    (10400, 2048, Keep(), 16),                             # every token slot used
    (10400, 4224, Keep(k_keep=4096), 9),                   # exactly 32 kept groups of a longer row
    (10400, 4224, Keep(k_keep=4100), 8),                   # 33 groups: the per-wave staging again
    (12800, 1024, Keep(n_keep=100 * 108, row_seg_stride=128, row_seg_keep=108, row_seg_limit=12800), 6),   # row segments
])
@pytest.mark.parametrize("sym", [False, True])
def test_decode_batches_on_tall_matrices(env, uref, N, K, keep, M, sym):
    """2..16 tokens on tall row-prefix x column-prefix matrices (small decode batches on gate / up shaped
    linears), every output against the oracle."""
    uq, torch = env
    rng = wl.rng_for(15, N + K + M)
    w = wl.gen_linear(rng, N, K)
    if sym:
        w["zeros"] = None
    qw = uq.QuantLinear.from_numpy(w)
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, M, kk)
    y = run_linear(uq, torch, w, qw, keep, x, pad=5)
    ref = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    assert y.shape == ref.shape and linear_err(y, ref) <= TOL


# ------------------------------------------------- prompt-sized RoPE calls
@pytest.mark.parametrize("spec", [
    wl.RopeSpec(T=64, Hq=32, Hkv=8, H_tab=8, D_full=128, D_keep=108, theta=5.0e5, pos_max=8192),     # 64 tokens
    wl.RopeSpec(T=1027, Hq=32, Hkv=8, H_tab=8, D_full=128, D_keep=108, theta=5.0e5, pos_max=-1),     # odd token count
    wl.RopeSpec(T=4099, Hq=28, Hkv=4, H_tab=4, D_full=128, D_keep=96, theta=1.0e6, pos_max=131072),  # Qwen heads
    wl.RopeSpec(T=300, Hq=8, Hkv=8, H_tab=8, D_full=64, D_keep=64, theta=1.0e4, pos_max=4096),       # one table row per head, unpruned
    wl.RopeSpec(T=257, Hq=6, Hkv=0, H_tab=2, D_full=256, D_keep=200, theta=1.0e4, pos_max=4096),     # no K tensor
    wl.RopeSpec(T=128, Hq=2, Hkv=2, H_tab=1, D_full=32, D_keep=4, theta=1.0e4, pos_max=100),         # one word per half head
    wl.RopeSpec(T=96, Hq=3, Hkv=1, H_tab=1, D_full=64, D_keep=44, theta=1.0e4, pos_max=100),         # token rows not a multiple of 16 bytes
    wl.RopeSpec(T=70, Hq=4, Hkv=4, H_tab=4, D_full=64, D_keep=54, theta=1.0e4, pos_max=100),         # odd pair count: 2-byte accesses
    wl.RopeSpec(T=41, Hq=18, Hkv=6, H_tab=2, D_full=256, D_keep=256, theta=1.0e4, pos_max=4096),     # a row fills a wave; 9 Q and 3 K heads per table row: several chunks of head steps
    wl.RopeSpec(T=33, Hq=14, Hkv=6, H_tab=2, D_full=128, D_keep=40, theta=1.0e6, pos_max=70000),     # six rows per wave step, the last step of Q and of K partly filled
    wl.RopeSpec(T=32, Hq=5, Hkv=5, H_tab=5, D_full=128, D_keep=124, theta=5.0e5, pos_max=8192),      # 31 units per row: odd half row, two rows per step, one head per table row
    wl.RopeSpec(T=31, Hq=32, Hkv=8, H_tab=8, D_full=128, D_keep=108, theta=5.0e5, pos_max=8192),     # one token below the whole-row kernel's threshold
])
def test_rope_prompt_sized_calls(env, uref, spec):
    uq, torch = env
    r = wl.gen_rope_inputs(wl.rng_for(16, spec.T + spec.D_keep), spec)
    qo, ko = uref.pruned_rope(r["q"], r["k"], r["positions"], r["kept_idx"], spec.D_full, spec.theta)
    gq, gk = run_rope(uq, torch, r, spec)
    assert rope_err(gq, qo) <= TOL
    if ko is not None:
        assert rope_err(gk, ko) <= TOL
    # pair norms survive the rotation (to fp16 rounding)
    hk = spec.D_keep // 2
    n_in = r["q"][..., :hk].astype(np.float64) ** 2 + r["q"][..., hk:].astype(np.float64) ** 2
    n_out = gq[..., :hk].astype(np.float64) ** 2 + gq[..., hk:].astype(np.float64) ** 2
    assert np.max(np.abs(n_out - n_in) / np.maximum(n_in, 1e-3)) < 5e-3


# ------------------------------------------------- the read probe (measurement aid)
@pytest.mark.parametrize("nbytes", [16, 8192, 8192 * 3 + 4096 + 16, 5_000_000 // 16 * 16])
def test_read_probe_xor_words(env, nbytes):
    """One xor word per 8 KB read (the last piece may be short); words past the last piece stay untouched."""
    uq, torch = env
    rng = wl.rng_for(15, nbytes % 1000)
    src = rng.integers(0, 2 ** 32, size=nbytes // 4 + 64, dtype=np.uint64).astype(np.uint32)
    pieces = (nbytes + 8191) // 8192
    out = torch.full((pieces + 5,), 0x5a5a5a5a, dtype=torch.int32, device="cuda")
    uq.uniql_stream_read_probe(torch.from_numpy(src.view(np.int32)).cuda(), nbytes, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().view(np.uint32)
    words = src[: nbytes // 4]
    exp = [int(np.bitwise_xor.reduce(words[i * 2048:(i + 1) * 2048])) for i in range(pieces)]
    assert list(got[:pieces]) == exp
    assert np.all(got[pieces:] == 0x5a5a5a5a)


# ------------------------------------------------- HIP graph capture of the whole step
def test_graph_replays_equal_eager_launches(env, uref):
    """The four launches of a decode step (q/k/v + RoPE, o, gate + up + SiLU, down) captured once on a side stream and
    replayed with new activations between the replays give the bits of eager launches every time: the entry points
    allocate nothing, record no memset and never synchronise."""
    uq, torch = env
    rng = wl.rng_for(16, 0)
    specs = {s.name: s for s in wl.llama3_8b_layer(15)}
    rope = wl.llama3_8b_rope(15, T=1)
    lin = {n: uq.QuantLinear.from_numpy(wl.gen_linear(rng, s.N, s.K)) for n, s in specs.items()}
    r = wl.gen_rope_inputs(rng, rope)
    pos, idx = to_dev(torch, r["positions"][:1].copy()), to_dev(torch, r["kept_idx"])
    x_h = torch.empty(specs["q_proj"].k_keep, dtype=torch.float16, device="cuda")
    x_o = torch.empty((1, specs["o_proj"].k_keep), dtype=torch.float16, device="cuda")
    x_d = torch.empty((1, specs["down_proj"].k_keep), dtype=torch.float16, device="cuda")
    q = torch.empty((rope.Hq, rope.D_keep), dtype=torch.float16, device="cuda")
    k = torch.empty((rope.Hkv, rope.D_keep), dtype=torch.float16, device="cuda")
    v = torch.empty(specs["v_proj"].n_keep, dtype=torch.float16, device="cuda")
    yo = torch.empty((1, specs["o_proj"].n_keep), dtype=torch.float16, device="cuda")
    h = torch.empty(specs["gate_proj"].n_keep, dtype=torch.float16, device="cuda")
    yd = torch.empty((1, specs["down_proj"].n_keep), dtype=torch.float16, device="cuda")
    qkv = uq.QkvRopeCall([lin[n] for n in ("q_proj", "k_proj", "v_proj")], [specs[n].keep for n in ("q_proj", "k_proj", "v_proj")],
                         x_h, q, k, v, pos, idx, rope.D_full, rope.theta)
    glu = uq.GateUpCall([lin["gate_proj"], lin["up_proj"]], [specs["gate_proj"].keep, specs["up_proj"].keep], x_h, h)

    def step():
        qkv.run()
        uq.uniql_w4_linear(lin["o_proj"], specs["o_proj"].keep, x_o, yo)
        glu.run()
        uq.uniql_w4_linear(lin["down_proj"], specs["down_proj"].keep, x_d, yd)

    def new_inputs(i):
        x_h.copy_(to_dev(torch, wl.gen_activations(wl.rng_for(16, 10 + i), 1, x_h.numel())[0]))
        x_o.copy_(to_dev(torch, wl.gen_activations(wl.rng_for(16, 20 + i), 1, x_o.shape[1])))
        x_d.copy_(to_dev(torch, wl.gen_activations(wl.rng_for(16, 30 + i), 1, x_d.shape[1])))

    outs = (q, k, v, yo, h, yd)
    new_inputs(0)
    step()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        step()
    for i in range(1, 4):
        new_inputs(i)
        step()
        torch.cuda.synchronize()
        eager = [t.clone() for t in outs]
        for t in outs:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for got, exp in zip(outs, eager):
            assert torch.equal(got, exp), i
