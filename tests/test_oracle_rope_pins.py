"""Pins for the CPU oracle's pruned RoPE (no GPU): the textbook half-split RoPE
written with numpy, norm preservation, relative-position property, and the
reduction of the pruned case to the unpruned one."""
import numpy as np
import pytest

import workloads as wl


def textbook_rope(x, pos, theta):
    """Standard half-split RoPE on [T][H][D] (fp64): x * cos + rotate_half(x) * sin."""
    T, H, D = x.shape
    inv_freq = theta ** (-np.arange(0, D, 2, dtype=np.float64) / D)          # [D/2]
    ang = pos.astype(np.float64)[:, None] * inv_freq[None, :]                 # [T][D/2]
    cos = np.concatenate([np.cos(ang), np.cos(ang)], axis=1)[:, None, :]
    sin = np.concatenate([np.sin(ang), np.sin(ang)], axis=1)[:, None, :]
    rot = np.concatenate([-x[..., D // 2:], x[..., : D // 2]], axis=-1)
    return x * cos + rot * sin


def test_identity_table_full_dim_is_textbook_rope(uref):
    rng = np.random.default_rng(11)
    T, Hq, Hkv, D = 5, 4, 2, 64
    q = rng.standard_normal((T, Hq, D)).astype(np.float16)
    k = rng.standard_normal((T, Hkv, D)).astype(np.float16)
    pos = np.array([0, 1, 17, 4095, 32767], dtype=np.int32)
    idx = np.tile(np.arange(D // 2, dtype=np.int32), (2, 1))
    for theta in (10000.0, 1.0e6):
        qo, ko = uref.pruned_rope(q, k, pos, idx, D, theta)
        assert np.max(np.abs(qo - textbook_rope(q.astype(np.float64), pos, theta))) < 1e-9
        assert np.max(np.abs(ko - textbook_rope(k.astype(np.float64), pos, theta))) < 1e-9
    assert np.array_equal(qo[0], q[0].astype(np.float64))          # position 0 is the identity


@pytest.mark.parametrize("spec", [wl.small_rope(), wl.llama3_8b_rope(15, T=3), wl.qwen25_7b_rope(25, T=2),
                                  wl.llama3_8b_rope(35, T=2)])
def test_pruned_rope_is_full_rope_on_scattered_input(uref, spec):
    """Scatter the kept channels of each head to their original positions in a
    zero D_full vector, apply the textbook RoPE, gather back."""
    r = wl.gen_rope_inputs(wl.rng_for(0, 21), spec)
    qo, ko = uref.pruned_rope(r["q"], r["k"], r["positions"], r["kept_idx"], spec.D_full, spec.theta)
    half, hk = spec.D_full // 2, spec.D_keep // 2
    for x, out, H in ((r["q"], qo, spec.Hq), (r["k"], ko, spec.Hkv)):
        if x is None:
            assert out is None
            continue
        per = H // spec.H_tab
        full = np.zeros((spec.T, H, spec.D_full))
        for h in range(H):
            tab = r["kept_idx"][h // per]
            full[:, h, tab] = x[:, h, :hk]
            full[:, h, half + tab] = x[:, h, hk:]
        ref = textbook_rope(full, r["positions"], spec.theta)
        for h in range(H):
            tab = r["kept_idx"][h // per]
            got = out[:, h, :]
            assert np.max(np.abs(got[:, :hk] - ref[:, h, tab])) < 1e-9
            assert np.max(np.abs(got[:, hk:] - ref[:, h, half + tab])) < 1e-9


def test_pair_norms_preserved(uref):
    spec = wl.llama3_8b_rope(15, T=4)
    r = wl.gen_rope_inputs(wl.rng_for(1, 22), spec)
    qo, ko = uref.pruned_rope(r["q"], r["k"], r["positions"], r["kept_idx"], spec.D_full, spec.theta)
    hk = spec.D_keep // 2
    for x, out in ((r["q"], qo), (r["k"], ko)):
        x = x.astype(np.float64)
        n_in = x[..., :hk] ** 2 + x[..., hk:] ** 2
        n_out = out[..., :hk] ** 2 + out[..., hk:] ** 2
        assert np.max(np.abs(n_in - n_out)) < 1e-12


def test_scores_depend_on_relative_position_only(uref):
    """<RoPE_m q, RoPE_n k> is unchanged when both positions shift by the same amount."""
    rng = np.random.default_rng(23)
    D_full, Dk, H = 128, 96, 4
    idx = np.stack([rng.permutation(D_full // 2)[: Dk // 2] for _ in range(H)]).astype(np.int32)
    q = rng.standard_normal((1, H, Dk)).astype(np.float16)
    k = rng.standard_normal((1, H, Dk)).astype(np.float16)

    def score(m, n):
        qo, _ = uref.pruned_rope(q, None, np.array([m], dtype=np.int32), idx, D_full, 10000.0)
        ko, _ = uref.pruned_rope(k, None, np.array([n], dtype=np.int32), idx, D_full, 10000.0)
        return np.sum(qo * ko, axis=-1)

    assert np.max(np.abs(score(100, 37) - score(1100, 1037))) < 1e-9
    assert np.max(np.abs(score(5, 5) - np.sum(q.astype(np.float64) * k.astype(np.float64), axis=-1))) < 1e-9
    assert np.max(np.abs(score(100, 37) - score(100, 38))) > 1e-3     # and does depend on the difference


def test_heads_share_table_rows_in_contiguous_blocks(uref):
    """GQA: query heads h use table row h / (Hq / H_tab) (Alg. A1: one index vector per KV head)."""
    rng = np.random.default_rng(24)
    D_full, Dk, Hq, Hkv = 64, 32, 6, 2
    idx = np.stack([rng.permutation(D_full // 2)[: Dk // 2] for _ in range(Hkv)]).astype(np.int32)
    q = np.tile(rng.standard_normal((1, 1, Dk)).astype(np.float16), (1, Hq, 1))
    pos = np.array([77], dtype=np.int32)
    qo, _ = uref.pruned_rope(q, None, pos, idx, D_full, 10000.0)
    assert np.array_equal(qo[0, 0], qo[0, 1]) and np.array_equal(qo[0, 0], qo[0, 2])
    assert np.array_equal(qo[0, 3], qo[0, 4]) and np.array_equal(qo[0, 3], qo[0, 5])
    assert not np.array_equal(qo[0, 0], qo[0, 3])
    # each block equals the single-head call with its own table row
    for g in range(2):
        one, _ = uref.pruned_rope(np.ascontiguousarray(q[:, :1]), None, pos, idx[g:g + 1], D_full, 10000.0)
        assert np.array_equal(one[0, 0], qo[0, 3 * g])


def test_single_pair_closed_form(uref):
    """One kept pair with original index j at position p: rotation by p * theta^(-2j/D)."""
    D_full, theta = 16, 10000.0
    for j, p in ((0, 3), (5, 1000), (7, 32767)):
        q = np.array([[[1.0, 0.0]]], dtype=np.float16)
        idx = np.array([[j]], dtype=np.int32)
        qo, _ = uref.pruned_rope(q, None, np.array([p], dtype=np.int32), idx, D_full, theta)
        phi = p * theta ** (-2.0 * j / D_full)
        assert qo[0, 0, 0] == pytest.approx(np.cos(phi), abs=1e-12)
        assert qo[0, 0, 1] == pytest.approx(np.sin(phi), abs=1e-12)


# ---- the fp64-input rotation and the fused projection + rotation (y = RoPE(x W)) ----
def test_rope_f64_is_textbook_rope_on_arbitrary_fp64_input(uref):
    """Identity table, full dimension, inputs that are NOT fp16-representable."""
    rng = np.random.default_rng(12)
    T, H, D = 4, 6, 32
    x = rng.standard_normal((T, H, D)) * np.pi
    pos = np.array([0, 3, 1000, 32767], dtype=np.int32)
    idx = np.tile(np.arange(D // 2, dtype=np.int32), (3, 1))
    got = uref.pruned_rope_f64(x, pos, idx, D, 5.0e5)
    assert np.max(np.abs(got - textbook_rope(x, pos, 5.0e5))) < 1e-9
    assert np.array_equal(got[0], x[0])


@pytest.mark.parametrize("spec", [wl.small_rope(), wl.llama3_8b_rope(15, T=2), wl.qwen25_7b_rope(25, T=2)])
def test_rope_f64_scattered_and_same_as_fp16_entry(uref, spec):
    """Pruned case against the textbook RoPE on scattered inputs (as for the fp16 entry), and bit-for-bit
    agreement with the fp16 entry on fp16-representable inputs."""
    r = wl.gen_rope_inputs(wl.rng_for(0, 22), spec)
    qo, _ = uref.pruned_rope(r["q"], r["k"], r["positions"], r["kept_idx"], spec.D_full, spec.theta)
    x = r["q"].astype(np.float64) * 1.0000001          # off the fp16 grid
    got = uref.pruned_rope_f64(x, r["positions"], r["kept_idx"], spec.D_full, spec.theta)
    half, hk, per = spec.D_full // 2, spec.D_keep // 2, spec.Hq // spec.H_tab
    full = np.zeros((spec.T, spec.Hq, spec.D_full))
    for h in range(spec.Hq):
        tab = r["kept_idx"][h // per]
        full[:, h, tab] = x[:, h, :hk]
        full[:, h, half + tab] = x[:, h, hk:]
    ref = textbook_rope(full, r["positions"], spec.theta)
    for h in range(spec.Hq):
        tab = r["kept_idx"][h // per]
        assert np.max(np.abs(got[:, h, :hk] - ref[:, h, tab])) < 1e-9
        assert np.max(np.abs(got[:, h, hk:] - ref[:, h, half + tab])) < 1e-9
    same = uref.pruned_rope_f64(r["q"].astype(np.float64), r["positions"], r["kept_idx"], spec.D_full, spec.theta)
    assert np.array_equal(same, qo)


def test_fused_qkv_rope_is_numpy_matmul_then_textbook_rope(uref):
    """y = RoPE(x W) on a small attention block with pruned heads: an independently unpacked fp64 weight
    matrix, numpy matmul, scatter to the full head dimension, textbook RoPE, gather back."""
    rng = wl.rng_for(0, 23)
    Hq, Hkv, D, Dk, hidden, T = 4, 2, 64, 54, 256, 2
    hk = Dk // 2
    keep_q = wl.Keep(n_keep=Hq * Dk, row_seg_stride=D // 2, row_seg_keep=hk, row_seg_limit=Hq * D)
    keep_k = wl.Keep(n_keep=Hkv * Dk, row_seg_stride=D // 2, row_seg_keep=hk, row_seg_limit=Hkv * D)
    keep_v = wl.Keep(n_keep=Hkv * Dk, row_seg_stride=D, row_seg_keep=Dk, row_seg_limit=Hkv * D)
    wq, wk, wv = (wl.gen_linear(rng, H * D, hidden) for H in (Hq, Hkv, Hkv))
    x = wl.gen_activations(rng, T, hidden)
    pos = np.array([5, 4095], dtype=np.int32)
    idx = np.stack([rng.permutation(D // 2)[:hk] for _ in range(Hkv)]).astype(np.int32)
    theta = 1.0e4
    q, k, v = uref.qkv_rope(wq, keep_q, wk, keep_k, wv, keep_v, x, pos, idx, Hq, Hkv, D, Dk, theta)

    def dense(w):   # independent unpack: fp16(q - z) * s through numpy
        qw = w["qweight"]
        nib = np.stack([(qw >> np.uint32(4 * j)) & np.uint32(15) for j in range(8)], axis=-1).reshape(qw.shape[0], -1)
        s = np.repeat(w["scales"].astype(np.float64), 128, axis=1)
        z = np.repeat(w["zeros"].astype(np.float64), 128, axis=1)
        return ((nib.astype(np.float64) - z) * s).astype(np.float16).astype(np.float64)

    xf = x.astype(np.float64)
    for w, out, H in ((wq, q, Hq), (wk, k, Hkv)):
        full = (xf @ dense(w).T).reshape(T, H, D)            # unpruned projection, [T][H][D]
        # pruning keeps, of every head, the leading hk channels of each half; their ORIGINAL pair
        # indices are the table entries, so scatter kept channel i to position idx[i] before rotating
        per = H // Hkv
        scat = np.zeros((T, H, D))
        for h in range(H):
            tab = idx[h // per]
            scat[:, h, tab] = full[:, h, :hk]
            scat[:, h, D // 2 + tab] = full[:, h, D // 2: D // 2 + hk]
        ref = textbook_rope(scat, pos, theta)
        for h in range(H):
            tab = idx[h // per]
            assert np.max(np.abs(out[:, h, :hk] - ref[:, h, tab])) < 1e-9
            assert np.max(np.abs(out[:, h, hk:] - ref[:, h, D // 2 + tab])) < 1e-9
    vfull = (xf @ dense(wv).T).reshape(T, Hkv, D)[:, :, :Dk].reshape(T, -1)
    assert np.max(np.abs(v - vfull)) < 1e-9
