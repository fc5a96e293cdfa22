"""Pins for the CPU oracle's repack (Sec. 3.4: unpack the INT4 weights, drop the pruned channels, pack
again into INT32).  No GPU.

The oracle walks rows, groups and nibbles one by one.  Here the same compact matrix is built a second
way -- numpy unpacks the whole matrix into one code per element, index lists select rows and whole
groups, numpy packs again -- and the two must agree bit for bit; then the compact matrix must give
exactly the outputs and dequantised weights of the truncated source.
"""
import zlib

import numpy as np
import pytest

import workloads as wl
from workloads import Keep

GROUP = 128


def unpack_codes(qweight):
    N, K8 = qweight.shape
    sh = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    return ((qweight[:, :, None] >> sh) & np.uint32(15)).reshape(N, K8 * 8).astype(np.uint8)


def pack_codes(codes):
    N, K = codes.shape
    c = codes.reshape(N, K // 8, 8).astype(np.uint32)
    out = np.zeros((N, K // 8), dtype=np.uint32)
    for j in range(8):
        out |= c[:, :, j] << np.uint32(4 * j)
    return out


def kept_rows_cols(N, K, keep: Keep):
    r, k = np.arange(N), np.arange(K)
    rows = (r[(r >= keep.row_seg_limit) | (r % keep.row_seg_stride < keep.row_seg_keep)]
            if keep.row_seg_stride else r[: keep.n_keep or N])
    cols = k[k % keep.col_seg_stride < keep.col_seg_keep] if keep.col_seg_stride else k[: keep.k_keep or K]
    return rows, cols


def carried_groups(K, keep: Keep, cols):
    """Groups of the source that the compact matrix holds: those with a kept column, when the kept
    columns are a prefix or segments of a stride that is a multiple of the group; else all of them."""
    if keep.col_seg_stride and keep.col_seg_stride % GROUP:
        return np.arange(K // GROUP)
    return np.unique(cols // GROUP)


CASES = [
    ("unpruned", 24, 512, Keep()),
    ("row_prefix", 40, 256, Keep(n_keep=33)),
    ("col_prefix_ragged", 16, 1024, Keep(k_keep=870)),
    ("col_prefix_group_edge", 16, 1024, Keep(k_keep=768)),
    ("col_prefix_tiny", 8, 512, Keep(k_keep=3)),
    ("qk_heads", 256, 256, Keep(n_keep=216, row_seg_stride=64, row_seg_keep=54, row_seg_limit=256)),
    ("mamba_in_proj_like", 2 * 160 + 24, 256, Keep(n_keep=2 * 136 + 24, row_seg_stride=160, row_seg_keep=136, row_seg_limit=320)),
    ("o_proj_heads", 32, 1024, Keep(k_keep=8 * 108, col_seg_stride=128, col_seg_keep=108)),
    ("col_segments_two_groups_one_kept", 16, 1024, Keep(k_keep=4 * 100, col_seg_stride=256, col_seg_keep=100)),
    ("col_segments_wide", 16, 2048, Keep(k_keep=4 * 200, col_seg_stride=512, col_seg_keep=200)),
    ("col_segments_below_group", 16, 512, Keep(k_keep=8 * 54, col_seg_stride=64, col_seg_keep=54)),
    ("col_segments_stride_not_group_multiple", 16, 768, Keep(k_keep=4 * 10, col_seg_stride=192, col_seg_keep=10)),
    ("rows_and_cols", 96, 1024, Keep(n_keep=70, k_keep=500)),
]


@pytest.mark.parametrize("name,N,K,keep", CASES, ids=[c[0] for c in CASES])
def test_repack_equals_numpy_selection(uref, name, N, K, keep):
    rng = np.random.default_rng(zlib.crc32(name.encode()))
    w = wl.gen_linear(rng, N, K)
    q2, s2, z2, keep2 = uref.w4_repack(w["qweight"], w["scales"], w["zeros"], keep)
    rows, cols = kept_rows_cols(N, K, keep)
    groups = carried_groups(K, keep, cols)
    col_idx = (groups[:, None] * GROUP + np.arange(GROUP)[None, :]).reshape(-1)
    exp_q = pack_codes(unpack_codes(w["qweight"])[np.ix_(rows, col_idx)])
    assert q2.shape == exp_q.shape and np.array_equal(q2, exp_q)
    assert np.array_equal(s2.view(np.uint16), w["scales"][np.ix_(rows, groups)].view(np.uint16))
    assert np.array_equal(z2, w["zeros"][np.ix_(rows, groups)])
    # the descriptor for the compact matrix keeps every row and marks exactly the kept columns at
    # their new places
    k2 = Keep(*keep2)
    rows2, cols2 = kept_rows_cols(q2.shape[0], q2.shape[1] * 8, k2)
    assert np.array_equal(rows2, np.arange(rows.size))
    new_pos = {int(c): i for i, c in enumerate(col_idx)}
    assert np.array_equal(cols2, np.array([new_pos[int(c)] for c in cols]))


@pytest.mark.parametrize("name,N,K,keep", CASES, ids=[c[0] for c in CASES])
def test_repacked_matrix_gives_the_same_outputs(uref, name, N, K, keep):
    """y(W', keep') == y(W, keep) and dequant(W', keep') == dequant(W, keep), exactly: the sums run
    over the same numbers in the same order."""
    rng = np.random.default_rng(zlib.crc32((name + "y").encode()))
    w = wl.gen_linear(rng, N, K)
    q2, s2, z2, keep2 = uref.w4_repack(w["qweight"], w["scales"], w["zeros"], keep)
    nk, kk = uref.count_kept(N, K, keep)
    x = wl.gen_activations(rng, 3, kk)
    y_src = uref.w4_linear(w["qweight"], w["scales"], w["zeros"], x, keep)
    y_cmp = uref.w4_linear(q2, s2, z2, x, Keep(*keep2))
    assert np.array_equal(y_src, y_cmp)
    d_src = uref.w4_dequant(w["qweight"], w["scales"], w["zeros"], keep)
    d_cmp = uref.w4_dequant(q2, s2, z2, Keep(*keep2))
    assert np.array_equal(d_src.view(np.uint16), d_cmp.view(np.uint16))


def test_repack_sizes_of_the_model_shapes(uref):
    """Llama-3-8B shapes at 15 %: rows shrink exactly, a column prefix to whole groups, per-head
    column segments (a head is one group) not at all."""
    assert uref.w4_repack_plan(14336, 4096, Keep(n_keep=12185))[:2] == (12185, 4096)
    assert uref.w4_repack_plan(4096, 14336, Keep(k_keep=12185)) == (4096, 12288, (0, 12185, 0, 0, 0, 0, 0))
    assert uref.w4_repack_plan(4096, 4096, Keep(k_keep=32 * 108, col_seg_stride=128, col_seg_keep=108)) == \
        (4096, 4096, (0, 3456, 0, 0, 0, 128, 108))
    assert uref.w4_repack_plan(4096, 4096, Keep(n_keep=3456, row_seg_stride=64, row_seg_keep=54, row_seg_limit=4096))[:2] == (3456, 4096)
    # a column prefix that ends on a group edge needs no column descriptor at all
    assert uref.w4_repack_plan(64, 1024, Keep(k_keep=768)) == (64, 768, (0, 0, 0, 0, 0, 0, 0))


def test_repack_twice_is_stable(uref):
    """Repacking the compact matrix with its own descriptor changes nothing."""
    rng = np.random.default_rng(7)
    w = wl.gen_linear(rng, 48, 2048)
    keep = Keep(n_keep=40, k_keep=4 * 200, col_seg_stride=512, col_seg_keep=200)
    q2, s2, z2, keep2 = uref.w4_repack(w["qweight"], w["scales"], w["zeros"], keep)
    q3, s3, z3, keep3 = uref.w4_repack(q2, s2, z2, Keep(*keep2))
    assert np.array_equal(q2, q3) and np.array_equal(s2.view(np.uint16), s3.view(np.uint16)) and np.array_equal(z2, z3)
    assert keep3 == keep2
