"""Host-side checks of the C ABI (no GPU): the library loads, exports every
function the header declares, and rejects bad arguments before any launch."""
import ctypes as C
import re

import numpy as np
import pytest

import paper_2512_03383_amd as uq
from paper_2512_03383_amd import KeepDesc, W4


def declared_functions():
    text = open(uq.HEADER_PATH).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(uniql_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"uniql_w4_linear", "uniql_w4_dequant", "uniql_pruned_rope", "uniql_strerror",
            "uniql_last_hip_error"} <= set(names)
    L = uq.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert uq.lib().uniql_version() >= 100


def test_struct_layout_matches_header():
    assert C.sizeof(W4) == 3 * 8 + 6 * 4          # three pointers, six int32
    assert W4.dtype.offset == 36 and W4.col_interleave.offset == 40 and W4.bits.offset == 44
    assert C.sizeof(KeepDesc) == 10 * 4
    assert W4.N_total.offset == 24 and W4.group.offset == 32
    assert KeepDesc.col_seg_keep.offset == 24 and KeepDesc.row_seg2_limit.offset == 36


def test_strerror_covers_all_codes():
    msgs = {c: uq.strerror(c) for c in range(0, -8, -1)}
    assert msgs[0] == "ok" and "NULL" in msgs[-1] and "gfx950" in msgs[-5]
    assert len(set(msgs.values())) == 8


# fake but well-aligned "device" addresses: validation must reject before touching them
P = 0x10000


def _w(N=256, K=512, group=128, q=P, s=P, z=P):
    return W4(q, s, z, N, K, group)


def _lin(w, keep, x=P, ldx=512, y=P, ldy=256, M=1):
    kd = C.byref(keep) if keep is not None else None
    return uq.lib().uniql_w4_linear(C.byref(w) if w is not None else None, kd, C.c_void_p(x), ldx,
                                    C.c_void_p(y), ldy, M, None)


def test_linear_rejects_null_shape_keep_align():
    L = uq
    assert _lin(None, None) == L.UNIQL_E_NULL
    assert _lin(_w(q=0), None) == L.UNIQL_E_NULL
    assert _lin(_w(), None, x=0) == L.UNIQL_E_NULL
    assert _lin(_w(), None, y=0) == L.UNIQL_E_NULL
    assert _lin(_w(group=64), None) == L.UNIQL_E_SHAPE
    assert _lin(_w(K=520), None) == L.UNIQL_E_SHAPE
    assert _lin(_w(N=0), None) == L.UNIQL_E_SHAPE
    assert _lin(_w(), None, M=0) == L.UNIQL_E_SHAPE
    assert _lin(_w(), None, ldx=511) == L.UNIQL_E_SHAPE
    assert _lin(_w(), None, ldy=255) == L.UNIQL_E_SHAPE
    assert _lin(_w(), KeepDesc(n_keep=100), ldy=99) == L.UNIQL_E_SHAPE
    assert _lin(_w(q=P + 8), None) == L.UNIQL_E_ALIGN
    assert _lin(_w(s=P + 1), None) == L.UNIQL_E_ALIGN
    assert _lin(_w(), None, x=P + 1) == L.UNIQL_E_ALIGN
    assert _lin(_w(), KeepDesc(n_keep=257)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(k_keep=513)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(n_keep=-1)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(row_seg_stride=64, row_seg_keep=65, row_seg_limit=256)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(row_seg_stride=64, row_seg_keep=0, row_seg_limit=256)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(row_seg_stride=64, row_seg_keep=32, row_seg_limit=100)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(row_seg_stride=64, row_seg_keep=32, row_seg_limit=320)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(n_keep=100, row_seg_stride=64, row_seg_keep=32, row_seg_limit=256)) == L.UNIQL_E_KEEP
    # second family of row segments (N = 256): needs the first, keep within stride, span a multiple of the stride, inside the matrix
    assert _lin(_w(), KeepDesc(row_seg2_stride=32, row_seg2_keep=8, row_seg2_limit=64)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(row_seg_stride=64, row_seg_keep=32, row_seg_limit=128, row_seg2_stride=32, row_seg2_keep=33, row_seg2_limit=192)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(row_seg_stride=64, row_seg_keep=32, row_seg_limit=128, row_seg2_stride=32, row_seg2_keep=8, row_seg2_limit=200)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(row_seg_stride=64, row_seg_keep=32, row_seg_limit=128, row_seg2_stride=32, row_seg2_keep=8, row_seg2_limit=288)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(row_seg_stride=64, row_seg_keep=32, row_seg_limit=128, row_seg2_stride=32, row_seg2_keep=8, row_seg2_limit=96)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(n_keep=64 + 16 + 65, row_seg_stride=64, row_seg_keep=32, row_seg_limit=128, row_seg2_stride=32, row_seg2_keep=8, row_seg2_limit=192)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(col_seg_stride=100, col_seg_keep=50)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(col_seg_stride=128, col_seg_keep=129)) == L.UNIQL_E_KEEP
    assert _lin(_w(), KeepDesc(k_keep=7, col_seg_stride=128, col_seg_keep=64)) == L.UNIQL_E_KEEP


def test_matrix_without_zero_points_is_accepted():
    """zeros = NULL is the symmetric scheme, not an error: validation passes it on to the device check."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present; covered by the gpu tests")
    assert _lin(_w(z=0), None) in (uq.UNIQL_E_HIP, uq.UNIQL_E_ARCH)
    assert _lin(_w(z=0), KeepDesc(n_keep=300)) == uq.UNIQL_E_KEEP


def test_dequant_rejects_bad_arguments():
    L = uq.lib()
    w = _w()
    assert L.uniql_w4_dequant(None, None, C.c_void_p(P), None) == uq.UNIQL_E_NULL
    assert L.uniql_w4_dequant(C.byref(w), None, None, None) == uq.UNIQL_E_NULL
    assert L.uniql_w4_dequant(C.byref(w), C.byref(KeepDesc(n_keep=1000)), C.c_void_p(P), None) == uq.UNIQL_E_KEEP


def _rope(q=P, k=P, pos=P, idx=P, T=1, Hq=8, Hkv=2, H_tab=2, D_full=128, D_keep=108, theta=1e4):
    return uq.lib().uniql_pruned_rope(C.c_void_p(q), C.c_void_p(k) if k else None, C.c_void_p(pos),
                                      C.c_void_p(idx), T, Hq, Hkv, H_tab, D_full, D_keep, theta, None)


def test_dtype_field_is_validated():
    """0 = fp16, 1 = bfloat16, anything else is refused before any launch; a bfloat16 matrix passes the same
    host checks as an fp16 one; matrices that share a fused call must share the format."""
    w = _w()
    w.dtype = 2
    assert _lin(w, None) == uq.UNIQL_E_SHAPE
    w.dtype = -1
    assert _lin(w, None) == uq.UNIQL_E_SHAPE
    wb = _w()
    wb.dtype = uq.UNIQL_BF16
    assert _lin(wb, None, M=0) == uq.UNIQL_E_SHAPE
    assert _lin(wb, KeepDesc(n_keep=999), M=1) == uq.UNIQL_E_KEEP
    import torch
    if not torch.cuda.is_available():
        assert _lin(wb, None) in (uq.UNIQL_E_HIP, uq.UNIQL_E_ARCH)
    # gate (fp16) and up (bfloat16) in one fused call
    W = (W4 * 2)(_w(), wb)
    assert uq.lib().uniql_w4_gate_up_silu(W, None, C.c_void_p(P), C.c_void_p(P), None) == uq.UNIQL_E_SHAPE


def test_bits_field_is_validated():
    """0 and 4 = 4-bit codes, 8 / 6 / 3 = codes of those widths in the two calls that serve them, anything else refused;
    such a matrix passes the same host checks as a 4-bit one there and is refused everywhere else before any launch."""
    for bad in (1, 2, 5, 7, 16, -4):
        w = _w()
        w.bits = bad
        assert _lin(w, None) == uq.UNIQL_E_SHAPE
    w4 = _w()
    w4.bits = 4
    assert _lin(w4, None, M=0) == uq.UNIQL_E_SHAPE and _lin(w4, KeepDesc(n_keep=999)) == uq.UNIQL_E_KEEP
    for bits in (8, 6, 3):
        w8 = _w()
        w8.bits = bits
        assert _lin(w8, None, M=0) == uq.UNIQL_E_SHAPE             # validated like any other matrix ...
        assert _lin(w8, KeepDesc(n_keep=999)) == uq.UNIQL_E_KEEP
        assert _lin(w8, None, x=P + 1) == uq.UNIQL_E_ALIGN
        wi = _w()
        wi.bits, wi.col_interleave = bits, 4
        assert _lin(wi, None) == uq.UNIQL_E_SHAPE                  # ... but not head-interleaved
        assert _multi(ws=[_w(), w8]) == uq.UNIQL_E_SHAPE           # and not in the calls that only know 4-bit codes
        W = (W4 * 2)(w8, w8)
        assert uq.lib().uniql_w4_gate_up_silu(W, None, C.c_void_p(P), C.c_void_p(P), None) == uq.UNIQL_E_SHAPE
        assert uq.lib().uniql_w4_dequant(C.byref(w8), None, None, None) == uq.UNIQL_E_NULL   # dequant takes it (and then misses its output)


def test_rope_table_check_on_the_host():
    rng = np.random.default_rng(5)
    good = np.stack([rng.permutation(64)[:54] for _ in range(8)]).astype(np.int32)
    uq.uniql_rope_table_check(good, 128)
    for bad_value, at in ((64, (3, 10)), (-1, (0, 0)), (int(good[7, 0]), (7, 53))):   # too large, negative, repeated
        bad = good.copy()
        bad[at] = bad_value
        with pytest.raises(uq.UniqlError) as e:
            uq.uniql_rope_table_check(bad, 128)
        assert e.value.code == uq.UNIQL_E_KEEP
    with pytest.raises(uq.UniqlError):
        uq.uniql_rope_table_check(good, 100)          # 54 pairs do not fit a head of 100 channels
    assert uq.lib().uniql_rope_table_check(None, 8, 128, 108) == uq.UNIQL_E_NULL
    # the generated tables of the workloads pass
    import workloads as wl
    r = wl.gen_rope_inputs(wl.rng_for(1, 40), wl.llama3_8b_rope(15))
    uq.uniql_rope_table_check(r["kept_idx"], 128)


def test_read_probe_rejects_bad_arguments():
    L = uq.lib()

    def call(src=P, nbytes=4096, out=P):
        return L.uniql_stream_read_probe(C.c_void_p(src), nbytes, C.c_void_p(out), None)
    assert call(src=0) == uq.UNIQL_E_NULL and call(out=0) == uq.UNIQL_E_NULL
    assert call(nbytes=-16) == uq.UNIQL_E_SHAPE
    assert call(src=P + 8) == uq.UNIQL_E_ALIGN and call(out=P + 2) == uq.UNIQL_E_ALIGN


def test_rope_bf16_entry_validates_like_the_fp16_one():
    L = uq.lib()

    def call(fn, q=P, D_keep=108, theta=5e5):
        return fn(C.c_void_p(q), C.c_void_p(P), C.c_void_p(P), C.c_void_p(P), 1, 32, 8, 8, 128, D_keep, theta, None)
    for kw, code in ((dict(q=0), uq.UNIQL_E_NULL), (dict(D_keep=107), uq.UNIQL_E_KEEP), (dict(theta=0.0), uq.UNIQL_E_KEEP),
                     (dict(q=P + 1), uq.UNIQL_E_ALIGN)):
        assert call(L.uniql_pruned_rope_bf16, **kw) == code == call(L.uniql_pruned_rope, **kw)


def test_rope_rejects_bad_arguments():
    assert _rope(q=0) == uq.UNIQL_E_NULL
    assert _rope(pos=0) == uq.UNIQL_E_NULL
    assert _rope(idx=0) == uq.UNIQL_E_NULL
    assert _rope(k=0) == uq.UNIQL_E_NULL                 # Hkv > 0 needs k
    assert _rope(Hkv=0) == uq.UNIQL_E_SHAPE              # k given but Hkv == 0
    assert _rope(T=0) == uq.UNIQL_E_SHAPE
    assert _rope(D_keep=107) == uq.UNIQL_E_KEEP
    assert _rope(D_keep=130) == uq.UNIQL_E_KEEP
    assert _rope(D_keep=0) == uq.UNIQL_E_KEEP
    assert _rope(Hq=7) == uq.UNIQL_E_KEEP
    assert _rope(Hkv=3) == uq.UNIQL_E_KEEP
    assert _rope(theta=0.0) == uq.UNIQL_E_KEEP
    assert _rope(q=P + 1) == uq.UNIQL_E_ALIGN
    assert _rope(pos=P + 2) == uq.UNIQL_E_ALIGN


def _multi(n=2, ws=None, keeps=None, x=P, y=P, ldx=512, ldy=256, M=1):
    ws = ws if ws is not None else [_w() for _ in range(max(n, 1))]
    W = (W4 * len(ws))(*ws)
    K = (KeepDesc * len(ws))(*keeps) if keeps is not None else None
    cnt = len(ws)
    xs = (C.c_void_p * cnt)(*[x] * cnt)
    ys = (C.c_void_p * cnt)(*[y] * cnt)
    lx = (C.c_int64 * cnt)(*[ldx] * cnt)
    ly = (C.c_int64 * cnt)(*[ldy] * cnt)
    return uq.lib().uniql_w4_linear_multi(n, W, K, xs, lx, ys, ly, M, None)


def test_linear_multi_rejects_bad_arguments():
    assert _multi(n=0) == uq.UNIQL_E_SHAPE
    assert _multi(n=5, ws=[_w() for _ in range(5)]) == uq.UNIQL_E_SHAPE
    assert uq.lib().uniql_w4_linear_multi(1, None, None, None, None, None, None, 1, None) == uq.UNIQL_E_NULL
    assert _multi(ws=[_w(), _w(group=64)]) == uq.UNIQL_E_SHAPE           # any invalid entry fails the call
    assert _multi(ws=[_w(), _w(q=P + 8)]) == uq.UNIQL_E_ALIGN
    assert _multi(keeps=[KeepDesc(), KeepDesc(n_keep=257)]) == uq.UNIQL_E_KEEP
    assert _multi(x=0) == uq.UNIQL_E_NULL
    assert _multi(M=0) == uq.UNIQL_E_SHAPE


def _qkv(ws=None, keeps=None, x=P, q=P, k=P, v=P, pos=P, idx=P, Hq=4, Hkv=2, H_tab=2, D_full=64, D_keep=64, theta=1e4):
    ws = ws if ws is not None else [_w(N=Hq * D_full), _w(N=Hkv * D_full), _w(N=Hkv * D_full)]
    W = (W4 * 3)(*ws)
    K = (KeepDesc * 3)(*keeps) if keeps is not None else None
    return uq.lib().uniql_w4_qkv_rope(W, K, C.c_void_p(x), C.c_void_p(q), C.c_void_p(k), C.c_void_p(v),
                                      C.c_void_p(pos), C.c_void_p(idx), Hq, Hkv, H_tab, D_full, D_keep, theta, None)


def test_qkv_rope_rejects_bad_arguments():
    assert uq.lib().uniql_w4_qkv_rope(None, None, C.c_void_p(P), C.c_void_p(P), C.c_void_p(P), C.c_void_p(P),
                                      C.c_void_p(P), C.c_void_p(P), 4, 2, 2, 64, 64, 1e4, None) == uq.UNIQL_E_NULL
    assert _qkv(pos=0) == uq.UNIQL_E_NULL
    assert _qkv(idx=0) == uq.UNIQL_E_NULL
    assert _qkv(x=0) == uq.UNIQL_E_NULL
    assert _qkv(k=0) == uq.UNIQL_E_NULL
    assert _qkv(Hkv=0) == uq.UNIQL_E_SHAPE
    assert _qkv(D_keep=63) == uq.UNIQL_E_KEEP
    assert _qkv(D_keep=66) == uq.UNIQL_E_KEEP
    assert _qkv(H_tab=3) == uq.UNIQL_E_KEEP
    assert _qkv(theta=-1.0) == uq.UNIQL_E_KEEP
    assert _qkv(pos=P + 2) == uq.UNIQL_E_ALIGN
    assert _qkv(D_keep=32) == uq.UNIQL_E_KEEP                            # kept rows of q do not match Hq * D_keep
    assert _qkv(ws=[_w(N=256), _w(N=128), _w(N=128, K=1024)]) == uq.UNIQL_E_SHAPE   # v reads a different x
    assert _qkv(ws=[_w(N=256), _w(N=128, group=64), _w(N=128)]) == uq.UNIQL_E_SHAPE


def _glu(ws=None, keeps=None, x=P, h=P):
    ws = ws if ws is not None else [_w(), _w()]
    W = (W4 * 2)(*ws)
    K = (KeepDesc * 2)(*keeps) if keeps is not None else None
    return uq.lib().uniql_w4_gate_up_silu(W, K, C.c_void_p(x), C.c_void_p(h), None)


def test_gate_up_silu_rejects_bad_arguments():
    assert uq.lib().uniql_w4_gate_up_silu(None, None, C.c_void_p(P), C.c_void_p(P), None) == uq.UNIQL_E_NULL
    assert _glu(x=0) == uq.UNIQL_E_NULL
    assert _glu(h=0) == uq.UNIQL_E_NULL
    assert _glu(ws=[_w(), _w(group=64)]) == uq.UNIQL_E_SHAPE
    assert _glu(h=P + 1) == uq.UNIQL_E_ALIGN
    assert _glu(keeps=[KeepDesc(n_keep=100), KeepDesc(n_keep=101)]) == uq.UNIQL_E_KEEP
    assert _glu(keeps=[KeepDesc(k_keep=100), KeepDesc(k_keep=104)]) == uq.UNIQL_E_KEEP
    assert _glu(ws=[_w(), _w(K=1024)]) == uq.UNIQL_E_KEEP
    assert _glu(keeps=[KeepDesc(col_seg_stride=128, col_seg_keep=64), KeepDesc(k_keep=256)]) == uq.UNIQL_E_KEEP


def _glub(ws=None, keeps=None, x=P, h=P, ldx=512, ldh=512, M=4):
    ws = ws if ws is not None else [_w(), _w()]
    W = (W4 * 2)(*ws)
    K = (KeepDesc * 2)(*keeps) if keeps is not None else None
    return uq.lib().uniql_w4_gate_up_silu_batch(W, K, C.c_void_p(x), ldx, C.c_void_p(h), ldh, M, None)


def test_gate_up_silu_batch_rejects_bad_arguments():
    assert uq.lib().uniql_w4_gate_up_silu_batch(None, None, C.c_void_p(P), 512, C.c_void_p(P), 512, 4, None) == uq.UNIQL_E_NULL
    assert _glub(x=0) == uq.UNIQL_E_NULL
    assert _glub(h=0) == uq.UNIQL_E_NULL
    assert _glub(M=0) == uq.UNIQL_E_SHAPE
    assert _glub(ldx=100) == uq.UNIQL_E_SHAPE                      # shorter than the kept columns
    assert _glub(ws=[_w(), _w(group=64)]) == uq.UNIQL_E_SHAPE
    assert _glub(h=P + 1) == uq.UNIQL_E_ALIGN
    assert _glub(keeps=[KeepDesc(n_keep=100), KeepDesc(n_keep=101)]) == uq.UNIQL_E_KEEP
    assert _glub(keeps=[KeepDesc(k_keep=100), KeepDesc(k_keep=104)]) == uq.UNIQL_E_KEEP
    assert _glub(ws=[_w(), _w(K=1024)], ldx=1024) == uq.UNIQL_E_KEEP


def _emb(w=None, ids=P, n=4, out=P, ld=512):
    w = w if w is not None else _w()
    return uq.lib().uniql_w4_embedding(C.byref(w), C.c_void_p(ids), n, C.c_void_p(out), ld, None)


def test_embedding_rejects_bad_arguments():
    assert uq.lib().uniql_w4_embedding(None, C.c_void_p(P), 1, C.c_void_p(P), 512, None) == uq.UNIQL_E_NULL
    assert _emb(ids=0) == uq.UNIQL_E_NULL
    assert _emb(out=0) == uq.UNIQL_E_NULL
    assert _emb(n=0) == uq.UNIQL_E_SHAPE
    assert _emb(ld=504) == uq.UNIQL_E_SHAPE
    assert _emb(w=_w(group=64)) == uq.UNIQL_E_SHAPE
    assert _emb(ld=516) == uq.UNIQL_E_ALIGN
    assert _emb(out=P + 8) == uq.UNIQL_E_ALIGN
    assert _emb(ids=P + 2) == uq.UNIQL_E_ALIGN


def _repack(w=None, keep=None, oq=P, os_=P, oz=P, N_out=256, K_out=512):
    w = w if w is not None else _w()
    kd = C.byref(keep) if keep is not None else None
    return uq.lib().uniql_w4_repack(C.byref(w), kd, C.c_void_p(oq), C.c_void_p(os_), C.c_void_p(oz), N_out, K_out, None)


def test_repack_rejects_bad_arguments():
    assert uq.lib().uniql_w4_repack(None, None, C.c_void_p(P), C.c_void_p(P), C.c_void_p(P), 256, 512, None) == uq.UNIQL_E_NULL
    assert _repack(oq=0) == uq.UNIQL_E_NULL
    assert _repack(os_=0) == uq.UNIQL_E_NULL
    assert _repack(oz=0) == uq.UNIQL_E_NULL
    assert _repack(w=_w(group=64)) == uq.UNIQL_E_SHAPE
    assert _repack(N_out=255) == uq.UNIQL_E_SHAPE                        # not the size of the plan
    assert _repack(keep=KeepDesc(k_keep=300), K_out=512) == uq.UNIQL_E_SHAPE   # the plan says 384
    assert _repack(keep=KeepDesc(n_keep=300)) == uq.UNIQL_E_KEEP
    assert _repack(oq=P + 8) == uq.UNIQL_E_ALIGN
    assert _repack(os_=P + 1) == uq.UNIQL_E_ALIGN
    n, k, ko = C.c_int32(), C.c_int32(), KeepDesc()
    w = _w()
    assert uq.lib().uniql_w4_repack_plan(C.byref(w), None, None, C.byref(k), C.byref(ko)) == uq.UNIQL_E_NULL
    assert uq.lib().uniql_w4_repack_plan(None, None, C.byref(n), C.byref(k), C.byref(ko)) == uq.UNIQL_E_NULL
    bad = KeepDesc(col_seg_stride=96, col_seg_keep=200)
    assert uq.lib().uniql_w4_repack_plan(C.byref(w), C.byref(bad), C.byref(n), C.byref(k), C.byref(ko)) == uq.UNIQL_E_KEEP


def test_interleave_and_deinterleave_reject_bad_arguments():
    """The two word permutations validate before any launch: NULL, a matrix in the wrong storage order, head counts that do not
    cut the row into whole words, alignment; valid arguments get as far as the architecture check."""
    lib = uq.lib()
    il = lambda w, heads, out=P: lib.uniql_w4_interleave(C.byref(w) if w is not None else None, heads, C.c_void_p(out), None)
    de = lambda w, out=P: lib.uniql_w4_deinterleave(C.byref(w) if w is not None else None, C.c_void_p(out), None)
    plain, inter = _w(K=1024), _w(K=1024)
    inter.col_interleave = 8
    assert il(None, 8) == uq.UNIQL_E_NULL and de(None) == uq.UNIQL_E_NULL
    assert il(plain, 8, out=0) == uq.UNIQL_E_NULL and de(inter, out=0) == uq.UNIQL_E_NULL
    assert il(inter, 8) == uq.UNIQL_E_SHAPE                 # already interleaved
    assert de(plain) == uq.UNIQL_E_SHAPE                    # nothing to undo
    assert il(plain, 0) == uq.UNIQL_E_SHAPE and il(plain, 7) == uq.UNIQL_E_SHAPE and il(plain, 256) == uq.UNIQL_E_SHAPE
    bad = _w(K=1024)
    bad.col_interleave = 7                                  # a descriptor that claims an impossible head count
    assert de(bad) == uq.UNIQL_E_SHAPE
    assert il(plain, 8, out=P + 8) == uq.UNIQL_E_ALIGN and de(inter, out=P + 8) == uq.UNIQL_E_ALIGN
    assert il(_w(K=1024, group=64), 8) == uq.UNIQL_E_SHAPE
    import torch
    if not torch.cuda.is_available():
        assert il(plain, 8) in (uq.UNIQL_E_HIP, uq.UNIQL_E_ARCH) and de(inter) in (uq.UNIQL_E_HIP, uq.UNIQL_E_ARCH)


def test_repack_plan_matches_the_oracle(uref):
    """The plan is host arithmetic (closed forms); the oracle derives it by scanning rows, columns and
    groups one by one."""
    rng = np.random.default_rng(11)
    cases = [(1024, 1024, (870, 0, 0, 0, 0, 0, 0)), (4096, 14336, (0, 12185, 0, 0, 0, 0, 0)),
             (4096, 4096, (0, 0, 0, 0, 0, 128, 108)), (4096, 4096, (3456, 0, 64, 54, 4096, 0, 0)),
             (10576, 2560, (9040, 0, 5120, 4352, 10240, 0, 0)), (64, 1024, (0, 768, 0, 0, 0, 0, 0)),
             (64, 1024, None), (16, 2048, (0, 0, 0, 0, 0, 512, 200)), (16, 2048, (0, 0, 0, 0, 0, 256, 256)),
             (16, 768, (0, 0, 0, 0, 0, 192, 10)), (16, 512, (0, 0, 0, 0, 0, 64, 54)), (8, 512, (0, 3, 0, 0, 0, 0, 0))]
    for _ in range(60):
        K = 128 * int(rng.integers(1, 24))
        N = int(rng.integers(1, 300))
        kind = int(rng.integers(0, 3))
        keep = [0] * 7
        if rng.integers(0, 2):
            keep[0] = int(rng.integers(1, N + 1))
        if kind == 1:
            keep[1] = int(rng.integers(1, K + 1))
        elif kind == 2:
            divs = [d for d in range(8, K + 1) if K % d == 0]
            keep[5] = int(rng.choice(divs))
            keep[6] = int(rng.integers(1, keep[5] + 1))
        cases.append((N, K, tuple(keep)))
    for N, K, keep in cases:
        n, k, ko = uq.uniql_w4_repack_plan(N, K, keep)
        en, ek, eko = uref.w4_repack_plan(N, K, keep)
        got = (ko.n_keep, ko.k_keep, ko.row_seg_stride, ko.row_seg_keep, ko.row_seg_limit, ko.col_seg_stride, ko.col_seg_keep)
        # k_keep = 0 and k_keep = the full count name the same columns
        norm = lambda t, kk: tuple(t[:1]) + ((0,) if t[1] in (0, kk) and t[5] == 0 else (t[1],)) + tuple(t[2:])
        assert (n, k) == (en, ek), (N, K, keep)
        assert norm(got, k) == norm(eko, ek), (N, K, keep, got, eko)


def test_valid_arguments_without_gfx950_fail_loudly():
    """On a box without an MI355X a valid call must report E_HIP / E_ARCH, never pretend to work."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present; covered by the gpu tests")
    assert _lin(_w(), None) in (uq.UNIQL_E_HIP, uq.UNIQL_E_ARCH)
    assert _rope() in (uq.UNIQL_E_HIP, uq.UNIQL_E_ARCH)
    assert _multi() in (uq.UNIQL_E_HIP, uq.UNIQL_E_ARCH)
    assert _qkv() in (uq.UNIQL_E_HIP, uq.UNIQL_E_ARCH)
    assert _glu() in (uq.UNIQL_E_HIP, uq.UNIQL_E_ARCH)
    assert _emb() in (uq.UNIQL_E_HIP, uq.UNIQL_E_ARCH)
    assert _repack() in (uq.UNIQL_E_HIP, uq.UNIQL_E_ARCH)
