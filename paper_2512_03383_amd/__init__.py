"""Thin Python binding of libuniql (the C ABI in include/uniql.h).

Argument marshalling only: every step of the hot path runs in the HIP kernels
behind the C ABI.  PyTorch is used for device memory and streams.  There is no
CPU fallback: if the library has not been built, importing a function that
needs it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libuniql.so")
HEADER_PATH = os.path.join(os.path.dirname(_HERE), "include", "uniql.h")

UNIQL_OK = 0
UNIQL_E_NULL, UNIQL_E_SHAPE, UNIQL_E_KEEP, UNIQL_E_ALIGN, UNIQL_E_ARCH, UNIQL_E_HIP = -1, -2, -3, -4, -5, -6


class UniqlError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"uniql error {code}: {msg}")
        self.code = code


class W4(C.Structure):
    """uniql_w4_t"""
    _fields_ = [("qweight", C.c_void_p), ("scales", C.c_void_p), ("zeros", C.c_void_p),
                ("N_total", C.c_int32), ("K_total", C.c_int32), ("group", C.c_int32), ("dtype", C.c_int32),
                ("col_interleave", C.c_int32), ("bits", C.c_int32)]


UNIQL_F16, UNIQL_BF16 = 0, 1


class KeepDesc(C.Structure):
    """uniql_keep_t"""
    _fields_ = [("n_keep", C.c_int32), ("k_keep", C.c_int32),
                ("row_seg_stride", C.c_int32), ("row_seg_keep", C.c_int32), ("row_seg_limit", C.c_int32),
                ("col_seg_stride", C.c_int32), ("col_seg_keep", C.c_int32),
                ("row_seg2_stride", C.c_int32), ("row_seg2_keep", C.c_int32), ("row_seg2_limit", C.c_int32)]


_lib = None


def build() -> str:
    from .build import build_lib
    global _lib
    _lib = None
    return build_lib()


def lib():
    """Load libuniql.so (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it first (python -m paper_2512_03383_amd.build); "
                "there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
        L.uniql_w4_linear.restype = C.c_int
        L.uniql_w4_linear.argtypes = [C.POINTER(W4), C.POINTER(KeepDesc), vp, i64, vp, i64, i32, vp]
        L.uniql_w4_linear_multi.restype = C.c_int
        L.uniql_w4_linear_multi.argtypes = [i32, C.POINTER(W4), C.POINTER(KeepDesc), C.POINTER(vp), C.POINTER(i64),
                                            C.POINTER(vp), C.POINTER(i64), i32, vp]
        L.uniql_w4_dequant.restype = C.c_int
        L.uniql_w4_dequant.argtypes = [C.POINTER(W4), C.POINTER(KeepDesc), vp, vp]
        L.uniql_pruned_rope.restype = C.c_int
        L.uniql_pruned_rope.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, C.c_double, vp]
        L.uniql_pruned_rope_bf16.restype = C.c_int
        L.uniql_pruned_rope_bf16.argtypes = L.uniql_pruned_rope.argtypes
        L.uniql_rope_table_check.restype = C.c_int
        L.uniql_rope_table_check.argtypes = [vp, i32, i32, i32]
        L.uniql_stream_read_probe.restype = C.c_int
        L.uniql_w4_qkv_rope.restype = C.c_int
        L.uniql_w4_qkv_rope.argtypes = [C.POINTER(W4), C.POINTER(KeepDesc), vp, vp, vp, vp, vp, vp,
                                        i32, i32, i32, i32, i32, C.c_double, vp]
        L.uniql_w4_gate_up_silu.restype = C.c_int
        L.uniql_w4_gate_up_silu.argtypes = [C.POINTER(W4), C.POINTER(KeepDesc), vp, vp, vp]
        L.uniql_w4_gate_up_silu_batch.restype = C.c_int
        L.uniql_w4_gate_up_silu_batch.argtypes = [C.POINTER(W4), C.POINTER(KeepDesc), vp, i64, vp, i64, i32, vp]
        L.uniql_w4_interleave.restype = C.c_int
        L.uniql_w4_interleave.argtypes = [C.POINTER(W4), i32, vp, vp]
        L.uniql_w4_deinterleave.restype = C.c_int
        L.uniql_w4_deinterleave.argtypes = [C.POINTER(W4), vp, vp]
        L.uniql_w4_mlp.restype = C.c_int
        L.uniql_w4_mlp.argtypes = [C.POINTER(W4), C.POINTER(KeepDesc), vp, vp, vp, i64, vp]
        L.uniql_w4_mlp_static.restype = C.c_int
        L.uniql_w4_mlp_static.argtypes = [C.POINTER(W4), C.POINTER(KeepDesc), vp, vp, vp]
        L.uniql_w4_mlp_static_max_hidden.restype = i32
        L.uniql_w4_mlp_workspace_bytes.restype = i64
        L.uniql_w4_mlp_workspace_bytes.argtypes = [i32]
        L.uniql_w4_mlp_hidden.restype = C.c_int
        L.uniql_w4_mlp_hidden.argtypes = [vp, i32, C.POINTER(vp)]
        L.uniql_w4_mlp_status.restype = C.c_int
        L.uniql_w4_mlp_status.argtypes = [vp, C.POINTER(C.c_uint32), vp]
        L.uniql_w4_gate_up_stream_probe.restype = C.c_int
        L.uniql_w4_gate_up_stream_probe.argtypes = [C.POINTER(W4), C.POINTER(KeepDesc), vp, vp, vp]
        L.uniql_w4_embedding.restype = C.c_int
        L.uniql_w4_embedding.argtypes = [C.POINTER(W4), vp, i32, vp, i64, vp]
        L.uniql_w4_repack_plan.restype = C.c_int
        L.uniql_w4_repack_plan.argtypes = [C.POINTER(W4), C.POINTER(KeepDesc), C.POINTER(i32), C.POINTER(i32),
                                           C.POINTER(KeepDesc)]
        L.uniql_w4_repack.restype = C.c_int
        L.uniql_w4_repack.argtypes = [C.POINTER(W4), C.POINTER(KeepDesc), vp, vp, vp, i32, i32, vp]
        L.uniql_stream_read_probe.argtypes = [vp, i64, vp, vp]
        L.uniql_strerror.restype = C.c_char_p
        L.uniql_strerror.argtypes = [C.c_int]
        L.uniql_last_hip_error.restype = C.c_int
        L.uniql_version.restype = C.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().uniql_strerror(int(code)).decode()


def _check(code: int) -> None:
    if code != UNIQL_OK:
        msg = strerror(code)
        if code == UNIQL_E_HIP:
            msg += f" [hipError {lib().uniql_last_hip_error()}]"
        raise UniqlError(code, msg)


def _keep_desc(keep) -> Optional[KeepDesc]:
    if keep is None:
        return None
    if isinstance(keep, KeepDesc):
        return keep
    t = keep.as_tuple() if hasattr(keep, "as_tuple") else tuple(keep)
    return KeepDesc(*[int(v) for v in t])


def _stream_ptr(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


@dataclass
class QuantLinear:
    """Device tensors of one quantised linear (torch owns the memory)."""
    qweight: "torch.Tensor"   # int32 [N][K/8] (bit pattern of the uint32 words)
    scales: "torch.Tensor"    # float16 or bfloat16 [N][K/128]: the format of activations and outputs too
    zeros: "Optional[torch.Tensor]"     # uint8 [N][K/128], or None: symmetric scheme, every zero point 8
    col_interleave: int = 0   # > 0: the words of a row are stored head-interleaved over this many heads
    bits: int = 4             # width of a code: 4, or 8 / 6 / 3 (then qweight is [N][K * bits / 32], zeros 0..2^bits - 1 or None = 2^(bits-1))

    @property
    def N(self) -> int:
        return self.qweight.shape[0]

    @property
    def K(self) -> int:
        return self.qweight.shape[1] * 32 // self.bits

    @property
    def ftype(self):
        """torch dtype of the scales = of the activations and outputs that go with this matrix."""
        import torch
        assert self.scales.dtype in (torch.float16, torch.bfloat16)
        return self.scales.dtype

    def desc(self) -> W4:
        import torch
        return W4(self.qweight.data_ptr(), self.scales.data_ptr(),
                  self.zeros.data_ptr() if self.zeros is not None else None, self.N, self.K, 128,
                  UNIQL_BF16 if self.ftype == torch.bfloat16 else UNIQL_F16, int(self.col_interleave), int(self.bits))

    @staticmethod
    def from_numpy(w: dict, device="cuda", bits: int = 4) -> "QuantLinear":
        import numpy as np
        import torch
        scales = w["scales"]      # float16, or uint16 bit patterns of bfloat16
        scales = (torch.from_numpy(scales.view(np.int16)).view(torch.bfloat16) if scales.dtype == np.uint16
                  else torch.from_numpy(scales))
        return QuantLinear(torch.from_numpy(w["qweight"].view(np.int32)).to(device),
                           scales.to(device),
                           torch.from_numpy(w["zeros"]).to(device) if w.get("zeros") is not None else None, bits=bits)


def kept_dims(W: QuantLinear, keep) -> tuple:
    """(n_keep, k_keep) the descriptor yields (same rule as the C ABI)."""
    kd = _keep_desc(keep) or KeepDesc()
    if kd.row_seg_stride:
        n = (kd.row_seg_limit // kd.row_seg_stride) * kd.row_seg_keep
        tail_from = kd.row_seg_limit
        if kd.row_seg2_stride:
            n += ((kd.row_seg2_limit - kd.row_seg_limit) // kd.row_seg2_stride) * kd.row_seg2_keep
            tail_from = kd.row_seg2_limit
        n += W.N - tail_from
    else:
        n = kd.n_keep or W.N
    if kd.col_seg_stride:
        k = (W.K // kd.col_seg_stride) * kd.col_seg_keep
    else:
        k = kd.k_keep or W.K
    return n, k


def uniql_w4_linear(W: QuantLinear, keep, x, y=None, stream=None):
    """y[M][n_keep] = x[M][k_keep] @ W'^T on the current device; returns y."""
    import torch
    n_keep, k_keep = kept_dims(W, keep)
    assert x.dtype == W.ftype and x.is_cuda and x.dim() == 2 and x.stride(1) == 1
    M = x.shape[0]
    if y is None:
        y = torch.empty((M, n_keep), dtype=W.ftype, device=x.device)
    assert y.dtype == W.ftype and y.is_cuda and y.stride(1) == 1
    d, kd = W.desc(), _keep_desc(keep)
    rc = lib().uniql_w4_linear(C.byref(d), C.byref(kd) if kd is not None else None,
                               C.c_void_p(x.data_ptr()), x.stride(0), C.c_void_p(y.data_ptr()), y.stride(0),
                               M, _stream_ptr(stream))
    _check(rc)
    return y


class MultiCall:
    """Marshalled arguments of one uniql_w4_linear_multi call, reusable (e.g. for graph capture)."""

    def __init__(self, Ws, keeps, xs, ys):
        n = len(Ws)
        assert 1 <= n <= 4 and len(keeps) == n and len(xs) == n and len(ys) == n
        self.n = n
        self.M = xs[0].shape[0]
        self.W = (W4 * n)(*[w.desc() for w in Ws])
        self.keep = (KeepDesc * n)(*[(_keep_desc(k) or KeepDesc()) for k in keeps])
        self.x = (C.c_void_p * n)(*[t.data_ptr() for t in xs])
        self.y = (C.c_void_p * n)(*[t.data_ptr() for t in ys])
        self.ldx = (C.c_int64 * n)(*[t.stride(0) for t in xs])
        self.ldy = (C.c_int64 * n)(*[t.stride(0) for t in ys])
        self._refs = (Ws, xs, ys)      # keep the tensors alive

    def run(self, stream=None):
        rc = lib().uniql_w4_linear_multi(self.n, self.W, self.keep, self.x, self.ldx, self.y, self.ldy, self.M,
                                         _stream_ptr(stream))
        _check(rc)


def uniql_w4_linear_multi(Ws, keeps, xs, ys, stream=None):
    """Several independent linears with the same token count in one call; ys are written in place."""
    for W, x, y in zip(Ws, xs, ys):
        assert x.dtype == W.ftype and y.dtype == W.ftype and x.stride(1) == 1 and y.stride(1) == 1
        assert x.shape[0] == xs[0].shape[0]
    MultiCall(Ws, keeps, xs, ys).run(stream)
    return ys


def uniql_w4_dequant(W: QuantLinear, keep=None, out=None, stream=None):
    """[n_keep][k_keep] bit-exact dequantised weights, in the format of the scales."""
    import torch
    n_keep, k_keep = kept_dims(W, keep)
    if out is None:
        out = torch.empty((n_keep, k_keep), dtype=W.ftype, device=W.qweight.device)
    assert out.is_contiguous() and out.dtype == W.ftype
    d, kd = W.desc(), _keep_desc(keep)
    rc = lib().uniql_w4_dequant(C.byref(d), C.byref(kd) if kd is not None else None,
                                C.c_void_p(out.data_ptr()), _stream_ptr(stream))
    _check(rc)
    return out


def uniql_w4_repack_plan(N_total: int, K_total: int, keep=None):
    """(N_out, K_out, keep_out) of the compact matrix uniql_w4_repack writes (host only, no GPU)."""
    d = W4(None, None, None, int(N_total), int(K_total), 128)
    kd = _keep_desc(keep)
    n, k, ko = C.c_int32(0), C.c_int32(0), KeepDesc()
    _check(lib().uniql_w4_repack_plan(C.byref(d), C.byref(kd) if kd is not None else None, C.byref(n), C.byref(k),
                                      C.byref(ko)))
    return n.value, k.value, ko


def uniql_w4_repack(W: QuantLinear, keep=None, out: Optional[QuantLinear] = None, stream=None):
    """Compact copy of the kept channels: returns (QuantLinear, KeepDesc to use with it).  `out` may
    bring tensors of the plan's sizes (contiguous); otherwise they are allocated."""
    import torch
    n_out, k_out, ko = uniql_w4_repack_plan(W.N, W.K, keep)
    dev = W.qweight.device
    if out is None:
        out = QuantLinear(torch.empty((n_out, k_out // 8), dtype=torch.int32, device=dev),
                          torch.empty((n_out, k_out // 128), dtype=W.ftype, device=dev),
                          torch.empty((n_out, k_out // 128), dtype=torch.uint8, device=dev) if W.zeros is not None else None)
    assert out.qweight.shape == (n_out, k_out // 8) and out.scales.shape == (n_out, k_out // 128) \
        and (W.zeros is None or out.zeros.shape == out.scales.shape)
    assert out.qweight.is_contiguous() and out.scales.is_contiguous() and (W.zeros is None or out.zeros.is_contiguous())
    assert out.scales.dtype == W.ftype
    d, kd = W.desc(), _keep_desc(keep)
    _check(lib().uniql_w4_repack(C.byref(d), C.byref(kd) if kd is not None else None,
                                 C.c_void_p(out.qweight.data_ptr()), C.c_void_p(out.scales.data_ptr()),
                                 C.c_void_p(out.zeros.data_ptr()) if W.zeros is not None else None, n_out, k_out,
                                 _stream_ptr(stream)))
    return out, ko


def uniql_w4_embedding(W: QuantLinear, ids, out=None, stream=None):
    """[len(ids)][K] dequantised rows ids (int32 device tensor) of the quantised table W, in the format of its scales."""
    import torch
    assert ids.dtype == torch.int32 and ids.is_cuda and ids.is_contiguous() and ids.dim() == 1
    if out is None:
        out = torch.empty((ids.shape[0], W.K), dtype=W.ftype, device=ids.device)
    assert out.dtype == W.ftype and out.stride(1) == 1 and out.shape == (ids.shape[0], W.K)
    d = W.desc()
    _check(lib().uniql_w4_embedding(C.byref(d), C.c_void_p(ids.data_ptr()), ids.shape[0], C.c_void_p(out.data_ptr()),
                                    out.stride(0), _stream_ptr(stream)))
    return out


def uniql_pruned_rope(q, k, positions, kept_idx, D_full: int, theta: float, stream=None):
    """Rotate q [T][Hq][D_keep] and k [T][Hkv][D_keep] (or None) in place (float16 or bfloat16 tensors)."""
    import torch
    assert q.dtype in (torch.float16, torch.bfloat16) and q.is_cuda and q.is_contiguous() and q.dim() == 3
    T, Hq, Dk = q.shape
    Hkv = 0
    if k is not None:
        assert k.dtype == q.dtype and k.is_contiguous() and k.shape[0] == T and k.shape[2] == Dk
        Hkv = k.shape[1]
    assert positions.dtype == torch.int32 and positions.shape == (T,) and positions.is_contiguous()
    assert kept_idx.dtype == torch.int32 and kept_idx.is_contiguous() and kept_idx.shape[1] == Dk // 2
    fn = lib().uniql_pruned_rope_bf16 if q.dtype == torch.bfloat16 else lib().uniql_pruned_rope
    rc = fn(C.c_void_p(q.data_ptr()), C.c_void_p(k.data_ptr()) if k is not None else None,
            C.c_void_p(positions.data_ptr()), C.c_void_p(kept_idx.data_ptr()),
            T, Hq, Hkv, kept_idx.shape[0], D_full, Dk, float(theta), _stream_ptr(stream))
    _check(rc)
    return q, k


def uniql_rope_table_check(kept_idx, D_full: int) -> None:
    """Raise UniqlError unless the kept-index table (numpy or CPU tensor, int32 [H_tab][D_keep / 2]) holds distinct
    entries below D_full / 2 in every row -- what the rotary kernels assume without checking.  Host only."""
    import numpy as np
    a = np.ascontiguousarray(kept_idx.cpu().numpy() if hasattr(kept_idx, "cpu") else kept_idx)
    assert a.dtype == np.int32 and a.ndim == 2
    _check(lib().uniql_rope_table_check(a.ctypes.data_as(C.c_void_p), a.shape[0], int(D_full), 2 * a.shape[1]))


class QkvRopeCall:
    """Marshalled arguments of one uniql_w4_qkv_rope call, reusable (e.g. for graph capture):
    q, k, v projections of one token and the rotation of q and k in one launch."""

    def __init__(self, Ws, keeps, x, q, k, v, position, kept_idx, D_full: int, theta: float):
        import torch
        assert len(Ws) == 3 and len(keeps) == 3
        for t in (x, q, k, v):
            assert t.dtype == Ws[0].ftype and t.is_cuda and t.is_contiguous()
        assert q.dim() == 2 and k.dim() == 2 and q.shape[1] == k.shape[1], "q [Hq][D_keep], k [Hkv][D_keep]"
        assert position.dtype == torch.int32 and position.numel() == 1
        assert kept_idx.dtype == torch.int32 and kept_idx.is_contiguous() and kept_idx.shape[1] == q.shape[1] // 2
        self.W = (W4 * 3)(*[w.desc() for w in Ws])
        self.keep = (KeepDesc * 3)(*[(_keep_desc(kp) or KeepDesc()) for kp in keeps])
        self.args = (C.c_void_p(x.data_ptr()), C.c_void_p(q.data_ptr()), C.c_void_p(k.data_ptr()),
                     C.c_void_p(v.data_ptr()), C.c_void_p(position.data_ptr()), C.c_void_p(kept_idx.data_ptr()),
                     q.shape[0], k.shape[0], kept_idx.shape[0], int(D_full), q.shape[1], float(theta))
        self._refs = (Ws, x, q, k, v, position, kept_idx)

    def run(self, stream=None):
        _check(lib().uniql_w4_qkv_rope(self.W, self.keep, *self.args, _stream_ptr(stream)))


def uniql_w4_qkv_rope(Ws, keeps, x, position, kept_idx, Hq: int, Hkv: int, D_full: int, D_keep: int, theta: float,
                      stream=None):
    """q = RoPE(x Wq'), k = RoPE(x Wk'), v = x Wv' for one token x [k_keep]; returns q [Hq][D_keep],
    k [Hkv][D_keep], v [n_keep of v]."""
    import torch
    q = torch.empty((Hq, D_keep), dtype=x.dtype, device=x.device)
    k = torch.empty((Hkv, D_keep), dtype=x.dtype, device=x.device)
    v = torch.empty((kept_dims(Ws[2], keeps[2])[0],), dtype=x.dtype, device=x.device)
    QkvRopeCall(Ws, keeps, x, q, k, v, position, kept_idx, D_full, theta).run(stream)
    return q, k, v


class GateUpCall:
    """Marshalled arguments of one uniql_w4_gate_up_silu call, reusable (e.g. for graph capture)."""

    def __init__(self, Ws, keeps, x, h):
        import torch
        assert len(Ws) == 2 and len(keeps) == 2
        for t in (x, h):
            assert t.dtype == Ws[0].ftype and t.is_cuda and t.is_contiguous() and t.dim() == 1
        self.W = (W4 * 2)(*[w.desc() for w in Ws])
        self.keep = (KeepDesc * 2)(*[(_keep_desc(kp) or KeepDesc()) for kp in keeps])
        self.x, self.h = C.c_void_p(x.data_ptr()), C.c_void_p(h.data_ptr())
        self._refs = (Ws, x, h)

    def run(self, stream=None):
        _check(lib().uniql_w4_gate_up_silu(self.W, self.keep, self.x, self.h, _stream_ptr(stream)))

    def run_probe(self, stream=None):
        """uniql_w4_gate_up_stream_probe on the same arguments (measurement aid: h receives meaningless words)."""
        _check(lib().uniql_w4_gate_up_stream_probe(self.W, self.keep, self.x, self.h, _stream_ptr(stream)))


def uniql_w4_gate_up_silu(Ws, keeps, x, h=None, stream=None):
    """h = SiLU(x W_gate') * (x W_up') for one token x [k_keep]; returns h [n_keep]."""
    import torch
    if h is None:
        h = torch.empty((kept_dims(Ws[0], keeps[0])[0],), dtype=x.dtype, device=x.device)
    GateUpCall(Ws, keeps, x, h).run(stream)
    return h


def uniql_w4_gate_up_silu_batch(Ws, keeps, x, h=None, stream=None):
    """h[m] = SiLU(x[m] W_gate') * (x[m] W_up') for the tokens of a decode batch, x [M][k_keep]; returns h [M][n_keep]."""
    import torch
    assert len(Ws) == 2 and len(keeps) == 2 and x.dim() == 2 and x.stride(1) == 1 and x.dtype == Ws[0].ftype
    if h is None:
        h = torch.empty((x.shape[0], kept_dims(Ws[0], keeps[0])[0]), dtype=x.dtype, device=x.device)
    assert h.dim() == 2 and h.stride(1) == 1 and h.dtype == x.dtype and h.shape[0] == x.shape[0]
    W = (W4 * 2)(*[w.desc() for w in Ws])
    kd = (KeepDesc * 2)(*[(_keep_desc(kp) or KeepDesc()) for kp in keeps])
    _check(lib().uniql_w4_gate_up_silu_batch(W, kd, C.c_void_p(x.data_ptr()), x.stride(0), C.c_void_p(h.data_ptr()),
                                             h.stride(0), x.shape[0], _stream_ptr(stream)))
    return h


def uniql_w4_interleave(W: QuantLinear, heads: int, stream=None) -> QuantLinear:
    """The same matrix with the words of every row in head-interleaved order (shares scales and zero points with W)."""
    import torch
    out = torch.empty_like(W.qweight)
    _check(lib().uniql_w4_interleave(C.byref(W.desc()), int(heads), C.c_void_p(out.data_ptr()), _stream_ptr(stream)))
    return QuantLinear(out, W.scales, W.zeros, int(heads))


def uniql_w4_deinterleave(W: QuantLinear, stream=None) -> QuantLinear:
    """The same matrix with the words of every row back in column order (shares scales and zero points with W)."""
    import torch
    out = torch.empty_like(W.qweight)
    _check(lib().uniql_w4_deinterleave(C.byref(W.desc()), C.c_void_p(out.data_ptr()), _stream_ptr(stream)))
    return QuantLinear(out, W.scales, W.zeros, 0)


def mlp_workspace(n_hidden_keep: int, device="cuda"):
    """Zero-filled workspace for uniql_w4_mlp (uint8 tensor; reusable by calls that do not overlap on the device)."""
    import torch
    return torch.zeros(int(lib().uniql_w4_mlp_workspace_bytes(int(n_hidden_keep))), dtype=torch.uint8, device=device)


def mlp_hidden(workspace, n_hidden_keep: int, dtype):
    """View of the hidden vector the last uniql_w4_mlp call left in its workspace (for tests)."""
    p = C.c_void_p(0)
    _check(lib().uniql_w4_mlp_hidden(C.c_void_p(workspace.data_ptr()), int(n_hidden_keep), C.byref(p)))
    off = int(p.value) - workspace.data_ptr()
    return workspace[off:off + 2 * int(n_hidden_keep)].view(dtype)


class MlpCall:
    """Marshalled arguments of one uniql_w4_mlp call, reusable (e.g. for graph capture)."""

    def __init__(self, Ws, keeps, x, y, workspace):
        assert len(Ws) == 3 and len(keeps) == 3
        for t in (x, y):
            assert t.dtype == Ws[0].ftype and t.is_cuda and t.is_contiguous() and t.dim() == 1
        assert workspace.is_cuda and workspace.is_contiguous() and workspace.element_size() == 1
        self.W = (W4 * 3)(*[w.desc() for w in Ws])
        self.keep = (KeepDesc * 3)(*[(_keep_desc(kp) or KeepDesc()) for kp in keeps])
        self.x, self.y = C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr())
        self.ws, self.ws_bytes = C.c_void_p(workspace.data_ptr()), int(workspace.numel())
        self._refs = (Ws, x, y, workspace)

    def run(self, stream=None):
        _check(lib().uniql_w4_mlp(self.W, self.keep, self.x, self.y, self.ws, self.ws_bytes, _stream_ptr(stream)))


def uniql_w4_mlp(Ws, keeps, x, workspace, y=None, stream=None):
    """y = W_down' (SiLU(W_gate' x) * (W_up' x)) for one token x [k_keep]; Ws = (gate, up, down); returns y."""
    import torch
    if y is None:
        y = torch.empty((kept_dims(Ws[2], keeps[2])[0],), dtype=x.dtype, device=x.device)
    MlpCall(Ws, keeps, x, y, workspace).run(stream)
    return y


def uniql_w4_mlp_static(Ws, keeps, x, y=None, stream=None):
    """uniql_w4_mlp on the library's own static workspace (allocates nothing when y is given)."""
    import torch
    assert len(Ws) == 3 and len(keeps) == 3
    if y is None:
        y = torch.empty((kept_dims(Ws[2], keeps[2])[0],), dtype=x.dtype, device=x.device)
    for t in (x, y):
        assert t.dtype == Ws[0].ftype and t.is_cuda and t.is_contiguous() and t.dim() == 1
    Wd = (W4 * 3)(*[w.desc() for w in Ws])
    kd = (KeepDesc * 3)(*[(_keep_desc(kp) or KeepDesc()) for kp in keeps])
    _check(lib().uniql_w4_mlp_static(Wd, kd, C.c_void_p(x.data_ptr()), C.c_void_p(y.data_ptr()), _stream_ptr(stream)))
    return y


def uniql_w4_mlp_status(workspace, stream=None) -> int:
    """0 when no call on this workspace gave up waiting for the other blocks, else the serial number of the last that did."""
    out = C.c_uint32(0)
    _check(lib().uniql_w4_mlp_status(C.c_void_p(workspace.data_ptr()), C.byref(out), _stream_ptr(stream)))
    return int(out.value)


def uniql_stream_read_probe(src, nbytes: int, out, stream=None):
    """Read nbytes of the tensor src once (measurement aid: the read-stream ceiling).  out (int32) receives
    one word per 8 KB read."""
    assert src.is_cuda and out.is_cuda and out.is_contiguous() and out.element_size() == 4
    assert 0 <= int(nbytes) <= src.numel() * src.element_size(), "reads past the end of src"
    assert out.numel() >= (int(nbytes) + 8191) // 8192, "out needs one 32-bit word per 8 KB read"
    rc = lib().uniql_stream_read_probe(C.c_void_p(src.data_ptr()), int(nbytes), C.c_void_p(out.data_ptr()),
                                       _stream_ptr(stream))
    _check(rc)
