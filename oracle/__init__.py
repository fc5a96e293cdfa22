"""ctypes access to the CPU oracle (oracle/uref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg; never by the product package.  The arithmetic of
the single operations is in uref.c; two functions here compose them, in fp64:
qkv_rope (three linears, then the rotation of Sec. 3.4 on their fp64 outputs)
and gate_up_silu (two linears, then Eq. 1's SiLU(g) * u in numpy).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "uref.c")
# UREF_SANITIZE=1 in the environment: a second library built with AddressSanitizer and UndefinedBehaviorSanitizer
# (run the pins with it as  UREF_SANITIZE=1 LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0
# python -m pytest tests -m "not gpu"; the interpreter itself is not instrumented, so the runtime has to be preloaded)
_SAN = os.environ.get("UREF_SANITIZE", "") not in ("", "0")
_LIB = os.path.join(_HERE, "liburef_san.so" if _SAN else "liburef.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile uref.c with gcc into oracle/liburef.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        flags = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"] if _SAN else ["-O2"]
        subprocess.check_call(["gcc", *flags, "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
            build(force=True)
        L = C.CDLL(_LIB)
        vp, i32, i64, dbl = C.c_void_p, C.c_int, C.c_int64, C.c_double
        L.uref_half_to_double.restype = dbl
        L.uref_half_to_double.argtypes = [C.c_uint16]
        L.uref_double_to_half.restype = C.c_uint16
        L.uref_double_to_half.argtypes = [dbl]
        L.uref_bf16_to_double.restype = dbl
        L.uref_bf16_to_double.argtypes = [C.c_uint16]
        L.uref_double_to_bf16.restype = C.c_uint16
        L.uref_double_to_bf16.argtypes = [dbl]
        L.uref_w4_dequant_fmt.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, i32]
        L.uref_w4_linear_fmt.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, i64, vp, i64, i32, vp, i32, i32]
        L.uref_w4_linear_il.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, i64, vp, i64, i32, vp, i32, i32, i32]
        L.uref_w4_dequant_il.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, i32, i32]
        L.uref_w4_interleave.argtypes = [vp, i32, i32, i32, vp]
        L.uref_w4_deinterleave.argtypes = [vp, i32, i32, i32, vp]
        L.uref_w4_embedding_fmt.argtypes = [vp, vp, vp, i32, i32, i32, vp, i32, vp, i32]
        L.uref_pruned_rope_fmt.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, dbl, vp, vp, i32]
        L.uref_set_threads.argtypes = [i32]
        L.uref_get_max_threads.restype = i32
        L.uref_count_kept.argtypes = [i32, i32, vp, vp, vp]
        L.uref_w4_dequant.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
        L.uref_w4_linear.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, i64, vp, i64, i32, vp, i32]
        L.uref_w4_embedding.argtypes = [vp, vp, vp, i32, i32, i32, vp, i32, vp]
        L.uref_pruned_rope.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, dbl, vp, vp]
        L.uref_pruned_rope_f64.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, dbl]
        L.uref_w4_repack_plan.argtypes = [i32, i32, i32, vp, vp]
        L.uref_w4_repack.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp]
        L.uref_quantize_sym.argtypes = [vp, i32, i32, i32, vp, vp, vp]
        L.uref_quantize_asym.argtypes = [vp, i32, i32, i32, vp, vp, vp]
        L.uref_wq_dequant.argtypes = [i32, vp, vp, vp, i32, i32, i32, vp, vp, i32]
        L.uref_wq_linear.argtypes = [i32, vp, vp, vp, i32, i32, i32, vp, vp, i64, vp, i64, i32, vp, i32, i32]
        L.uref_quantize_sym_bits.argtypes = [i32, vp, i32, i32, i32, vp, vp, vp]
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a: np.ndarray, dtype, name: str) -> np.ndarray:
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: expected C-contiguous {np.dtype(dtype)}, got {a.dtype}")
    return a


FMTS = {"f16": 0, "bf16": 1}


def _f16_dtype(fmt: str):
    """numpy type of 16-bit float arrays: float16 for "f16"; "bf16" arrays are uint16 bit patterns
    (numpy has no bfloat16)."""
    return np.float16 if FMTS[fmt] == 0 else np.uint16


def _chkz(zeros) -> None:
    """zeros may be None: the symmetric scheme, every zero point 8."""
    if zeros is not None:
        _chk(zeros, np.uint8, "zeros")


def _keep_arr(keep) -> np.ndarray:
    if keep is None:
        return np.zeros(10, dtype=np.int32)
    t = keep.as_tuple() if hasattr(keep, "as_tuple") else tuple(keep)
    assert len(t) in (7, 10)      # the second row-segment family is optional
    return np.asarray(tuple(t) + (0,) * (10 - len(t)), dtype=np.int32)


def set_threads(n: int) -> None:
    lib().uref_set_threads(int(n))


def max_threads() -> int:
    return int(lib().uref_get_max_threads())


def half_to_double(bits: int) -> float:
    return float(lib().uref_half_to_double(int(bits)))


def double_to_half(x: float) -> int:
    return int(lib().uref_double_to_half(float(x)))


def bf16_to_double(bits: int) -> float:
    return float(lib().uref_bf16_to_double(int(bits)))


def double_to_bf16(x: float) -> int:
    return int(lib().uref_double_to_bf16(float(x)))


def count_kept(N_total: int, K_total: int, keep) -> tuple:
    n, k = C.c_int32(0), C.c_int32(0)
    ka = _keep_arr(keep)
    lib().uref_count_kept(N_total, K_total, _p(ka), C.addressof(n), C.addressof(k))
    return n.value, k.value


def w4_dequant(qweight, scales, zeros, keep=None, group: int = 128, fmt: str = "f16", il_heads: int = 0) -> np.ndarray:
    """[n_keep][k_keep] dequantised weights, RN16((q - z) * s), in the format of the scales.
    il_heads > 0: qweight stores its words head-interleaved over that many heads (see uref.c)."""
    N, K8 = qweight.shape
    K = K8 * 8
    ft = _f16_dtype(fmt)
    _chk(qweight, np.uint32, "qweight"); _chk(scales, ft, "scales"); _chkz(zeros)
    assert scales.shape == (N, K // group) and (zeros is None or zeros.shape == (N, K // group))
    ka = _keep_arr(keep)
    nk, kk = count_kept(N, K, ka)
    out = np.empty((nk, kk), dtype=ft)
    rc = lib().uref_w4_dequant_il(_p(qweight), _p(scales), _p(zeros), N, K, group, _p(ka), _p(out), FMTS[fmt], int(il_heads))
    assert rc == 0
    return out


def w4_embedding(qweight, scales, zeros, ids, group: int = 128, fmt: str = "f16") -> np.ndarray:
    """[len(ids)][K] dequantised rows ids of a quantised table, in the format of the scales."""
    N, K8 = qweight.shape
    K = K8 * 8
    ft = _f16_dtype(fmt)
    _chk(qweight, np.uint32, "qweight"); _chk(scales, ft, "scales"); _chkz(zeros)
    _chk(ids, np.int32, "ids")
    out = np.empty((ids.shape[0], K), dtype=ft)
    rc = lib().uref_w4_embedding_fmt(_p(qweight), _p(scales), _p(zeros), N, K, group, _p(ids), ids.shape[0],
                                     _p(out), FMTS[fmt])
    assert rc == 0, rc
    return out


def w4_linear(qweight, scales, zeros, x, keep=None, group: int = 128,
              rows: Optional[Sequence[int]] = None, fmt: str = "f16", il_heads: int = 0) -> np.ndarray:
    """fp64 y [M][n_keep] (or [M][len(rows)] for sampled compact rows); scales and x in format fmt.
    il_heads > 0: qweight stores its words head-interleaved over that many heads (see uref.c)."""
    N, K8 = qweight.shape
    K = K8 * 8
    ft = _f16_dtype(fmt)
    _chk(qweight, np.uint32, "qweight"); _chk(scales, ft, "scales"); _chkz(zeros)
    _chk(x, ft, "x")
    ka = _keep_arr(keep)
    nk, kk = count_kept(N, K, ka)
    M = x.shape[0]
    assert x.shape == (M, kk), (x.shape, kk)
    rl = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    n_out = nk if rl is None else rl.size
    y = np.empty((M, n_out), dtype=np.float64)
    rc = lib().uref_w4_linear_il(_p(qweight), _p(scales), _p(zeros), N, K, group, _p(ka),
                                 _p(x), kk, _p(y), n_out, M, _p(rl), 0 if rl is None else rl.size, FMTS[fmt], int(il_heads))
    assert rc == 0, rc
    return y


def wq_dequant(bits: int, qweight, scales, zeros, keep=None, group: int = 128, fmt: str = "f16") -> np.ndarray:
    """Kept part of the dequantised matrix with codes of `bits` bits (3, 4, 6 or 8: qweight uint32 [N][K * bits / 32],
    a row's codes as one little-endian bit stream; zeros 0..2^bits - 1 or None = 2^(bits-1)), as float16 (fmt "f16") or bfloat16 bit patterns (uint16, fmt "bf16")."""
    _chk(qweight, np.uint32, "qweight"); _chk(scales, _f16_dtype(fmt), "scales"); _chkz(zeros)
    N, Kw = qweight.shape
    K = Kw * 32 // bits
    ka = _keep_arr(keep)
    nk, kk = count_kept(N, K, ka)
    out = np.empty((nk, kk), dtype=_f16_dtype(fmt))
    rc = lib().uref_wq_dequant(bits, _p(qweight), _p(scales), _p(zeros), N, K, group, _p(ka), _p(out), FMTS[fmt])
    assert rc == 0, rc
    return out


def wq_linear(bits: int, qweight, scales, zeros, x, keep=None, group: int = 128, rows=None, fmt: str = "f16") -> np.ndarray:
    """fp64 y [M][n_keep] (or [M][len(rows)]) of the linear over codes of `bits` bits (see wq_dequant)."""
    _chk(qweight, np.uint32, "qweight"); _chk(scales, _f16_dtype(fmt), "scales"); _chkz(zeros)
    _chk(x, _f16_dtype(fmt), "x")
    N, Kw = qweight.shape
    K = Kw * 32 // bits
    ka = _keep_arr(keep)
    nk, kk = count_kept(N, K, ka)
    M = x.shape[0]
    assert x.shape == (M, kk), (x.shape, kk)
    rl = None if rows is None else np.ascontiguousarray(rows, dtype=np.int32)
    n_out = nk if rl is None else rl.size
    y = np.empty((M, n_out), dtype=np.float64)
    rc = lib().uref_wq_linear(bits, _p(qweight), _p(scales), _p(zeros), N, K, group, _p(ka),
                              _p(x), kk, _p(y), n_out, M, _p(rl), 0 if rl is None else rl.size, FMTS[fmt])
    assert rc == 0, rc
    return y


def quantize_sym_bits(bits: int, w: np.ndarray, group: int = 128):
    """Eq. 3 with N = bits: (qweight uint32 [N][K * bits / 32], scales float16, zeros uint8)."""
    w = np.ascontiguousarray(w, dtype=np.float64)
    N, K = w.shape
    qweight = np.zeros((N, K * bits // 32), dtype=np.uint32)
    scales = np.empty((N, K // group), dtype=np.float16)
    zeros = np.empty((N, K // group), dtype=np.uint8)
    rc = lib().uref_quantize_sym_bits(bits, _p(w), N, K, group, _p(qweight), _p(scales), _p(zeros))
    assert rc == 0, rc
    return qweight, scales, zeros


def w4_interleave(qweight, heads: int) -> np.ndarray:
    """The words of every row in head-interleaved order over `heads` heads (Sec. 3.4's on-device repack for o_proj)."""
    _chk(qweight, np.uint32, "qweight")
    N, K8 = qweight.shape
    out = np.empty_like(qweight)
    rc = lib().uref_w4_interleave(_p(qweight), N, K8 * 8, int(heads), _p(out))
    assert rc == 0, rc
    return out


def w4_deinterleave(qweight_il, heads: int) -> np.ndarray:
    """The words of a matrix that is head-interleaved over `heads` heads, back in column order."""
    _chk(qweight_il, np.uint32, "qweight_il")
    N, K8 = qweight_il.shape
    out = np.empty_like(qweight_il)
    rc = lib().uref_w4_deinterleave(_p(qweight_il), N, K8 * 8, int(heads), _p(out))
    if rc != 0:
        raise ValueError(f"uref_w4_deinterleave: {rc}")
    return out


def pruned_rope(q, k, positions, kept_idx, D_full: int, theta: float, fmt: str = "f16"):
    """fp64 rotated copies of q [T][Hq][D_keep] and k [T][Hkv][D_keep] (k may be None), inputs in format fmt."""
    ft = _f16_dtype(fmt)
    _chk(q, ft, "q"); _chk(positions, np.int32, "positions"); _chk(kept_idx, np.int32, "kept_idx")
    T, Hq, Dk = q.shape
    H_tab = kept_idx.shape[0]
    assert kept_idx.shape == (H_tab, Dk // 2) and positions.shape == (T,)
    q_out = np.empty(q.shape, dtype=np.float64)
    Hkv, k_out = 0, None
    if k is not None:
        _chk(k, ft, "k")
        assert k.shape[0] == T and k.shape[2] == Dk
        Hkv = k.shape[1]
        k_out = np.empty(k.shape, dtype=np.float64)
    rc = lib().uref_pruned_rope_fmt(_p(q), _p(k), _p(positions), _p(kept_idx), T, Hq, Hkv, H_tab,
                                    D_full, Dk, float(theta), _p(q_out), _p(k_out), FMTS[fmt])
    assert rc == 0, rc
    return q_out, k_out


def pruned_rope_f64(x, positions, kept_idx, D_full: int, theta: float):
    """Rotated fp64 copy of x [T][H][D_keep] (fp64 in, fp64 out): the rotation of `pruned_rope` without
    the fp16 input format."""
    x = np.array(x, dtype=np.float64, order="C", copy=True)
    _chk(positions, np.int32, "positions"); _chk(kept_idx, np.int32, "kept_idx")
    T, H, Dk = x.shape
    H_tab = kept_idx.shape[0]
    assert kept_idx.shape == (H_tab, Dk // 2) and positions.shape == (T,)
    rc = lib().uref_pruned_rope_f64(_p(x), _p(positions), _p(kept_idx), T, H, H_tab, D_full, Dk, float(theta))
    assert rc == 0, rc
    return x


def qkv_rope(wq, keep_q, wk, keep_k, wv, keep_v, x, positions, kept_idx, Hq: int, Hkv: int, D_full: int,
             D_keep: int, theta: float, fmt: str = "f16"):
    """The fused decode step y = RoPE(x W) for the q and k projections and y = x W for v, all fp64:
    each w* is a dict(qweight, scales, zeros); x is fp16 [T][k_keep].  Returns q [T][Hq][D_keep],
    k [T][Hkv][D_keep], v [T][n_keep_v]."""
    T = x.shape[0]
    q = w4_linear(wq["qweight"], wq["scales"], wq["zeros"], x, keep_q, fmt=fmt).reshape(T, Hq, D_keep)
    k = w4_linear(wk["qweight"], wk["scales"], wk["zeros"], x, keep_k, fmt=fmt).reshape(T, Hkv, D_keep)
    v = w4_linear(wv["qweight"], wv["scales"], wv["zeros"], x, keep_v, fmt=fmt)
    return (pruned_rope_f64(q, positions, kept_idx, D_full, theta),
            pruned_rope_f64(k, positions, kept_idx, D_full, theta), v)


def gate_up_silu(wg, keep_g, wu, keep_u, x, fmt: str = "f16"):
    """The gated MLP's hidden vector h = sigma(x W_gate) * (x W_up) of Eq. 1 with sigma = SiLU
    (g / (1 + exp(-g))), fp64: each w* is a dict(qweight, scales, zeros); x is fp16 [T][k_keep]."""
    g = w4_linear(wg["qweight"], wg["scales"], wg["zeros"], x, keep_g, fmt=fmt)
    u = w4_linear(wu["qweight"], wu["scales"], wu["zeros"], x, keep_u, fmt=fmt)
    return g / (1.0 + np.exp(-g)) * u


def w4_repack_plan(N_total: int, K_total: int, keep=None, group: int = 128):
    """(N_out, K_out, keep_out) of the compact matrix: keep_out is the 7-tuple to use with it."""
    plan = np.zeros(9, dtype=np.int32)
    rc = lib().uref_w4_repack_plan(N_total, K_total, group, _p(_keep_arr(keep)), _p(plan))
    assert rc == 0
    return int(plan[0]), int(plan[1]), tuple(int(v) for v in plan[2:])


def w4_repack(qweight, scales, zeros, keep=None, group: int = 128):
    """The compact quantised matrix of the kept channels (Sec. 3.4: unpack, prune, pack again):
    (qweight', scales', zeros', keep') with y(W', keep') == y(W, keep)."""
    N, K8 = qweight.shape
    K = K8 * 8
    _chk(qweight, np.uint32, "qweight"); _chkz(zeros)
    if scales.dtype != np.uint16:     # scales are carried as they are stored: fp16, or bfloat16 bit patterns
        _chk(scales, np.float16, "scales")
    n_out, k_out, keep_out = w4_repack_plan(N, K, keep, group)
    q2 = np.zeros((n_out, k_out // 8), dtype=np.uint32)
    s2 = np.zeros((n_out, k_out // group), dtype=scales.dtype)
    z2 = None if zeros is None else np.zeros((n_out, k_out // group), dtype=np.uint8)
    rc = lib().uref_w4_repack(_p(qweight), _p(scales), _p(zeros), N, K, group, _p(_keep_arr(keep)),
                              _p(q2), _p(s2), _p(z2))
    assert rc == 0
    return q2, s2, z2, keep_out


def _quantize(fn, w: np.ndarray, group: int):
    w = np.ascontiguousarray(w, dtype=np.float64)
    N, K = w.shape
    assert K % group == 0 and K % 8 == 0
    qweight = np.zeros((N, K // 8), dtype=np.uint32)
    scales = np.zeros((N, K // group), dtype=np.float16)
    zeros = np.zeros((N, K // group), dtype=np.uint8)
    fn(_p(w), N, K, group, _p(qweight), _p(scales), _p(zeros))
    return qweight, scales, zeros


def quantize_sym(w: np.ndarray, group: int = 128):
    return _quantize(lib().uref_quantize_sym, w, group)


def quantize_asym(w: np.ndarray, group: int = 128):
    return _quantize(lib().uref_quantize_asym, w, group)
