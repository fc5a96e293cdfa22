"""Seeded synthetic inputs and workload shape tables.

This module is the only code shared by the CPU oracle's tests and the HIP
path's tests/benchmark.  It holds no arithmetic of the method: it draws random
bytes / numbers with the distributions of the benchmark workloads and lists the
layer shapes and the kept dimensions that follow from a pruning rate.

Everything is generated from ``numpy.random.default_rng(SEED_BASE + config
index)`` and stands in for real model tensors (Llama-3-8B, Qwen2.5-7B and
Mamba2-2.7B shaped layers); no model weights or datasets are used.

Storage convention of one quantised linear with N outputs and K inputs:
  qweight  uint32 [N][K/8]   nibble j (bits 4j..4j+3) of word w in a row is
                             input column 8w + j
  scales   float16 [N][K/G]  one per group of G = 128 input columns
  zeros    uint8  [N][K/G]   values 0..15
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np

SEED_BASE = 20251203
GROUP = 128


# --------------------------------------------------------------------------
# kept dimensions for a pruning rate given in whole percent
# --------------------------------------------------------------------------
def kept_dim(d: int, rate_pct: int) -> int:
    """floor(d * (1 - rate)) with the rate in integer percent."""
    return d * (100 - rate_pct) // 100


def kept_head_dim(d: int, rate_pct: int) -> int:
    """Even kept head dimension: 2 * floor(d * (1 - rate) / 2)."""
    return 2 * (d * (100 - rate_pct) // 200)


@dataclass(frozen=True)
class Keep:
    """Which stored rows / columns of a linear survive (all zero = unpruned).

    rows: if row_seg_stride == 0 the first n_keep stored rows are kept.
          Otherwise stored row r below row_seg_limit is kept iff
          (r % row_seg_stride) < row_seg_keep; a row from row_seg_limit up to
          row_seg2_limit iff ((r - row_seg_limit) % row_seg2_stride) < row_seg2_keep
          (when row_seg2_stride > 0); every row behind that is kept.  n_keep is the
          resulting count.
    cols: if col_seg_stride == 0 the first k_keep stored columns are kept,
          otherwise column k is kept iff (k % col_seg_stride) < col_seg_keep.
    Kept rows / columns appear in the compact y / x in increasing stored order.
    """
    n_keep: int = 0
    k_keep: int = 0
    row_seg_stride: int = 0
    row_seg_keep: int = 0
    row_seg_limit: int = 0
    col_seg_stride: int = 0
    col_seg_keep: int = 0
    row_seg2_stride: int = 0
    row_seg2_keep: int = 0
    row_seg2_limit: int = 0

    def as_tuple(self):
        return (self.n_keep, self.k_keep, self.row_seg_stride, self.row_seg_keep,
                self.row_seg_limit, self.col_seg_stride, self.col_seg_keep,
                self.row_seg2_stride, self.row_seg2_keep, self.row_seg2_limit)


@dataclass(frozen=True)
class LinearSpec:
    name: str
    K: int            # stored input columns
    N: int            # stored output rows
    keep: Keep = field(default_factory=Keep)

    @property
    def n_keep(self) -> int:
        return self.keep.n_keep if self.keep.n_keep else self.N

    @property
    def k_keep(self) -> int:
        return self.keep.k_keep if self.keep.k_keep else self.K

    def groups_touched(self) -> int:
        """Quantisation groups per kept row that hold at least one kept column."""
        kp = self.keep
        if kp.col_seg_stride:
            # every segment of a uniform column pattern starts a kept run
            kept_cols = np.nonzero((np.arange(self.K) % kp.col_seg_stride) < kp.col_seg_keep)[0]
            return int(np.unique(kept_cols // GROUP).size)
        return (self.k_keep + GROUP - 1) // GROUP

    def algorithmic_bytes(self, M: int = 1) -> int:
        """Bytes one call must move: kept nibbles + (fp16 scale + half-byte zero)
        per touched group + compact x + compact y."""
        nk, kk = self.n_keep, self.k_keep
        return int(nk * kk / 2 + nk * self.groups_touched() * 2.5 + M * kk * 2 + M * nk * 2)

    def flops(self, M: int) -> int:
        return 2 * M * self.n_keep * self.k_keep


@dataclass(frozen=True)
class RopeSpec:
    T: int            # tokens
    Hq: int
    Hkv: int          # 0 = no K tensor
    H_tab: int        # rows of the kept-index table
    D_full: int
    D_keep: int
    theta: float
    pos_max: int      # positions ~ U{0..pos_max-1}; -1 = arange(T)

    def algorithmic_bytes(self) -> int:
        elems = self.T * (self.Hq + self.Hkv) * self.D_keep
        return elems * 2 * 2 + self.T * 4 + self.H_tab * (self.D_keep // 2) * 4


# --------------------------------------------------------------------------
# layer shape tables
# --------------------------------------------------------------------------
def _rows_prefix(n):
    return Keep(n_keep=n)


def _rows_seg(n_total, stride, keep, limit=None):
    limit = n_total if limit is None else limit
    n = (limit // stride) * keep + (n_total - limit)
    return Keep(n_keep=n, row_seg_stride=stride, row_seg_keep=keep, row_seg_limit=limit)


def _cols_prefix(k):
    return Keep(k_keep=k)


def _cols_seg(k_total, stride, keep):
    return Keep(k_keep=(k_total // stride) * keep, col_seg_stride=stride, col_seg_keep=keep)


def attention_mlp_layer(hidden: int, inter: int, Hq: int, Hkv: int, D: int,
                        rate_pct: int) -> List[LinearSpec]:
    """The seven linears of one decoder layer at a pruning rate.

    Q/K heads keep the leading D'/2 channels of each half (symmetric sort), V
    heads and the matching o_proj inputs keep the leading D' channels per head,
    the MLP keeps the leading D_int' intermediate channels.  The hidden size is
    never pruned.
    """
    Dk = kept_head_dim(D, rate_pct)
    Ik = kept_dim(inter, rate_pct)
    if rate_pct == 0:
        none = Keep()
        return [LinearSpec("q_proj", hidden, Hq * D, none),
                LinearSpec("k_proj", hidden, Hkv * D, none),
                LinearSpec("v_proj", hidden, Hkv * D, none),
                LinearSpec("o_proj", Hq * D, hidden, none),
                LinearSpec("gate_proj", hidden, inter, none),
                LinearSpec("up_proj", hidden, inter, none),
                LinearSpec("down_proj", inter, hidden, none)]
    return [LinearSpec("q_proj", hidden, Hq * D, _rows_seg(Hq * D, D // 2, Dk // 2)),
            LinearSpec("k_proj", hidden, Hkv * D, _rows_seg(Hkv * D, D // 2, Dk // 2)),
            LinearSpec("v_proj", hidden, Hkv * D, _rows_seg(Hkv * D, D, Dk)),
            LinearSpec("o_proj", Hq * D, hidden, _cols_seg(Hq * D, D, Dk)),
            LinearSpec("gate_proj", hidden, inter, _rows_prefix(Ik)),
            LinearSpec("up_proj", hidden, inter, _rows_prefix(Ik)),
            LinearSpec("down_proj", inter, hidden, _cols_prefix(Ik))]


def llama3_8b_layer(rate_pct: int) -> List[LinearSpec]:
    return attention_mlp_layer(4096, 14336, 32, 8, 128, rate_pct)


def llama3_8b_rope(rate_pct: int, T: int = 1, pos_max: int = 4096) -> RopeSpec:
    return RopeSpec(T=T, Hq=32, Hkv=8, H_tab=8, D_full=128,
                    D_keep=kept_head_dim(128, rate_pct), theta=500000.0, pos_max=pos_max)


def qwen25_7b_layer(rate_pct: int = 25) -> List[LinearSpec]:
    return attention_mlp_layer(3584, 18944, 28, 4, 128, rate_pct)


def qwen25_7b_rope(rate_pct: int = 25, T: int = 1) -> RopeSpec:
    return RopeSpec(T=T, Hq=28, Hkv=4, H_tab=4, D_full=128,
                    D_keep=kept_head_dim(128, rate_pct), theta=1.0e6, pos_max=32768)


def mamba2_2p7b_layer(rate_pct: int = 15) -> List[LinearSpec]:
    """in_proj 2560 -> 10576 = [z 5120 | x 5120 | B 128 | C 128 | dt 80];
    out_proj 5120 -> 2560.  z and x keep their leading channels, the tail is
    kept whole; out_proj keeps the matching leading input columns."""
    d_inner, tail = 5120, 336
    kd = kept_dim(d_inner, rate_pct)
    if rate_pct == 0:
        return [LinearSpec("in_proj", 2560, 2 * d_inner + tail), LinearSpec("out_proj", d_inner, 2560)]
    return [LinearSpec("in_proj", 2560, 2 * d_inner + tail,
                       _rows_seg(2 * d_inner + tail, d_inner, kd, limit=2 * d_inner)),
            LinearSpec("out_proj", d_inner, 2560, _cols_prefix(kd))]


def mamba2_2p7b_layer_heads_and_state(rate_pct: int = 15) -> List[LinearSpec]:
    """The same block pruned the way Alg. 4 and Alg. 5 sort it: every one of the 80 SSM heads (64
    channels) keeps its leading channels in the z and x parts, and the single SSM group keeps the
    leading state channels of its 128 in the B and in the C part (Sec. 3.4 prunes both the head and the
    state dimension of a Mamba layer); the 80 step-size rows stay.  out_proj keeps the matching columns
    of every head."""
    H, D, Ds, G = 80, 64, 128, 1
    d_inner = H * D
    Dk, Sk = kept_head_dim(D, rate_pct), kept_dim(Ds, rate_pct)
    N = 2 * d_inner + 2 * G * Ds + H
    keep = Keep(n_keep=2 * H * Dk + 2 * G * Sk + H, row_seg_stride=D, row_seg_keep=Dk, row_seg_limit=2 * d_inner,
                row_seg2_stride=Ds, row_seg2_keep=Sk, row_seg2_limit=2 * d_inner + 2 * G * Ds)
    return [LinearSpec("in_proj", 2560, N, keep),
            LinearSpec("out_proj", d_inner, 2560, _cols_seg(d_inner, D, Dk))]


def lm_head_llama3() -> LinearSpec:
    """The 4-bit output head of a Llama-3-8B shaped model (Sec. 3.4 quantises the embedding and
    output layers too): 128256 vocabulary rows x 4096, not pruned.  The largest GEMV of a decode step."""
    return LinearSpec("lm_head", K=4096, N=128256)


def small_case() -> LinearSpec:
    """The 1024x1024 parity case: keep the first 870 output rows."""
    return LinearSpec("small", 1024, 1024, _rows_prefix(kept_dim(1024, 15)))


def small_rope() -> RopeSpec:
    return RopeSpec(T=1, Hq=8, Hkv=0, H_tab=8, D_full=64, D_keep=kept_head_dim(64, 15),
                    theta=10000.0, pos_max=4096)


def prefill_linears(rate_pct: int = 15) -> List[LinearSpec]:
    Ik = kept_dim(14336, rate_pct)
    return [LinearSpec("gate_up_proj", 4096, 14336, _rows_prefix(Ik)),
            LinearSpec("down_proj", 14336, 4096, _cols_prefix(Ik))]


def prefill_rope(rate_pct: int = 15, T: int = 4096) -> RopeSpec:
    return RopeSpec(T=T, Hq=32, Hkv=8, H_tab=8, D_full=128,
                    D_keep=kept_head_dim(128, rate_pct), theta=500000.0, pos_max=-1)


# --------------------------------------------------------------------------
# seeded tensors
# --------------------------------------------------------------------------
def rng_for(config_index: int, stream: int = 0) -> np.random.Generator:
    return np.random.default_rng([SEED_BASE + config_index, stream])


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Storage format of generated inputs: float32 -> bfloat16 bit patterns (the upper half of the
    binary32, rounded to nearest even) as uint16; numpy has no bfloat16 type."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """The values of bfloat16 bit patterns (exact: a bfloat16 is a binary32 with a zero lower half)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _store16(a: np.ndarray, fmt: str) -> np.ndarray:
    return a.astype(np.float16) if fmt == "f16" else to_bf16_bits(a.astype(np.float32))


def gen_linear(rng: np.random.Generator, N: int, K: int,
               sym_zero: bool = False, fmt: str = "f16") -> Dict[str, np.ndarray]:
    """Random packed nibbles (uniform 32-bit words are eight uniform nibbles),
    scales ~ U(0.005, 0.02) stored as fp16 (fmt "f16") or as bfloat16 bit patterns (fmt "bf16", uint16)
    and zeros ~ U{0..15} (or all 8 when sym_zero)."""
    assert K % GROUP == 0
    qweight = rng.integers(0, 2 ** 32, size=(N, K // 8), dtype=np.uint64).astype(np.uint32)
    scales = _store16(rng.uniform(0.005, 0.02, size=(N, K // GROUP)), fmt)
    if sym_zero:
        zeros = np.full((N, K // GROUP), 8, dtype=np.uint8)
    else:
        zeros = rng.integers(0, 16, size=(N, K // GROUP), dtype=np.uint8)
    return {"qweight": qweight, "scales": scales, "zeros": zeros}


def gen_linear8(rng: np.random.Generator, N: int, K: int,
                sym_zero: bool = False, fmt: str = "f16") -> Dict[str, np.ndarray]:
    """8-bit codes: random 32-bit words (four uniform bytes each), scales ~ U(0.0003, 0.0012) (the 4-bit range
    divided by 16: the same weight range on a grid 16 times finer) and zeros ~ U{0..255} (or all 128 when sym_zero)."""
    assert K % GROUP == 0
    qweight = rng.integers(0, 2 ** 32, size=(N, K // 4), dtype=np.uint64).astype(np.uint32)
    scales = _store16(rng.uniform(0.0003, 0.0012, size=(N, K // GROUP)), fmt)
    if sym_zero:
        zeros = np.full((N, K // GROUP), 128, dtype=np.uint8)
    else:
        zeros = rng.integers(0, 256, size=(N, K // GROUP), dtype=np.uint8)
    return {"qweight": qweight, "scales": scales, "zeros": zeros}


def gen_linear_bits(rng: np.random.Generator, N: int, K: int, bits: int,
                    sym_zero: bool = False, fmt: str = "f16") -> Dict[str, np.ndarray]:
    """Codes of 3 or 6 bits (any width that divides into whole words per group): random 32-bit words, i.e. a uniform
    bit stream of K * bits / 32 words per row, scales ~ U(0.005, 0.02) * 16 / 2^bits (the 4-bit weight range on a
    grid of 2^bits levels) and zeros ~ U{0..2^bits - 1} (or all 2^(bits-1) when sym_zero)."""
    assert K % GROUP == 0 and (K * bits) % 32 == 0
    qweight = rng.integers(0, 2 ** 32, size=(N, K * bits // 32), dtype=np.uint64).astype(np.uint32)
    f = 16.0 / (1 << bits)
    scales = _store16(rng.uniform(0.005 * f, 0.02 * f, size=(N, K // GROUP)), fmt)
    if sym_zero:
        zeros = np.full((N, K // GROUP), 1 << (bits - 1), dtype=np.uint8)
    else:
        zeros = rng.integers(0, 1 << bits, size=(N, K // GROUP), dtype=np.uint8)
    return {"qweight": qweight, "scales": scales, "zeros": zeros}


def gen_activations(rng: np.random.Generator, M: int, K: int, fmt: str = "f16") -> np.ndarray:
    return _store16(rng.standard_normal((M, K)), fmt)


def gen_rope_inputs(rng: np.random.Generator, spec: RopeSpec, fmt: str = "f16") -> Dict[str, Optional[np.ndarray]]:
    """q [T][Hq][D_keep], k [T][Hkv][D_keep] ~ N(0,1) in fp16 (or bfloat16 bit patterns), int32 positions
    and a kept-index table whose rows are the first D_keep/2 entries of a random
    permutation of 0..D_full/2-1 (importance order, not numerically sorted)."""
    q = _store16(rng.standard_normal((spec.T, spec.Hq, spec.D_keep)), fmt)
    k = (_store16(rng.standard_normal((spec.T, spec.Hkv, spec.D_keep)), fmt)
         if spec.Hkv else None)
    if spec.pos_max < 0:
        pos = np.arange(spec.T, dtype=np.int32)
    else:
        pos = rng.integers(0, spec.pos_max, size=spec.T, dtype=np.int32)
    half = spec.D_full // 2
    idx = np.stack([rng.permutation(half)[: spec.D_keep // 2] for _ in range(spec.H_tab)])
    return {"q": q, "k": k, "positions": pos, "kept_idx": idx.astype(np.int32)}


def with_keep(spec: LinearSpec, keep: Keep) -> LinearSpec:
    return replace(spec, keep=keep)
