"""Error metrics used by the GPU parity tests.

Linear outputs: err_i = |y_i - ref_i| / max(|ref_i|, 1e-2 * rms(ref)) per token row;
the bar is max err <= 2e-3.  The floor keeps outputs that cancel to almost zero
from making a pure element-wise relative error meaningless.
RoPE outputs: the floor is 1e-2 times the norm of the element's own pair.
"""
import numpy as np

TOL = 2e-3
# bfloat16 outputs: the one rounding of the fp32 sum to 8 significant bits is up to 2^-8 = 3.9e-3 of the
# value by itself (fp16: 2^-11 = 4.9e-4, inside the 2e-3 bar); fp32 accumulation adds of the order of 1e-6 rms.
TOL_BF16 = 2.0 ** -8 + 1e-4


def linear_err(y_gpu_f16: np.ndarray, ref_f64: np.ndarray) -> float:
    y = y_gpu_f16.astype(np.float64)
    assert y.shape == ref_f64.shape, (y.shape, ref_f64.shape)
    if not np.all(np.isfinite(y)):
        return float("inf")
    rms = np.sqrt(np.mean(ref_f64 ** 2, axis=-1, keepdims=True))
    den = np.maximum(np.abs(ref_f64), 1e-2 * rms)
    den = np.where(den == 0.0, 1.0, den)
    return float(np.max(np.abs(y - ref_f64) / den))


def rope_err(y_gpu_f16: np.ndarray, ref_f64: np.ndarray) -> float:
    y = y_gpu_f16.astype(np.float64)
    assert y.shape == ref_f64.shape
    if not np.all(np.isfinite(y)):
        return float("inf")
    hk = ref_f64.shape[-1] // 2
    pn = np.sqrt(ref_f64[..., :hk] ** 2 + ref_f64[..., hk:] ** 2)
    pn = np.concatenate([pn, pn], axis=-1)
    den = np.maximum(np.abs(ref_f64), 1e-2 * pn)
    den = np.where(den == 0.0, 1.0, den)
    return float(np.max(np.abs(y - ref_f64) / den))


def normwise_err(y_gpu: np.ndarray, ref_f64: np.ndarray) -> float:
    """max over token rows of ||y - ref||_2 / ||ref||_2 (no floor needed: a norm does not cancel)."""
    y = y_gpu.astype(np.float64)
    assert y.shape == ref_f64.shape
    num = np.sqrt(np.sum((y - ref_f64) ** 2, axis=-1))
    den = np.sqrt(np.sum(ref_f64 ** 2, axis=-1))
    return float(np.max(num / np.where(den == 0.0, 1.0, den)))


# Norm-wise bars: the output rounding is uniform within half an ulp, so its root mean square is about
# 2^-11 / sqrt(3) = 2.8e-4 of the value in fp16 and 2^-8 / sqrt(3) = 2.3e-3 in bfloat16; accumulation adds ~1e-6.
NORM_TOL = 4e-4
NORM_TOL_BF16 = 3e-3
