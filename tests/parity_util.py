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
