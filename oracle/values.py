"""Token-wise value quantization (oracle; test infrastructure only).

The paper's optional value quantizer is the standard token-wise one of its Background section
(Section 2, following KIVI; used in Section 6.3 "+ value quantization" and the dagger rows of the
throughput table, group size 128 = one head): for token n of a head,
    Q(V_n[j]) = Clamp(round((V_n[j] - z_n) / s_n), 0, 2^b - 1),
    z_n = min_j V_n[j],  s_n = (max_j V_n[j] - min_j V_n[j]) / (2^b - 1),
and the dequantized value is Q * s_n + z_n (the standard rule restated at the start of Section 3.3).
Readings fixed here: round is round-half-to-even; s and z are stored as fp16 (16-bit scale and
zero-point per token, Appendix B.1) and the code is taken against the stored values in float32
with a true division; s == 0 (constant row) gives code 0.  Values arrive as fp16, so z = min is
stored exactly.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32
F64 = np.float64


def quantize_values(v: np.ndarray, bits: int):
    """v fp16 [L, H, d] -> (codes int64 [L, H, d], scale fp16 [L, H], zero fp16 [L, H])."""
    vf = v.astype(F32)
    mn = vf.min(axis=-1)
    mx = vf.max(axis=-1)
    s32 = (mx - mn) / F32((1 << bits) - 1)
    scale = s32.astype(np.float16)
    zero = mn.astype(np.float16)
    s = scale.astype(F32)[..., None]
    z = zero.astype(F32)[..., None]
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.rint((vf - z) / s)
    q = np.where(s == 0, F32(0), q)
    return np.clip(q, 0, (1 << bits) - 1).astype(np.int64), scale, zero


def dequant_values(codes: np.ndarray, scale: np.ndarray, zero: np.ndarray) -> np.ndarray:
    """V~ = Q * s + z in float64."""
    return codes.astype(F64) * scale.astype(F64)[..., None] + zero.astype(F64)[..., None]
