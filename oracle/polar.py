"""Polar encoder and mid-point dequantizer (oracle; test infrastructure only).

Follows Section 3.2 of the paper step by step, with these readings fixed:

* Pair j of a d-dim key is (K[j], K[j + d/2]) -- the rotate-half pairing that
  real RoPE implementations use (footnote 2 of Section 3.1); x = K[j] is the
  first coordinate, y = K[j + d/2] the second.
* rho = sqrt(x^2 + y^2) is evaluated in float32 with every operation rounded
  on its own (two products, one sum, one square root): radius codes are an
  integer decision, so the precision is part of the definition.
* theta = atan2(y, x); the paper's "+ pi" only makes the bin index start at 0.
  The angle quantizer is the UNIFORM grid of 2^t bins over [-pi, pi): bin k is
  the half-open arc [-pi + k*D, -pi + (k+1)*D), D = 2*pi / 2^t.  theta = +pi
  (y = +0, x < 0) is clamped into the last bin; x = y = 0 goes to bin 2^(t-1)
  (theta = 0).  The bin is the floor of the EXACT real-number quotient: for the
  only directions where a float pair can sit exactly on an edge (multiples of
  pi/4: an axis or a diagonal) the quotient is taken as an exact rational
  instead of through rounded float64 arithmetic.
* Radius: asymmetric, per pair, statistics over the valid tokens of a group of
  g consecutive tokens: zero-point z = min, scale s = (max - min) / 2^r (the
  printed zero-point formula repeats the scale; the appendix listing names the
  same quantity "rmn", the minimum).  s and z are STORED in 16 bits (Appendix
  B.1) as IEEE fp16, round-to-nearest-even, and the code is computed against
  the stored values: Q = Clamp(floor((rho - z) / s), 0, 2^r - 1), float32, true
  division; Q = 0 when s == 0.
* Dequantizer: rho~ = (Q + 1/2) s + z and theta~ = -pi + (Q_theta + 1/2) D,
  key~ = (rho~ cos theta~, rho~ sin theta~) at dims (j, j + d/2).

Grouped angle quantizer (Section 3.2 as printed: the angle is quantized like the
radius, asymmetric and group-wise; the appendix listing rebuilds the angle
levels from "tscale" and "tmn" per group):
* theta = atan2(y, x) in float64, in [-pi, pi].  The printed "+ pi" would only
  add pi to every zero-point; it is dropped, so that cos / sin of the
  reconstructed angle give the key back and not its negative.
* per pair and group: z = min theta, s = (max - min) / 2^t over the valid
  tokens, both stored as fp16 (rounded once, from float64, to nearest even),
  Q = Clamp(floor((theta - z) / s), 0, 2^t - 1) against the stored values in
  float64, Q = 0 when s == 0;  theta~ = (Q + 1/2) s + z.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32
F64 = np.float64


def split_pairs(keys: np.ndarray):
    """x = K[..., j], y = K[..., j + d/2] for j < d/2 (footnote 2, Section 3.1)."""
    d = keys.shape[-1]
    assert d % 2 == 0
    return keys[..., : d // 2], keys[..., d // 2:]


def radius_f32(x: np.ndarray, y: np.ndarray) -> np.ndarray:
    """rho = sqrt(x^2 + y^2) (Section 3.2), four separately rounded float32 operations."""
    x = x.astype(F32)
    y = y.astype(F32)
    xx = x * x
    yy = y * y
    return np.sqrt(xx + yy)


def angle_bin(x: np.ndarray, y: np.ndarray, t_bits: int):
    """Uniform t-bit angle code of each pair and its distance to the nearest bin edge.

    Returns (code int64, edge_dist float64 in radians).  edge_dist is what a
    comparison with another implementation uses to tell a genuine error from
    a pair that sits on a bin boundary.
    """
    n_bins = 1 << t_bits
    xd = x.astype(F64)
    yd = y.astype(F64)
    theta = np.arctan2(yd, xd)
    u = (theta + np.pi) * n_bins / (2.0 * np.pi)
    code = np.floor(u).astype(np.int64)
    edge_dist = np.abs(u - np.rint(u)) * (2.0 * np.pi / n_bins)

    # Directions that are an exact multiple of pi/4: theta = m*pi/4 exactly,
    # so u = (m + 4) * 2^t / 8 is rational and its floor is integer arithmetic.
    ax, ay = np.abs(xd), np.abs(yd)
    exact = (xd == 0) | (yd == 0) | (ax == ay)
    if np.any(exact):
        m = np.zeros(x.shape, np.int64)
        xp, xn, yp, yn = xd > 0, xd < 0, yd > 0, yd < 0
        m = np.where((yd == 0) & xn, np.where(np.signbit(yd), -4, 4), m)
        m = np.where((xd == 0) & yp, 2, m)
        m = np.where((xd == 0) & yn, -2, m)
        diag = (ax == ay) & (xd != 0)
        m = np.where(diag & xp & yp, 1, m)
        m = np.where(diag & xn & yp, 3, m)
        m = np.where(diag & xn & yn, -3, m)
        m = np.where(diag & xp & yn, -1, m)
        num = (m + 4) * n_bins            # u = num / 8
        code = np.where(exact, num // 8, code)
        edge_dist = np.where(exact & (num % 8 == 0), 0.0, edge_dist)
    code = np.clip(code, 0, n_bins - 1)
    return code, edge_dist


def radius_group_params(rho: np.ndarray, group_tokens: int, r_bits: int, param_dtype=np.float16):
    """Per (group, head, pair) scale and zero-point of the radius quantizer.

    rho: float32 [L, H, P].  Groups are tokens [k*g, min((k+1)*g, L)); the
    statistics of a partial last group run over its valid tokens only.
    Returns (scale, zero) of dtype param_dtype, shape [ceil(L/g), H, P].
    """
    L = rho.shape[0]
    n_groups = (L + group_tokens - 1) // group_tokens
    scale = np.empty((n_groups,) + rho.shape[1:], param_dtype)
    zero = np.empty_like(scale)
    for k in range(n_groups):
        blk = rho[k * group_tokens: min((k + 1) * group_tokens, L)]
        mn = blk.min(axis=0)
        mx = blk.max(axis=0)
        s32 = (mx - mn) / F32(1 << r_bits)
        scale[k] = s32.astype(param_dtype)
        zero[k] = mn.astype(param_dtype)
    return scale, zero


def radius_codes(rho: np.ndarray, scale: np.ndarray, zero: np.ndarray, group_tokens: int, r_bits: int):
    """Q(rho) = Clamp(floor((rho - z) / s), 0, 2^r - 1) against the stored parameters."""
    L = rho.shape[0]
    grp = np.arange(L) // group_tokens
    s = scale.astype(F32)[grp]
    z = zero.astype(F32)[grp]
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.floor((rho - z) / s)
    q = np.where(s == 0, F32(0), q)
    return np.clip(q, 0, (1 << r_bits) - 1).astype(np.int64)


def angle_group_params(theta: np.ndarray, group_tokens: int, t_bits: int, param_dtype=np.float16):
    """Per (group, head, pair) scale and zero-point of the grouped angle quantizer.

    theta: float64 [L, H, P] = atan2(y, x).  Same grouping as radius_group_params.
    Returns (scale, zero) of dtype param_dtype, shape [ceil(L/g), H, P].
    """
    L = theta.shape[0]
    n_groups = (L + group_tokens - 1) // group_tokens
    scale = np.empty((n_groups,) + theta.shape[1:], param_dtype)
    zero = np.empty_like(scale)
    for k in range(n_groups):
        blk = theta[k * group_tokens: min((k + 1) * group_tokens, L)]
        mn = blk.min(axis=0)
        mx = blk.max(axis=0)
        scale[k] = ((mx - mn) / F64(1 << t_bits)).astype(param_dtype)
        zero[k] = mn.astype(param_dtype)
    return scale, zero


def angle_group_codes(theta: np.ndarray, scale: np.ndarray, zero: np.ndarray, group_tokens: int, t_bits: int):
    """Q(theta) = Clamp(floor((theta - z) / s), 0, 2^t - 1) against the stored parameters.

    Returns (code int64, edge_dist float64): edge_dist is the distance in radians from theta
    to the nearest boundary between two bins of its group's grid (z + k s, 0 < k < 2^t).
    """
    n_bins = 1 << t_bits
    grp = np.arange(theta.shape[0]) // group_tokens
    s = scale.astype(F64)[grp]
    z = zero.astype(F64)[grp]
    with np.errstate(divide="ignore", invalid="ignore"):
        u = (theta - z) / s
    u = np.where(s == 0, 0.0, u)
    code = np.clip(np.floor(u), 0, n_bins - 1).astype(np.int64)
    nearest = np.clip(np.rint(u), 1, n_bins - 1)           # interior boundaries only
    edge_dist = np.abs(u - nearest) * s
    edge_dist = np.where(s == 0, np.inf, edge_dist)
    return code, edge_dist


def encode_keys(keys: np.ndarray, r_bits: int, t_bits: int, group_tokens: int, param_dtype=np.float16,
                grouped_angles: bool = False):
    """Encode post-RoPE keys [L, H, d] of one sequence.

    Returns a dict with
      a     int64 [L, H, P]   angle codes
      c     int64 [L, H, P]   radius codes
      scale, zero  param_dtype [ceil(L/g), H, P]
      rho   float32 [L, H, P] (for audits)
      edge_dist float64 [L, H, P] distance of theta to the nearest bin edge, radians
    and, with grouped_angles (the paper's own angle quantizer instead of the uniform grid),
      t_scale, t_zero  param_dtype [ceil(L/g), H, P]
    """
    x, y = split_pairs(keys)
    rho = radius_f32(x, y)
    scale, zero = radius_group_params(rho, group_tokens, r_bits, param_dtype)
    c = radius_codes(rho, scale, zero, group_tokens, r_bits)
    if not grouped_angles:
        a, edge = angle_bin(x, y, t_bits)
        return dict(a=a, c=c, scale=scale, zero=zero, rho=rho, edge_dist=edge)
    theta = np.arctan2(y.astype(F64), x.astype(F64))
    t_scale, t_zero = angle_group_params(theta, group_tokens, t_bits, param_dtype)
    a, edge = angle_group_codes(theta, t_scale, t_zero, group_tokens, t_bits)
    return dict(a=a, c=c, scale=scale, zero=zero, rho=rho, edge_dist=edge, t_scale=t_scale, t_zero=t_zero)


def dequant_radius(c: np.ndarray, scale: np.ndarray, zero: np.ndarray, group_tokens: int) -> np.ndarray:
    """rho~ = (Q + 1/2) * s + z in float64 (mid-point of the radius bin)."""
    grp = np.arange(c.shape[0]) // group_tokens
    return (c.astype(F64) + 0.5) * scale.astype(F64)[grp] + zero.astype(F64)[grp]


def dequant_angle(a: np.ndarray, t_bits: int) -> np.ndarray:
    """theta~ = -pi + (Q + 1/2) * 2*pi / 2^t in float64 (mid-point of the angle bin)."""
    return -np.pi + (a.astype(F64) + 0.5) * (2.0 * np.pi / (1 << t_bits))


def dequant_angle_grouped(a: np.ndarray, t_scale: np.ndarray, t_zero: np.ndarray, group_tokens: int) -> np.ndarray:
    """theta~ = (Q + 1/2) * s + z in float64 with the group's angle parameters."""
    grp = np.arange(a.shape[0]) // group_tokens
    return (a.astype(F64) + 0.5) * t_scale.astype(F64)[grp] + t_zero.astype(F64)[grp]


def dequant_keys(a, c, scale, zero, t_bits: int, group_tokens: int, t_scale=None, t_zero=None) -> np.ndarray:
    """Reconstructed keys float64 [L, H, d]: (rho~ cos theta~, rho~ sin theta~) at dims (j, j+d/2).

    With t_scale / t_zero the angle levels are the group's own (grouped angle quantizer)."""
    rho = dequant_radius(c, scale, zero, group_tokens)
    th = dequant_angle(a, t_bits) if t_scale is None else dequant_angle_grouped(a, t_scale, t_zero, group_tokens)
    return np.concatenate([rho * np.cos(th), rho * np.sin(th)], axis=-1)
