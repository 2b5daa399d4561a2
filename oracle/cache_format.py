"""Packed key-cache page layout (oracle's own write-up; test infrastructure only).

The paper fixes what is stored per pair -- an r-bit radius code, a t-bit angle
code, and per group a 16-bit scale and a 16-bit zero-point per pair (Section
3.2; Appendix B.1 for the 16-bit parameters) -- but not the byte layout.  The
layout below is this project's; the HIP library documents the same layout in
its public header and the two write-ups share no code.

  symbol      = (angle_code << r) | radius_code                    w = r + t bits
  unit        = 16 consecutive pairs' symbols of one token, as a little-endian
                bit string: symbol k occupies bits [k*w, (k+1)*w); bit i of the
                string is bit (i % 8) of byte (i // 8).  A unit is 2*w bytes.
  codes page  = [kv_head][pair_block = pair // 16][token_in_page][unit]
  params page = [kv_head][pair]{fp16 scale, fp16 zero}
                with the grouped angle quantizer: [kv_head][2][pair]{fp16 scale, fp16 zero},
                the radius parameters first, then the angle parameters
  value page  = [kv_head][token_in_page][d] fp16

A page holds `g` tokens (one quantization group).  Slots of a partial last
page beyond the sequence length hold zero bytes.

Quantized values (optional, b = 4 or 2 bits per element, token-wise parameters):
  value unit  = 16 bytes = T = 16 / b consecutive tokens x 8 consecutive dims:
                token i of the unit is the b*8-bit field [i*8*b, (i+1)*8*b) of the unit (little
                endian), and dim k of that token is the b-bit field k of it
  vq page     = [kv_head][token block = token // T][dim slice = dim // 8][unit]
  vq params   = [kv_head][token]{fp16 scale, fp16 zero}
"""
from __future__ import annotations

import numpy as np

PAIRS_PER_UNIT = 16


def unit_bytes(r_bits: int, t_bits: int) -> int:
    return 2 * (r_bits + t_bits)


def pack_units(a: np.ndarray, c: np.ndarray, r_bits: int, t_bits: int) -> np.ndarray:
    """[..., 16] angle and radius codes -> [..., 2*w] bytes."""
    w = r_bits + t_bits
    assert a.shape[-1] == PAIRS_PER_UNIT and a.shape == c.shape
    assert a.min(initial=0) >= 0 and a.max(initial=0) < (1 << t_bits)
    assert c.min(initial=0) >= 0 and c.max(initial=0) < (1 << r_bits)
    sym = (a.astype(np.int64) << r_bits) | c.astype(np.int64)
    bits = ((sym[..., None] >> np.arange(w)) & 1).astype(np.uint8)       # [..., 16, w], LSB first
    bits = bits.reshape(sym.shape[:-1] + (PAIRS_PER_UNIT * w,))
    return np.packbits(bits, axis=-1, bitorder="little")


def unpack_units(units: np.ndarray, r_bits: int, t_bits: int):
    """[..., 2*w] bytes -> (angle codes, radius codes), each int64 [..., 16]."""
    w = r_bits + t_bits
    assert units.dtype == np.uint8 and units.shape[-1] == 2 * w
    bits = np.unpackbits(units, axis=-1, bitorder="little")
    bits = bits.reshape(units.shape[:-1] + (PAIRS_PER_UNIT, w)).astype(np.int64)
    sym = (bits << np.arange(w)).sum(axis=-1)
    return sym >> r_bits, sym & ((1 << r_bits) - 1)


def pack_sequence(a, c, scale, zero, r_bits: int, t_bits: int, group_tokens: int, t_scale=None, t_zero=None):
    """Pages of one sequence.

    a, c: [L, H, P] codes; scale, zero (and t_scale, t_zero of the grouped angle quantizer):
    fp16 [n_pages, H, P].
    Returns (codes uint8 [n_pages, H, P/16, g, 2w], params fp16 [n_pages, H, P, 2], or
    [n_pages, H, 2, P, 2] with angle parameters).
    """
    L, H, P = a.shape
    assert P % PAIRS_PER_UNIT == 0
    g = group_tokens
    n_pages = (L + g - 1) // g
    nb = P // PAIRS_PER_UNIT
    ub = unit_bytes(r_bits, t_bits)
    codes = np.zeros((n_pages, H, nb, g, ub), np.uint8)
    units = pack_units(a.reshape(L, H, nb, PAIRS_PER_UNIT), c.reshape(L, H, nb, PAIRS_PER_UNIT),
                       r_bits, t_bits)                                    # [L, H, nb, ub]
    for p in range(n_pages):
        n0, n1 = p * g, min((p + 1) * g, L)
        codes[p, :, :, : n1 - n0, :] = units[n0:n1].transpose(1, 2, 0, 3)
    params = np.stack([scale.astype(np.float16), zero.astype(np.float16)], axis=-1)
    if t_scale is not None:
        t_params = np.stack([t_scale.astype(np.float16), t_zero.astype(np.float16)], axis=-1)
        params = np.stack([params, t_params], axis=2)
    return codes, params


def unpack_pages(codes: np.ndarray, params: np.ndarray, length: int, r_bits: int, t_bits: int):
    """Inverse of pack_sequence for the pages of one sequence, in order.

    codes uint8 [n_pages, H, P/16, g, 2w]; params fp16 [n_pages, H, P, 2].
    Returns (a, c) int64 [length, H, P] and (scale, zero) fp16 [n_pages, H, P]; for params of
    shape [n_pages, H, 2, P, 2] (grouped angle quantizer) also (t_scale, t_zero).
    """
    n_pages, H, nb, g, _ = codes.shape
    a, c = unpack_units(codes, r_bits, t_bits)                            # [n_pages, H, nb, g, 16]
    a = a.transpose(0, 3, 1, 2, 4).reshape(n_pages * g, H, nb * PAIRS_PER_UNIT)[:length]
    c = c.transpose(0, 3, 1, 2, 4).reshape(n_pages * g, H, nb * PAIRS_PER_UNIT)[:length]
    if params.ndim == 5:
        return a, c, params[:, :, 0, :, 0], params[:, :, 0, :, 1], params[:, :, 1, :, 0], params[:, :, 1, :, 1]
    return a, c, params[..., 0], params[..., 1]


def codes_bytes_per_page(n_kv_heads: int, head_dim: int, r_bits: int, t_bits: int, group_tokens: int) -> int:
    return n_kv_heads * group_tokens * (head_dim // 2) * (r_bits + t_bits) // 8


def params_bytes_per_page(n_kv_heads: int, head_dim: int, grouped_angles: bool = False) -> int:
    return n_kv_heads * (head_dim // 2) * 2 * 2 * (2 if grouped_angles else 1)


def _value_unit_order(bits: int):
    """How the T x 8 codes of a unit (T = 16 / bits tokens, 8 dims) are laid into its four 32-bit words.

    A word holds the codes of two consecutive tokens: the even token in the low 16 bits, the odd
    token in the high 16 bits, the same dims in both halves, dims in increasing order from bit 0.
    4-bit codes: a half holds 4 dims, so word j = 2 * (token pair) + (dim half: dims 0-3 / 4-7).
    2-bit codes: a half holds all 8 dims, so word j = token pair.
    Returns (token index, dim index) arrays of the 128 / bits fields in storage order (field 0 at
    bit 0 of word 0).
    """
    T = 16 // bits
    per_half = 16 // bits                       # fields in a 16-bit half
    tok, dim = [], []
    for word in range(4):
        if bits == 4:
            pair, dims0 = word // 2, 4 * (word % 2)
        else:
            pair, dims0 = word, 0
        for half in range(2):
            for f in range(per_half):
                tok.append(2 * pair + half)
                dim.append(dims0 + f)
    assert sorted(zip(tok, dim)) == [(t, k) for t in range(T) for k in range(8)]
    return np.array(tok), np.array(dim)


def pack_value_page_stream(codes: np.ndarray, bits: int, group_tokens: int) -> np.ndarray:
    """Quantized value codes of one sequence -> pages.

    codes int [L, H, d] (b-bit each) -> uint8 [n_pages, H, g / T, d / 8, 16], T = 16 / bits tokens
    per unit (see _value_unit_order for the inside of a unit); slots past the sequence end are zero.
    """
    L, H, d = codes.shape
    g = group_tokens
    T = 16 // bits
    n_pages = (L + g - 1) // g
    full = np.zeros((n_pages * g, H, d), np.int64)
    full[:L] = codes
    assert full.min() >= 0 and full.max() < (1 << bits)
    # [page, token block, token in unit, H, dim slice, dim in slice]
    x = full.reshape(n_pages, g // T, T, H, d // 8, 8)
    x = x.transpose(0, 3, 1, 4, 2, 5)                                       # [page, H, block, slice, T, 8]
    tok, dim = _value_unit_order(bits)
    fields = x[..., tok, dim]                                               # storage order
    bit_planes = ((fields[..., None] >> np.arange(bits)) & 1).astype(np.uint8)   # LSB first per field
    stream = bit_planes.reshape(n_pages, H, g // T, d // 8, T * 8 * bits)
    return np.packbits(stream, axis=-1, bitorder="little")


def unpack_value_pages(pages: np.ndarray, length: int, bits: int) -> np.ndarray:
    """Inverse of pack_value_page_stream: uint8 [n_pages, H, g/T, d/8, 16] -> int64 [length, H, d]."""
    n_pages, H, n_blocks, n_slices, _ = pages.shape
    T = 16 // bits
    b = np.unpackbits(pages, axis=-1, bitorder="little").reshape(n_pages, H, n_blocks, n_slices, T * 8, bits)
    fields = (b.astype(np.int64) << np.arange(bits)).sum(axis=-1)           # storage order
    tok, dim = _value_unit_order(bits)
    x = np.zeros((n_pages, H, n_blocks, n_slices, T, 8), np.int64)
    x[..., tok, dim] = fields
    x = x.transpose(0, 2, 4, 1, 3, 5).reshape(n_pages * n_blocks * T, H, n_slices * 8)
    return x[:length]
