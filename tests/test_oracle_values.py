"""Pins for the oracle's token-wise value quantizer and its packed layout."""
import math
import os

import numpy as np
import torch

from oracle import attention, cache_format, values


def test_worked_example(golden_dir):
    """Section 2 value quantizer on hand-worked rows: round-to-nearest (ties to even), divisor
    2^b - 1, zero-point = min, constant row, and Q * s + z."""
    with open(os.path.join(golden_dir, "value_quant_worked_example.txt")) as f:
        rows = [l for l in f if l.strip() and not l.startswith("#")]
    for line in rows:
        bits, v, sz, codes, deq = [[float(x) for x in part.split()] for part in line.split("|")]
        arr = np.array(v, np.float16).reshape(1, 1, -1)
        c, s, z = values.quantize_values(arr, int(bits[0]))
        assert [float(s[0, 0]), float(z[0, 0])] == sz
        assert c[0, 0].tolist() == codes
        assert values.dequant_values(c, s, z)[0, 0].tolist() == deq


def test_error_bound_and_extremes():
    """|V~ - V| <= s/2 up to the fp16 rounding of the scale; the row minimum is reproduced exactly
    (code 0, zero-point = min), the row maximum within that bound."""
    rng = np.random.default_rng(21)
    v = (rng.standard_normal((500, 3, 128)) * 2).astype(np.float16)
    for bits in (2, 4, 8):
        c, s, z = values.quantize_values(v, bits)
        vd = values.dequant_values(c, s, z)
        sd = s.astype(np.float64)[..., None]
        levels = (1 << bits) - 1
        bound = sd / 2 + levels * sd * 2.0 ** -11 + 1e-12
        assert np.all(np.abs(vd - v.astype(np.float64)) <= bound)
        assert c.min() == 0 and c.max() == levels
        imin = v.astype(np.float32).argmin(-1)
        np.testing.assert_array_equal(np.take_along_axis(vd, imin[..., None], -1)[..., 0], v.min(-1).astype(np.float64))
        assert np.all(np.take_along_axis(c, v.astype(np.float32).argmax(-1)[..., None], -1) == levels)


def test_error_halves_per_bit():
    rng = np.random.default_rng(22)
    v = rng.standard_normal((200, 2, 128)).astype(np.float16)
    errs = []
    for bits in (2, 3, 4, 5, 6, 7, 8):
        c, s, z = values.quantize_values(v, bits)
        errs.append(np.abs(values.dequant_values(c, s, z) - v.astype(np.float64)).max())
    for lo, hi in zip(errs[1:], errs[:-1]):
        assert lo < hi / 1.7


def test_value_pack_layout_by_hand():
    """Units: [token block][dim slice][16 bytes = four little-endian 32-bit words].  A word holds two
    consecutive tokens, the even one in bits 0-15 and the odd one in bits 16-31, dims upward from
    bit 0.  4 bits: word 2 * pair + (dims 0-3 | dims 4-7); 2 bits: word pair, all 8 dims of the slice."""
    L, H, d, g = 130, 1, 16, 128
    rng = np.random.default_rng(23)
    c4 = rng.integers(0, 16, (L, H, d))
    p4 = cache_format.pack_value_page_stream(c4, 4, g)
    assert p4.shape == (2, 1, 32, 2, 16)
    n, dim = 7, 13            # token block 1, token 3 of it = pair 1, odd; slice 1, dim 5 of it = upper dims, field 1
    word = int.from_bytes(bytes(p4[0, 0, 1, 1, 12:16]), "little")          # word 2 * 1 + 1 = 3
    assert (word >> (16 + 4 * 1)) & 15 == c4[n, 0, dim]
    assert (word >> (4 * 3)) & 15 == c4[6, 0, 15]                           # the even token of the pair, dim 7 of the slice
    n = 129                   # page 1, token 1: block 0, pair 0, odd
    w0 = int.from_bytes(bytes(p4[1, 0, 0, 0, 0:4]), "little")
    assert w0 == sum(int(c4[128, 0, f]) << (4 * f) for f in range(4)) | sum(int(c4[129, 0, f]) << (16 + 4 * f) for f in range(4))
    assert not p4[1, 0, 1:].any() and not p4[1, 0, 0, :, 8:].any()    # slots past token 129 are zero
    c2 = rng.integers(0, 4, (L, H, d))
    p2 = cache_format.pack_value_page_stream(c2, 2, g)
    assert p2.shape == (2, 1, 16, 2, 16)
    n, dim = 21, 10           # block 2 (8 tokens per unit), token 5 = pair 2, odd; slice 1, dim 2
    word = int.from_bytes(bytes(p2[0, 0, 2, 1, 8:12]), "little")            # word 2
    assert (word >> (16 + 2 * 2)) & 3 == c2[n, 0, dim]
    assert (word >> (2 * 7)) & 3 == c2[20, 0, 15]
    for bits, c in ((4, c4), (2, c2)):
        np.testing.assert_array_equal(cache_format.unpack_value_pages(
            cache_format.pack_value_page_stream(c, bits, g), L, bits), c)


def test_attention_over_quantized_values():
    """decode_attention with quantized value pages == attention over the dequantized values, and
    with 8-bit values it is within the quantization bound of attention over the fp16 values."""
    rng = np.random.default_rng(24)
    L, H, Hq, d, g = 300, 2, 4, 128, 128
    keys = rng.standard_normal((L, H, d)).astype(np.float16)
    vals = rng.standard_normal((L, H, d)).astype(np.float16)
    q = rng.standard_normal((1, Hq, d))
    from oracle import polar
    enc = polar.encode_keys(keys, 4, 4, g)
    codes, params = cache_format.pack_sequence(enc["a"], enc["c"], enc["scale"], enc["zero"], 4, 4, g)
    k_hat = polar.dequant_keys(enc["a"], enc["c"], enc["scale"], enc["zero"], 4, g)
    for bits in (4, 2):
        vc, vs, vz = values.quantize_values(vals, bits)
        pool = cache_format.pack_value_page_stream(vc, bits, g)
        par = np.zeros((3 * g, H, 2), np.float16)
        par[:L, :, 0], par[:L, :, 1] = vs, vz
        vq_params = par.reshape(3, g, H, 2).transpose(0, 2, 1, 3)
        got = attention.decode_attention(q, codes, params, pool, np.arange(3)[None], [L], 4, 4, g, 0.09,
                                         vq_params=vq_params, v_bits=bits)[0]
        want = attention.attend(q[0], k_hat, values.dequant_values(vc, vs, vz), 0.09)
        np.testing.assert_allclose(got[1], want[1], atol=1e-12)
        exact = attention.attend(q[0], k_hat, vals.astype(np.float64), 0.09)
        assert np.abs(got[1] - exact[1]).max() <= float(vs.astype(np.float64).max()) / 2 + 1e-3
