"""Pins for the CPU oracle: it is checked against what the paper and the
mathematics fix, never against itself.

Each test names the passage it pins.  A plausible mistake anywhere in the
oracle (round instead of floor, 2^r-1 instead of 2^r, a missing mid-point,
pairs (2j, 2j+1) instead of (j, j+d/2), a "+pi" left in the reconstruction, a
transposed gather, statistics over padded tokens ...) fails at least one.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import attention, cache_format, polar
from paper_2502_00527_amd import workloads

pytestmark = pytest.mark.filterwarnings("ignore::RuntimeWarning")


# --------------------------------------------------------------------------- worked example

def _read_golden(path):
    rows = []
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            rows.append([[float(v) for v in part.split()] for part in line.split("|")])
    return rows


def test_worked_example(golden_dir):
    """Section 3.2 quantizer + dequantizer and the Appendix A product, on hand-worked numbers."""
    rows = _read_golden(os.path.join(golden_dir, "polar_worked_example.txt"))
    keys = np.array([r[0] for r in rows], np.float32).reshape(4, 1, 2)
    enc = polar.encode_keys(keys, r_bits=2, t_bits=3, group_tokens=4)
    assert enc["rho"][:, 0, 0].tolist() == [r[1][0] for r in rows]
    assert enc["c"][:, 0, 0].tolist() == [int(r[2][0]) for r in rows]
    assert enc["a"][:, 0, 0].tolist() == [int(r[2][1]) for r in rows]
    assert float(enc["scale"][0, 0, 0]) == 1.0 and float(enc["zero"][0, 0, 0]) == 1.0
    rho_t = polar.dequant_radius(enc["c"], enc["scale"], enc["zero"], 4)[:, 0, 0]
    th_t = polar.dequant_angle(enc["a"], 3)[:, 0, 0]
    np.testing.assert_allclose(rho_t, [r[3][0] for r in rows], atol=1e-12)
    np.testing.assert_allclose(th_t, [r[3][1] for r in rows], atol=1e-9)
    k_hat = polar.dequant_keys(enc["a"], enc["c"], enc["scale"], enc["zero"], 3, 4)
    np.testing.assert_allclose(k_hat[:, 0, :], [r[4] for r in rows], atol=1e-9)
    scores, _ = attention.attend(np.array([[1.0, 2.0]]), k_hat, np.zeros((4, 1, 2)), 1.0)
    np.testing.assert_allclose(scores[0], [r[5][0] for r in rows], atol=1e-8)


# --------------------------------------------------------------------------- radius

def test_radius_is_norm_of_rotate_half_pair():
    """rho_n[j] = ||(K[j], K[j+d/2])|| (Section 3.2 with the pairing of footnote 2)."""
    rng = np.random.default_rng(1)
    keys = rng.standard_normal((37, 3, 128)).astype(np.float32)
    enc = polar.encode_keys(keys, 4, 4, 16)
    for j in (0, 1, 17, 63):
        ref = np.hypot(keys[..., j].astype(np.float64), keys[..., j + 64].astype(np.float64))
        np.testing.assert_allclose(enc["rho"][..., j], ref, rtol=2e-7)
    # one-hot pair: only dims 5 and 69 are non-zero -> only pair 5 has a radius
    k = np.zeros((1, 1, 128), np.float32)
    k[0, 0, 5], k[0, 0, 69] = 3.0, -4.0
    rho = polar.encode_keys(k, 4, 4, 1)["rho"][0, 0]
    assert rho[5] == 5.0 and np.count_nonzero(rho) == 1


def test_rotation_preserves_radius():
    """RoPE is a rotation of each pair, so radii are those of the un-rotated key (Section 1)."""
    rng = np.random.default_rng(2)
    k = rng.standard_normal((64, 2, 128)).astype(np.float32)
    cos, sin = workloads.rope_tables(128, 1.0e4, np.arange(1000, 1064))
    kr = workloads.apply_rope_rotate_half(k, cos, sin)
    r0 = polar.radius_f32(*polar.split_pairs(k))
    r1 = polar.radius_f32(*polar.split_pairs(kr))
    np.testing.assert_allclose(r1, r0, rtol=1e-5, atol=1e-6)


def test_outlier_pair_has_narrow_radius_range():
    """An outlier in one coordinate of a pair widens the per-channel range far more than
    the radius range once it is rotated (Section 3.1, the Observation)."""
    wl = workloads.WORKLOADS["tiny"].scaled(max_len=2048, min_len=2048)
    k = workloads.keys_for_seq(wl, 0, 2048).astype(np.float64)
    pairs, _ = workloads.outlier_channels(wl)
    rho = np.hypot(k[..., :64], k[..., 64:])
    for p in pairs[0]:
        chan_range = np.ptp(k[:, 0, p])                      # channel-wise quantizer sees [-max, +max]
        rad_range = np.ptp(rho[:, 0, p])
        chan_mean = np.abs(k[:, 0, p]).mean()
        assert rad_range < chan_range                        # radius is one-sided
        assert chan_mean > 2.0                               # the outlier channel is an outlier


# --------------------------------------------------------------------------- angle grid

def test_angle_bins_on_axes_and_diagonals():
    """Uniform grid over [-pi, pi), half-open bins, theta=+pi clamped, origin -> theta=0."""
    t = 4                                                     # bins of pi/8; bin k starts at -pi + k*pi/8
    x = np.array([1, 1, 0, -1, -1, -1, 0, 1, 0, -1], np.float32)
    y = np.array([0, 1, 1, 1, 0.0, -1, -1, -1, 0, -0.0], np.float32)
    #     theta: 0 pi/4 pi/2 3pi/4 pi  -3pi/4 -pi/2 -pi/4  0   -pi
    want = [8, 10, 12, 14, 15, 2, 4, 6, 8, 0]
    code, edge = polar.angle_bin(x, y, t)
    assert code.tolist() == want
    assert np.all(edge == 0.0)
    # scale invariance of the ties (fp16-sized magnitudes, tiny and huge)
    for s in (2.0 ** -14, 3.0, 1024.0):
        assert polar.angle_bin(x * np.float32(s), y * np.float32(s), t)[0].tolist() == want
    # t = 2: diagonals are bin centres, not edges
    code2, edge2 = polar.angle_bin(x[:8], y[:8], 2)
    assert code2.tolist() == [2, 2, 3, 3, 3, 0, 1, 1]
    np.testing.assert_allclose(edge2[1::2], np.pi / 4, rtol=1e-12)


def test_angle_bin_matches_bruteforce_scan():
    """floor((theta+pi)/D) equals a brute-force scan for the arc that contains theta."""
    rng = np.random.default_rng(3)
    x = rng.standard_normal(2000).astype(np.float32)
    y = rng.standard_normal(2000).astype(np.float32)
    for t in (1, 3, 4, 6):
        code, edge = polar.angle_bin(x, y, t)
        D = 2 * math.pi / (1 << t)
        for i in range(0, 2000, 7):
            th = math.atan2(float(y[i]), float(x[i]))
            k = [k for k in range(1 << t) if -math.pi + k * D <= th < -math.pi + (k + 1) * D]
            assert k == [int(code[i])]
            lo = th - (-math.pi + code[i] * D)
            assert abs(min(lo, D - lo) - edge[i]) < 1e-12


# --------------------------------------------------------------------------- radius quantizer details

def test_partial_group_uses_valid_tokens_only():
    """Group statistics run over the tokens the group really has."""
    rng = np.random.default_rng(4)
    keys = rng.standard_normal((10, 1, 32)).astype(np.float32)
    enc = polar.encode_keys(keys, 3, 3, 8)                  # groups: tokens 0..7 and 8..9
    rho = enc["rho"]
    assert enc["scale"].shape == (2, 1, 16)
    np.testing.assert_array_equal(enc["zero"][1], rho[8:10].min(0).astype(np.float16))
    np.testing.assert_array_equal(enc["scale"][1], ((rho[8:10].max(0) - rho[8:10].min(0)) / np.float32(8)).astype(np.float16))
    np.testing.assert_array_equal(enc["zero"][0], rho[0:8].min(0).astype(np.float16))


def test_codes_are_taken_against_stored_fp16_params():
    """16-bit parameters (Appendix B.1): the code uses the rounded zero-point, so a
    zero-point rounded above the minimum gives a negative quotient that Clamp absorbs."""
    # radius 1.0004 rounds to fp16 1.0009765625 (above): quotient < 0 -> code 0
    keys = np.zeros((4, 1, 2), np.float32)
    keys[:, 0, 0] = [1.0006, 1.3, 1.7, 2.0]
    enc = polar.encode_keys(keys, 2, 2, 4)
    z = float(enc["zero"][0, 0, 0])
    assert z > 1.0006
    assert enc["c"][0, 0, 0] == 0
    s = float(enc["scale"][0, 0, 0])
    for n in range(4):
        want = min(3, max(0, math.floor((float(enc["rho"][n, 0, 0]) - z) / s)))
        assert enc["c"][n, 0, 0] == want


def test_constant_radius_group_is_exact():
    """max == min -> scale 0 -> code 0 and rho~ = z: the radius is reproduced exactly."""
    # identical float32 radii: exactly representable points on axes / 3-4-5 triangles
    keys = np.array([[3, 4], [4, 3], [-3, 4], [5, 0], [0, -5], [-4, -3], [-5, 0], [0, 5]], np.float32).reshape(8, 1, 2)
    enc = polar.encode_keys(keys, 4, 4, 8)
    assert float(enc["scale"][0, 0, 0]) == 0.0 and np.all(enc["c"] == 0)
    np.testing.assert_array_equal(polar.dequant_radius(enc["c"], enc["scale"], enc["zero"], 8), 5.0)


# --------------------------------------------------------------------------- reconstruction quality

def _recon_error(keys, r, t, g, pdt):
    enc = polar.encode_keys(keys, r, t, g, param_dtype=pdt)
    k_hat = polar.dequant_keys(enc["a"], enc["c"], enc["scale"], enc["zero"], t, g)
    return np.abs(k_hat - keys.astype(np.float64)).max(), enc, k_hat


def test_reconstruction_error_bound_per_pair():
    """Mid-point reconstruction of a floor quantizer: |rho~-rho| <= s/2 (+ fp16 rounding of
    the zero-point) and |theta~-theta| <= D/2, so the pair error is bounded by
    s/2 + eps16 + 2*rho*sin(D/4).  Also pins k~ ~ k (not -k: no +pi in the reconstruction)."""
    wl = workloads.WORKLOADS["mha"].scaled(n_kv_heads=2, n_q_heads=2)
    keys = workloads.keys_for_seq(wl, 0, 300)
    for r, t in ((4, 4), (3, 3), (2, 5)):
        enc = polar.encode_keys(keys, r, t, 128)
        k_hat = polar.dequant_keys(enc["a"], enc["c"], enc["scale"], enc["zero"], t, 128)
        kd = keys.astype(np.float64)
        err = np.hypot(k_hat[..., :64] - kd[..., :64], k_hat[..., 64:] - kd[..., 64:])
        grp = np.arange(300) // 128
        s = enc["scale"].astype(np.float64)[grp]
        z = enc["zero"].astype(np.float64)[grp]
        rho = enc["rho"].astype(np.float64)
        D = 2 * np.pi / (1 << t)
        eps16 = 2.0 ** -11 * np.maximum(z, 2.0 ** -14) + (1 << r) * 2.0 ** -11 * s   # fp16 rounding of z and s
        bound = s / 2 + eps16 + 2 * np.maximum(rho, z + (1 << r) * s) * np.sin(D / 4) + 1e-6
        assert np.all(err <= bound)
        assert np.sum(k_hat * kd) > 0.9 * np.sum(kd * kd)


def test_lossless_as_bits_grow():
    """Each extra radius+angle bit halves the worst-case error; with float32 parameters
    (no 16-bit floor) the reconstruction converges to the key."""
    rng = np.random.default_rng(5)
    keys = rng.standard_normal((256, 2, 64)).astype(np.float32)
    errs = [_recon_error(keys, b, b, 128, np.float32)[0] for b in (2, 4, 6, 8, 10, 12, 14)]
    for lo, hi in zip(errs[1:], errs[:-1]):
        assert lo < hi / 3.0                                  # two bits each: ~4x
    assert errs[-1] < 2e-3 and _recon_error(keys, 16, 16, 128, np.float32)[0] < 4e-4
    # with the paper's 16-bit parameters the floor is the fp16 rounding of the zero-point
    assert _recon_error(keys, 14, 14, 128, np.float16)[0] < 4e-3


# --------------------------------------------------------------------------- scores

def test_lut_identity_bruteforce():
    """q . k~ = sum_j rho~_j |q_j| cos(theta~_j - phi_j), phi_j = atan2(q_y, q_x)
    (the lookup-table view of Section 3.3), by scalar loops on a tiny input."""
    rng = np.random.default_rng(6)
    L, H, d, g, r, t = 9, 1, 32, 4, 3, 4
    keys = rng.standard_normal((L, H, d)).astype(np.float32)
    q = rng.standard_normal((1, d))
    enc = polar.encode_keys(keys, r, t, g)
    k_hat = polar.dequant_keys(enc["a"], enc["c"], enc["scale"], enc["zero"], t, g)
    scores, _ = attention.attend(q, k_hat, np.zeros((L, H, d)), 1.0)
    for n in range(L):
        acc = 0.0
        for j in range(d // 2):
            s = float(enc["scale"][n // g, 0, j])
            z = float(enc["zero"][n // g, 0, j])
            rho = (int(enc["c"][n, 0, j]) + 0.5) * s + z
            th = -math.pi + (int(enc["a"][n, 0, j]) + 0.5) * 2 * math.pi / (1 << t)
            qx, qy = float(q[0, j]), float(q[0, j + d // 2])
            acc += rho * math.hypot(qx, qy) * math.cos(th - math.atan2(qy, qx))
        assert abs(acc - scores[0, n]) < 1e-12 * max(1.0, abs(acc))


def _lut_gather_product(q, a, c, scale, zero, r_bits, t_bits):
    """Semantics of the appendix's reference listing for ONE group: a table of the 2^t
    angle states times the query pair, gathered by angle code, times the gathered radius
    level, summed over pairs.  q [d]; a, c [G, P]; scale, zero [P] -> [G]."""
    P = a.shape[1]
    phi = (np.arange(1 << t_bits) + 0.5) * (2 * np.pi / (1 << t_bits)) - np.pi          # [2^t]
    table = q[None, :P] * np.cos(phi)[:, None] + q[None, P:] * np.sin(phi)[:, None]      # [2^t, P]
    levels = (np.arange(1 << r_bits)[:, None] + 0.5) * scale[None, :] + zero[None, :]    # [2^r, P]
    cols = np.arange(P)[None, :]
    return (table[a, cols] * levels[c, cols]).sum(axis=1)


def test_table_gather_formulation_equals_dequant_dot():
    """Appendix A: the table/gather product is the dequantize-then-dot product re-ordered."""
    rng = np.random.default_rng(7)
    g, r, t = 128, 4, 4
    keys = rng.standard_normal((g, 1, 128)).astype(np.float32) * 3
    q = rng.standard_normal(128)
    enc = polar.encode_keys(keys, r, t, g)
    k_hat = polar.dequant_keys(enc["a"], enc["c"], enc["scale"], enc["zero"], t, g)
    direct, _ = attention.attend(q[None], k_hat, np.zeros((g, 1, 128)), 1.0)
    lut = _lut_gather_product(q, enc["a"][:, 0], enc["c"][:, 0], enc["scale"][0, 0].astype(np.float64),
                              enc["zero"][0, 0].astype(np.float64), r, t)
    np.testing.assert_allclose(lut, direct[0], rtol=0, atol=1e-11)


# --------------------------------------------------------------------------- attention

def test_attention_reduces_to_textbook_in_the_fine_limit():
    """With many bits and float32 parameters the path is softmax(q K^T / sqrt(d)) V."""
    rng = np.random.default_rng(8)
    L, Hq, Hkv, d, g = 200, 4, 2, 64, 64
    keys = rng.standard_normal((L, Hkv, d)).astype(np.float32)
    v = rng.standard_normal((L, Hkv, d)).astype(np.float16)
    q = rng.standard_normal((Hq, d))
    enc = polar.encode_keys(keys, 15, 15, g, param_dtype=np.float32)
    k_hat = polar.dequant_keys(enc["a"], enc["c"], enc["scale"], enc["zero"], 15, g)
    scores, out = attention.attend(q, k_hat, v.astype(np.float64), 1 / math.sqrt(d))
    tq = torch.from_numpy(q)[None, :, None, :]                                         # [1, Hq, 1, d]
    tk = torch.from_numpy(keys.astype(np.float64)).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    tv = torch.from_numpy(v.astype(np.float64)).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    np.testing.assert_allclose(out, ref, atol=2e-3)
    ref_scores = torch.einsum("hd,hld->hl", torch.from_numpy(q), tk[0]).numpy()
    np.testing.assert_allclose(scores, ref_scores, atol=2e-3)
    # GQA mapping: query heads 0,1 -> kv head 0; 2,3 -> kv head 1 (a swapped mapping fails above)


def test_softmax_weights_are_convex():
    rng = np.random.default_rng(9)
    k_hat = rng.standard_normal((50, 1, 8))
    v = np.ones((50, 1, 8)) * 3.25
    _, out = attention.attend(rng.standard_normal((1, 8)) * 30, k_hat, v, 1.0)
    np.testing.assert_allclose(out, 3.25, rtol=1e-14)


# --------------------------------------------------------------------------- packed format

def test_pack_roundtrip_all_symbols_and_size():
    """Every (angle, radius) symbol at every pair position survives pack/unpack; the packed
    cache costs (r+t)/2 bits per element plus 32/g bits per PAIR of parameters -- i.e.
    4 + 16/128 = 4.125 bits per key element at r=t=4, g=128 (Appendix B.1 accounting with
    the uniform angle grid: no angle parameters)."""
    for r, t in ((4, 4), (3, 3), (5, 3), (2, 4)):
        n_sym = 1 << (r + t)
        sym = (np.arange(n_sym)[:, None] + np.arange(16)[None, :] * 7) % n_sym
        a, c = sym >> r, sym & ((1 << r) - 1)
        units = cache_format.pack_units(a, c, r, t)
        assert units.shape == (n_sym, 2 * (r + t))
        a2, c2 = cache_format.unpack_units(units, r, t)
        np.testing.assert_array_equal(a2, a)
        np.testing.assert_array_equal(c2, c)
    cb = cache_format.codes_bytes_per_page(8, 128, 4, 4, 128)
    pb = cache_format.params_bytes_per_page(8, 128)
    assert (cb + pb) * 8 / (8 * 128 * 128) == 4.125
    assert (cache_format.codes_bytes_per_page(8, 128, 3, 3, 128) + pb) * 8 / (8 * 128 * 128) == 3.125


def test_pack_bit_order_by_hand():
    """4+4: byte k of a unit is (angle << 4) | radius.  3+3: symbols are 6-bit fields of a
    little-endian bit string: bytes 0..2 hold symbols 0..3 as s0 | s1<<6 | s2<<12 | s3<<18."""
    a = np.arange(16)[None, :] % 16
    c = (15 - np.arange(16))[None, :]
    u = cache_format.pack_units(a, c, 4, 4)[0]
    assert u.tolist() == [(int(a[0, k]) << 4) | int(c[0, k]) for k in range(16)]
    a3 = np.array([[5, 0, 7, 1] + [0] * 12])
    c3 = np.array([[2, 7, 0, 4] + [0] * 12])
    s = [(int(a3[0, k]) << 3) | int(c3[0, k]) for k in range(4)]
    word = s[0] | (s[1] << 6) | (s[2] << 12) | (s[3] << 18)
    u3 = cache_format.pack_units(a3, c3, 3, 3)[0]
    assert u3[:3].tolist() == [word & 255, (word >> 8) & 255, (word >> 16) & 255]
    assert len(u3) == 12 and not u3[3:].any()


def test_page_layout_and_padding():
    """codes page = [head][pair block][token][unit]; padded slots are zero bytes."""
    rng = np.random.default_rng(10)
    L, H, P, g = 150, 2, 32, 128
    a = rng.integers(0, 16, (L, H, P))
    c = rng.integers(0, 16, (L, H, P))
    scale = rng.random((2, H, P)).astype(np.float16)
    zero = rng.random((2, H, P)).astype(np.float16)
    codes, params = cache_format.pack_sequence(a, c, scale, zero, 4, 4, g)
    assert codes.shape == (2, H, 2, g, 16) and params.shape == (2, H, P, 2)
    n, h, j = 131, 1, 21                                        # page 1, slot 3, block 1, k 5
    assert codes[1, h, 1, 3, 5] == (a[n, h, j] << 4) | c[n, h, j]
    assert not codes[1, :, :, L - g:, :].any()
    assert params[1, h, j, 0] == scale[1, h, j] and params[1, h, j, 1] == zero[1, h, j]
    a2, c2, s2, z2 = cache_format.unpack_pages(codes, params, L, 4, 4)
    np.testing.assert_array_equal(a2, a)
    np.testing.assert_array_equal(c2, c)


def test_paged_decode_equals_contiguous():
    """Scattering a sequence's pages through the pool changes nothing."""
    wl = workloads.WORKLOADS["ragged"].scaled(n_seqs=3, n_q_heads=4, n_kv_heads=2, max_len=400, min_len=100)
    lens = workloads.seq_lengths(wl)
    table, total = workloads.page_table(wl, lens)
    assert sorted(table[table >= 0].tolist()) == list(range(total))
    g, r, t = 128, 4, 4
    codes_pool = np.zeros((total, 2, 4, g, 16), np.uint8)
    params_pool = np.zeros((total, 2, 64, 2), np.float16)
    v_pool = np.zeros((total, 2, g, 128), np.float16)
    q = workloads.queries(wl)
    want = {}
    for s in range(3):
        L = int(lens[s])
        keys = workloads.keys_for_seq(wl, s, L)
        vals = workloads.values_for_seq(wl, s, L)
        enc = polar.encode_keys(keys, r, t, g)
        cp, pp = cache_format.pack_sequence(enc["a"], enc["c"], enc["scale"], enc["zero"], r, t, g)
        ids = table[s, : cp.shape[0]]
        codes_pool[ids], params_pool[ids] = cp, pp
        vp = np.zeros((cp.shape[0] * g, 2, 128), np.float16)
        vp[:L] = vals
        v_pool[ids] = vp.reshape(cp.shape[0], g, 2, 128).transpose(0, 2, 1, 3)
        k_hat = polar.dequant_keys(enc["a"], enc["c"], enc["scale"], enc["zero"], t, g)
        want[s] = attention.attend(q[s].astype(np.float64), k_hat, vals.astype(np.float64), 0.1)
    got = attention.decode_attention(q, codes_pool, params_pool, v_pool, table, lens, r, t, g, 0.1)
    for s in range(3):
        np.testing.assert_allclose(got[s][0], want[s][0], atol=1e-12)
        np.testing.assert_allclose(got[s][1], want[s][1], atol=1e-12)


# --------------------------------------------------------------------------- residual keys

def test_residual_keys_are_scored_unquantized():
    """With a residual buffer the incomplete last group is plain fp16 keys (Appendix B.1): a
    sequence shorter than one group is textbook attention on the fp16 keys, and in a longer one
    only the complete groups are reconstructed from codes."""
    rng = np.random.default_rng(11)
    g, H, Hq, d, r, t = 128, 2, 4, 128, 4, 4
    L = 300
    keys = rng.standard_normal((L, H, d)).astype(np.float16)
    vals = rng.standard_normal((L, H, d)).astype(np.float16)
    q = rng.standard_normal((1, Hq, d))
    n_full = L // g
    enc = polar.encode_keys(keys[: n_full * g], r, t, g)
    codes, params = cache_format.pack_sequence(enc["a"], enc["c"], enc["scale"], enc["zero"], r, t, g)
    n_pages = n_full + 1
    codes_pool = np.concatenate([codes, np.full((1,) + codes.shape[1:], 0xEE, np.uint8)])      # junk page
    params_pool = np.concatenate([params, np.full((1,) + params.shape[1:], np.nan, np.float16)])
    v = np.zeros((n_pages * g, H, d), np.float16)
    v[:L] = vals
    v_pool = v.reshape(n_pages, g, H, d).transpose(0, 2, 1, 3)
    residual = np.full((1, H, g, d), np.nan, np.float16)
    residual[0, :, : L - n_full * g] = keys[n_full * g:].transpose(1, 0, 2)
    table = np.arange(n_pages)[None, :]
    res = attention.decode_attention(q, codes_pool, params_pool, v_pool, table, [L], r, t, g, 0.09,
                                     residual=residual)[0]
    k_hat = polar.dequant_keys(enc["a"], enc["c"], enc["scale"], enc["zero"], t, g)
    k_all = np.concatenate([k_hat, keys[n_full * g:].astype(np.float64)])
    want = attention.attend(q[0], k_all, vals.astype(np.float64), 0.09)
    np.testing.assert_allclose(res[0], want[0], atol=1e-12)
    np.testing.assert_allclose(res[1], want[1], atol=1e-12)
    # the tail scores are exact dot products with the fp16 keys
    exact = np.einsum("hd,ld->hl", q[0][:2], keys[n_full * g:, 0, :].astype(np.float64))
    np.testing.assert_allclose(res[0][:2, n_full * g:], exact, atol=1e-12)
    # shorter than a group: textbook attention (torch float64) on the fp16 keys
    Ls = 77
    resid2 = np.full((1, H, g, d), np.nan, np.float16)
    resid2[0, :, :Ls] = keys[:Ls].transpose(1, 0, 2)
    v2 = np.zeros((g, H, d), np.float16)
    v2[:Ls] = vals[:Ls]
    out2 = attention.decode_attention(q, codes_pool[-1:], params_pool[-1:], v2.reshape(1, g, H, d).transpose(0, 2, 1, 3),
                                      np.zeros((1, 1), int), [Ls], r, t, g, 1 / math.sqrt(d), residual=resid2)[0][1]
    tq = torch.from_numpy(q[0])[None, :, None, :]
    tk = torch.from_numpy(keys[:Ls].astype(np.float64)).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    tv = torch.from_numpy(vals[:Ls].astype(np.float64)).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv)[0, :, 0, :].numpy()
    np.testing.assert_allclose(out2, ref, atol=1e-12)
