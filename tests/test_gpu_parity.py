"""Parity of the HIP library (through its C ABI) with the CPU oracle, element by element.

Small cases span several pages, several chunks, ragged tails, every supported bit
allocation and query-group size; full-size cases run the launch configuration the
benchmark times and compare sampled sequences.
"""
import sys

import numpy as np
import pytest
import torch

from paper_2502_00527_amd import workloads as W

from parity import (EDGE_FRACTION, OUT_ABS, SCORE_REL, OracleSeq, compare_encoding, score_errors)

pytestmark = pytest.mark.gpu

WL = W.WORKLOADS


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


SMALL = {
    # name: (workload, explicit lengths or None)
    "tiny_full_config": (WL["tiny"], None),                                               # G=1, fp32, 32 pages
    "mha_two_seqs": (WL["mha"].scaled(n_seqs=2, n_q_heads=4, n_kv_heads=4, max_len=700, min_len=700), None),
    "gqa_ragged_tail": (WL["gqa"].scaled(n_seqs=2, n_q_heads=8, n_kv_heads=2, max_len=1000, min_len=1000), None),
    "gqa_many_chunks": (WL["gqa"].scaled(n_seqs=1, n_q_heads=4, n_kv_heads=1, max_len=5000, min_len=5000), None),
    "long33": (WL["long33"].scaled(n_q_heads=8, n_kv_heads=2, max_len=3001, min_len=3001), None),
    "ragged_pages": (WL["ragged"].scaled(n_seqs=6, n_q_heads=8, n_kv_heads=2, max_len=2000, min_len=1), None),
    "group_of_two": (WL["gqa"].scaled(n_seqs=2, n_q_heads=4, n_kv_heads=2, max_len=900, min_len=900), None),
    "edge_lengths": (WL["gqa"].scaled(n_seqs=5, n_q_heads=4, n_kv_heads=1, max_len=300, min_len=300),
                     np.array([0, 1, 128, 129, 300], np.int32)),
    "many_units_big_chunks": (WL["mha"].scaled(n_seqs=64, max_len=200, min_len=200), None),
    "bits_r5t3": (WL["gqa"].scaled(n_seqs=1, n_q_heads=4, n_kv_heads=1, max_len=777, min_len=777, r_bits=5, t_bits=3), None),
    "bits_r3t5": (WL["gqa"].scaled(n_seqs=1, n_q_heads=4, n_kv_heads=1, max_len=777, min_len=777, r_bits=3, t_bits=5), None),
    "bits_r4t2": (WL["gqa"].scaled(n_seqs=1, n_q_heads=2, n_kv_heads=1, max_len=777, min_len=777, r_bits=4, t_bits=2), None),
    "bits_r2t4": (WL["gqa"].scaled(n_seqs=1, n_q_heads=1, n_kv_heads=1, max_len=777, min_len=777, r_bits=2, t_bits=4), None),
    "tiny33_fp32": (WL["tiny"].scaled(max_len=1500, min_len=1500, r_bits=3, t_bits=3), None),
    "group_of_six": (WL["gqa"].scaled(n_seqs=2, n_q_heads=12, n_kv_heads=2, max_len=650, min_len=650), None),   # 4 + 2
    "group_of_seven": (WL["gqa"].scaled(n_seqs=1, n_q_heads=7, n_kv_heads=1, max_len=400, min_len=400, r_bits=3, t_bits=3), None),
    "group_of_eight": (WL["gqa"].scaled(n_seqs=1, n_q_heads=16, n_kv_heads=2, max_len=520, min_len=520), None),  # 4 + 4
    # the paper's grouped (per-group min / scale) angle quantizer
    "grouped_angles_gqa": (WL["gqa"].scaled(n_seqs=2, n_q_heads=8, n_kv_heads=2, max_len=1000, min_len=1000,
                                            grouped_angles=True), None),
    "grouped_angles_tiny_fp32": (WL["tiny"].scaled(max_len=2100, min_len=2100, grouped_angles=True), None),
    "grouped_angles_r3t3_many_chunks": (WL["long33"].scaled(n_q_heads=4, n_kv_heads=2, max_len=5001, min_len=5001,
                                                            grouped_angles=True), None),
    "grouped_angles_edge_lengths": (WL["gqa"].scaled(n_seqs=5, n_q_heads=6, n_kv_heads=1, max_len=300, min_len=300,
                                                     grouped_angles=True), np.array([0, 1, 128, 129, 300], np.int32)),
    "grouped_angles_ragged_pages": (WL["ragged"].scaled(n_seqs=6, n_q_heads=8, n_kv_heads=2, max_len=2000, min_len=1,
                                                        grouped_angles=True), None),
    # ... with the bit allocations of the paper's ablation (Section 6.1)
    "grouped_angles_r5t3": (WL["gqa"].scaled(n_seqs=2, n_q_heads=8, n_kv_heads=2, max_len=700, min_len=700, r_bits=5, t_bits=3,
                                             grouped_angles=True), None),
    "grouped_angles_r3t5": (WL["gqa"].scaled(n_seqs=2, n_q_heads=4, n_kv_heads=2, max_len=700, min_len=700, r_bits=3, t_bits=5,
                                             grouped_angles=True), None),
    "grouped_angles_r4t2": (WL["mha"].scaled(n_seqs=2, n_q_heads=2, n_kv_heads=2, max_len=700, min_len=700, r_bits=4, t_bits=2,
                                             grouped_angles=True), None),
    "grouped_angles_r2t4": (WL["gqa"].scaled(n_seqs=2, n_q_heads=12, n_kv_heads=2, max_len=700, min_len=700, r_bits=2, t_bits=4,
                                             grouped_angles=True, key_dtype="f32"), None),
}


# Launches of at least 256 work-groups with fp16 values and the uniform grid are served by the
# role-specialised attention kernel; these cases stay small for the oracle (a few hundred tokens
# per sequence) but have enough (sequence, KV head, chunk) units to be dispatched to it.  Between
# them they cover every bit allocation, both query dtypes, query groups of 1, 2, 4 and the
# multi-pass groups 6 and 8, chunks with an odd page count, ragged and empty sequences.
_BIG = dict(n_seqs=32, n_kv_heads=8, max_len=777, min_len=777)
LARGE_GRID = {
    "big_r4t4_g4": (WL["gqa"].scaled(n_q_heads=32, **_BIG), None),
    "big_r3t3_g4": (WL["gqa"].scaled(n_q_heads=32, r_bits=3, t_bits=3, **_BIG), None),
    "big_r5t3_g4": (WL["gqa"].scaled(n_q_heads=32, r_bits=5, t_bits=3, **_BIG), None),
    "big_r3t5_g2": (WL["gqa"].scaled(n_q_heads=16, r_bits=3, t_bits=5, **_BIG), None),
    "big_r4t2_g1": (WL["gqa"].scaled(n_q_heads=8, r_bits=4, t_bits=2, **_BIG), None),
    "big_r2t4_g4": (WL["gqa"].scaled(n_q_heads=32, r_bits=2, t_bits=4, **_BIG), None),
    "big_r5t3_g1": (WL["mha"].scaled(n_q_heads=8, r_bits=5, t_bits=3, **_BIG), None),
    "big_r2t4_g2": (WL["mha"].scaled(n_q_heads=16, r_bits=2, t_bits=4, **_BIG), None),
    "big_fp32_r4t4_g4": (WL["gqa"].scaled(n_q_heads=32, key_dtype="f32", **_BIG), None),
    "big_fp32_r3t3_g2": (WL["gqa"].scaled(n_q_heads=16, key_dtype="f32", r_bits=3, t_bits=3, **_BIG), None),
    "big_fp32_r3t5_g1": (WL["gqa"].scaled(n_q_heads=8, key_dtype="f32", r_bits=3, t_bits=5, **_BIG), None),
    "big_group_of_six": (WL["gqa"].scaled(n_q_heads=48, **_BIG), None),                           # 4 + 2
    "big_group_of_eight_r3t3": (WL["gqa"].scaled(n_q_heads=64, r_bits=3, t_bits=3, **_BIG), None),  # 4 + 4
    "big_group_of_seven_r4t2": (WL["gqa"].scaled(n_q_heads=56, r_bits=4, t_bits=2, **_BIG), None),  # 4 + 2 + 1
    # 8 query heads per KV head are served in one pass (two tables, fp16 probability pairs)
    "big_group_of_eight_r4t4": (WL["gqa"].scaled(n_q_heads=64, **_BIG), None),
    "big_group_of_eight_r5t3_fp32": (WL["gqa"].scaled(n_q_heads=64, r_bits=5, t_bits=3, key_dtype="f32", **_BIG), None),
    "big_group_of_eight_r3t5": (WL["mha"].scaled(n_q_heads=64, r_bits=3, t_bits=5, **_BIG), None),
    "big_group_of_twelve_r4t2": (WL["gqa"].scaled(n_seqs=32, n_kv_heads=8, n_q_heads=96, max_len=520, min_len=520,
                                                  r_bits=4, t_bits=2), None),                              # 8 + 4
    "big_group_of_sixteen_r2t4": (WL["gqa"].scaled(n_seqs=32, n_kv_heads=8, n_q_heads=128, max_len=520, min_len=520,
                                                   r_bits=2, t_bits=4), None),                             # 8 + 8
    "big_ragged_group_of_eight": (WL["ragged"].scaled(n_seqs=48, n_q_heads=64, n_kv_heads=8, max_len=1500, min_len=1),
                                  "ragged_with_zeros"),
    # few (sequence, KV head) units, each cut into many chunks: one work-group per chunk + merge kernel
    "few_units_group_of_eight": (WL["gqa"].scaled(n_seqs=1, n_q_heads=64, n_kv_heads=8, max_len=20011, min_len=20011), None),
    "few_units_group_of_four_r3t3": (WL["long33"].scaled(n_seqs=2, n_q_heads=32, n_kv_heads=8, max_len=12000, min_len=12000), None),
    "big_ragged_with_empty": (WL["ragged"].scaled(n_seqs=48, n_q_heads=32, n_kv_heads=8, max_len=1500, min_len=1),
                              "ragged_with_zeros"),
    "big_ragged_r3t3": (WL["ragged"].scaled(n_seqs=40, n_q_heads=16, n_kv_heads=8, max_len=2100, min_len=1,
                                            r_bits=3, t_bits=3), "ragged_with_zeros"),
}


def _lengths(wl, spec):
    if isinstance(spec, str) and spec == "ragged_with_zeros":
        lens = W.seq_lengths(wl).copy()
        lens[3] = 0
        lens[wl.n_seqs - 1] = 0
        lens[5] = wl.max_len
        lens[7] = 128
        lens[8] = 129
        lens[9] = 1
        return lens
    return spec


def _check_workload(name, wl, lens, sample_seqs=None, check_scores=True, expect_kernel=None):
    from paper_2502_00527_amd import pq_decode_kernel_name
    from paper_2502_00527_amd.cache import build_device_cache, make_layout

    if expect_kernel is not None:
        max_len = wl.max_len if lens is None else int(max(1, np.max(lens)))
        assert pq_decode_kernel_name(make_layout(wl), wl.n_seqs, wl.n_q_heads, max_len) == expect_kernel

    _say(f"[parity] {name}: S={wl.n_seqs} Hq={wl.n_q_heads} Hkv={wl.n_kv_heads} L<={wl.max_len} "
         f"r{wl.r_bits}t{wl.t_bits} {wl.key_dtype}")
    cache = build_device_cache(wl, lens=lens)
    S, Hq, d, g = wl.n_seqs, wl.n_q_heads, wl.head_dim, wl.group_tokens
    out = torch.full((S, Hq, d), float("nan"), dtype=torch.float32, device="cuda:0")
    scores = None
    if check_scores:
        scores = torch.full((S, Hq, cache.max_seq_len), float("nan"), dtype=torch.float32, device="cuda:0")
    _say(f"[parity] {name}: decode launch")
    cache.decode(out, scores)
    torch.cuda.synchronize()
    out_h = out.cpu().numpy()
    assert np.all(np.isfinite(out_h)), "non-finite attention output"

    q_h = W.queries(wl)
    seqs = range(S) if sample_seqs is None else sample_seqs
    n_codes = n_edge = 0
    worst_score = worst_out = 0.0
    for s in seqs:
        L = int(cache.lens[s])
        if L <= 0:
            assert not out_h[s].any(), "empty sequence must give a zero output row"
            continue
        n_pages = (L + g - 1) // g
        ids = torch.from_numpy(cache.table[s, :n_pages].astype(np.int64)).to("cuda:0")
        ref = OracleSeq(wl, s, L)
        nc, ne = compare_encoding(ref, cache.codes[ids].cpu().numpy(), cache.params[ids].cpu().numpy())
        n_codes += nc
        n_edge += ne
        ref_scores, ref_out, k_hat = ref.attend(q_h[s], cache.sm_scale)
        if check_scores:
            got = scores[s, :, :L].cpu().numpy()
            err = score_errors(got, ref_scores, q_h[s], k_hat)
            worst_score = max(worst_score, float(err.max()))
        worst_out = max(worst_out, float(np.abs(out_h[s] - ref_out).max()))
    _say(f"[parity] {name}: codes={n_codes} edge_mismatches={n_edge} "
         f"max_score_err={worst_score:.3e} max_out_err={worst_out:.3e}")
    assert n_edge <= EDGE_FRACTION * n_codes, "too many angle codes differ on bin edges"
    assert worst_score <= SCORE_REL
    assert worst_out <= OUT_ABS
    return cache


@pytest.mark.parametrize("name", list(SMALL))
def test_small_case(name):
    wl, lens = SMALL[name]
    _check_workload(name, wl, lens)


@pytest.mark.parametrize("name", list(LARGE_GRID))
def test_large_grid_case(name):
    """Small sequences, many of them: the launch shape that selects the role-specialised kernel."""
    wl, spec = LARGE_GRID[name]
    _check_workload(name, wl, _lengths(wl, spec), expect_kernel="pq_decode_roles_kernel")


def test_decode_on_oracle_packed_bytes():
    """Decode alone: the cache bytes come from the oracle's encoder and packer."""
    from paper_2502_00527_amd import Layout, pq_decode_attention, pq_decode_workspace_bytes

    wl = WL["gqa"].scaled(n_seqs=2, n_q_heads=8, n_kv_heads=2, max_len=1300, min_len=1300)
    lens = W.seq_lengths(wl)
    table, total = W.page_table(wl, lens)
    g, H, d = wl.group_tokens, wl.n_kv_heads, wl.head_dim
    codes = np.zeros((total, H, 4, g, 16), np.uint8)
    params = np.zeros((total, H, 64, 2), np.float16)
    values = np.zeros((total, H, g, d), np.float16)
    refs = []
    for s in range(wl.n_seqs):
        L = int(lens[s])
        ref = OracleSeq(wl, s, L)
        n_pages = ref.codes.shape[0]
        ids = table[s, :n_pages]
        codes[ids], params[ids] = ref.codes, ref.params
        v = np.zeros((n_pages * g, H, d), np.float16)
        v[:L] = W.values_for_seq(wl, s, L)
        values[ids] = v.reshape(n_pages, g, H, d).transpose(0, 2, 1, 3)
        refs.append(ref)
    dev = "cuda:0"
    layout = Layout(d, wl.r_bits, wl.t_bits, g, H)
    ws = torch.empty(pq_decode_workspace_bytes(layout, wl.n_seqs, wl.n_q_heads, wl.max_len), dtype=torch.uint8, device=dev)
    out = torch.empty((wl.n_seqs, wl.n_q_heads, d), dtype=torch.float32, device=dev)
    sc = torch.zeros((wl.n_seqs, wl.n_q_heads, wl.max_len), dtype=torch.float32, device=dev)
    q_h = W.queries(wl)
    _say("[parity] decode_on_oracle_packed_bytes: launch")
    pq_decode_attention(layout, torch.from_numpy(q_h).to(dev), torch.from_numpy(codes).to(dev),
                        torch.from_numpy(params).to(dev), torch.from_numpy(values).to(dev),
                        torch.from_numpy(table).to(dev), torch.from_numpy(lens).to(dev), wl.max_len,
                        1.0 / np.sqrt(d), out, ws, sc)
    torch.cuda.synchronize()
    for s, ref in enumerate(refs):
        ref_scores, ref_out, k_hat = ref.attend(q_h[s], 1.0 / np.sqrt(d))
        err = score_errors(sc[s, :, : ref.length].cpu().numpy(), ref_scores, q_h[s], k_hat)
        assert err.max() <= SCORE_REL
        assert np.abs(out[s].cpu().numpy() - ref_out).max() <= OUT_ABS


def test_results_are_deterministic():
    """Two runs of encode + decode give identical bytes."""
    from paper_2502_00527_amd.cache import build_device_cache

    wl = WL["gqa"].scaled(n_seqs=2, n_q_heads=8, n_kv_heads=2, max_len=2100, min_len=2100)
    a = build_device_cache(wl)
    b = build_device_cache(wl)
    assert torch.equal(a.codes, b.codes)
    assert torch.equal(a.params.view(torch.int16), b.params.view(torch.int16))
    oa, ob = a.decode(), b.decode()
    torch.cuda.synchronize()
    assert torch.equal(oa, ob)


@pytest.mark.parametrize("name", ["gqa_ragged_tail", "tiny33_fp32", "group_of_two", "ragged_pages", "bits_r5t3",
                                  "group_of_six", "grouped_angles_gqa", "grouped_angles_edge_lengths",
                                  "grouped_angles_r3t3_many_chunks", "grouped_angles_r3t5", "grouped_angles_r4t2",
                                  # launches of hundreds of work-groups, several chunks per sequence: every
                                  # (r, t) of the token-lane kernel, 1 / 2 / 4 heads per pass, fp32 queries
                                  "big_r4t4_g4", "big_r3t3_g4", "big_r5t3_g1", "big_r3t5_g2", "big_r4t2_g1",
                                  "big_r2t4_g2", "big_fp32_r3t3_g2", "big_group_of_seven_r4t2", "big_ragged_r3t3",
                                  "few_units_group_of_four_r3t3"])
def test_score_keys_entry_point(name):
    """pq_score_keys (the query-key product alone) against the oracle's dequantize-then-dot scores,
    and against the scores pq_decode_attention reports for the same cache."""
    from paper_2502_00527_amd import pq_score_keys
    from paper_2502_00527_amd.cache import build_device_cache

    wl, lens = SMALL[name] if name in SMALL else LARGE_GRID[name]
    lens = _lengths(wl, lens)
    cache = build_device_cache(wl, lens=lens)
    S, Hq = wl.n_seqs, wl.n_q_heads
    got = torch.full((S, Hq, cache.max_seq_len), float("nan"), dtype=torch.float32, device="cuda:0")
    _say(f"[parity] score_keys {name}: launch")
    pq_score_keys(cache.layout, cache.q, cache.codes, cache.params, cache.block_table, cache.seq_lens,
                  cache.max_seq_len, got)
    via_attention = torch.full_like(got, float("nan"))
    cache.decode(scores=via_attention)
    torch.cuda.synchronize()
    q_h = W.queries(wl)
    for s in range(S):
        L = int(cache.lens[s])
        if L <= 0:
            continue
        ref = OracleSeq(wl, s, L)
        ref_scores, _, k_hat = ref.attend(q_h[s], cache.sm_scale)
        err = score_errors(got[s, :, :L].cpu().numpy(), ref_scores, q_h[s], k_hat)
        assert err.max() <= SCORE_REL
        assert torch.equal(got[s, :, :L], via_attention[s, :, :L])
        assert torch.isnan(got[s, :, L:]).all(), "scores past the sequence end must stay untouched"


@pytest.mark.parametrize("case", [("gqa_ragged_tail", 4), ("gqa_ragged_tail", 2), ("tiny_full_config", 4),
                                  ("long33", 2), ("group_of_two", 4), ("edge_lengths", 4), ("ragged_pages", 2),
                                  ("group_of_seven", 4), ("grouped_angles_gqa", 4), ("grouped_angles_r3t3_many_chunks", 2),
                                  ("grouped_angles_edge_lengths", 2), ("bits_r5t3", 4), ("bits_r3t5", 2), ("bits_r4t2", 4),
                                  ("bits_r2t4", 2), ("grouped_angles_r5t3", 2), ("grouped_angles_r2t4", 4),
                                  ("big_r5t3_g1", 4), ("big_r2t4_g2", 2), ("big_r4t4_g4", 4), ("big_r3t5_g2", 4),
                                  ("big_fp32_r3t3_g2", 2), ("big_ragged_r3t3", 4), ("mha_two_seqs", 2)])
def test_quantized_values(case):
    """Token-wise 4/2-bit values: pq_encode_values bit-exact against the oracle's quantizer and
    packer; decode attention over them within the output bar of the oracle's attention over the
    dequantized values."""
    from oracle import cache_format, values as ovalues
    from paper_2502_00527_amd.cache import build_device_cache

    name, v_bits = case
    wl, lens = SMALL[name] if name in SMALL else LARGE_GRID[name]
    lens = _lengths(wl, lens)
    cache = build_device_cache(wl, lens=lens, v_bits=v_bits)
    _say(f"[parity] quantized values {name} v{v_bits}: decode launch")
    out = cache.decode().cpu().numpy()
    torch.cuda.synchronize()
    q_h = W.queries(wl)
    g = wl.group_tokens
    worst = 0.0
    for s in range(wl.n_seqs):
        L = int(cache.lens[s])
        if L <= 0:
            assert not out[s].any()
            continue
        n_pages = (L + g - 1) // g
        ids = torch.from_numpy(cache.table[s, :n_pages].astype(np.int64)).to("cuda:0")
        vals = W.values_for_seq(wl, s, L)
        vc, vs, vz = ovalues.quantize_values(vals, v_bits)
        want_pool = cache_format.pack_value_page_stream(vc, v_bits, g)
        np.testing.assert_array_equal(cache.values[ids].cpu().numpy(), want_pool, err_msg="value codes differ")
        par = np.zeros((n_pages * g, wl.n_kv_heads, 2), np.float16)
        par[:L, :, 0], par[:L, :, 1] = vs, vz
        want_par = par.reshape(n_pages, g, wl.n_kv_heads, 2).transpose(0, 2, 1, 3)
        np.testing.assert_array_equal(cache.v_params[ids].cpu().numpy().view(np.uint16), want_par.view(np.uint16),
                                      err_msg="value scale / zero-point bits differ")
        ref = OracleSeq(wl, s, L)
        _, _, k_hat = ref.attend(q_h[s], cache.sm_scale)
        from oracle import attention as oattention
        _, ref_out = oattention.attend(q_h[s].astype(np.float64), k_hat, ovalues.dequant_values(vc, vs, vz), cache.sm_scale)
        worst = max(worst, float(np.abs(out[s] - ref_out).max()))
    _say(f"[parity] quantized values {name} v{v_bits}: max_out_err={worst:.3e}")
    assert worst <= OUT_ABS


def test_block_table_entry_outside_pool_is_masked():
    """A page id outside the pool makes that page count as masked: nothing is read for it and the
    result is attention over the remaining tokens."""
    from oracle import attention
    from paper_2502_00527_amd.cache import build_device_cache

    wl = WL["gqa"].scaled(n_seqs=2, n_q_heads=8, n_kv_heads=2, max_len=1100, min_len=1100)
    cache = build_device_cache(wl)
    bad_seq, bad_page = 1, 3
    bt = cache.block_table.clone()
    bt[bad_seq, bad_page] = cache.n_pool_pages + 7
    bt[0, 0] = -5
    cache.block_table = bt
    _say("[parity] masked_page: decode launch")
    out = cache.decode().cpu().numpy()
    torch.cuda.synchronize()
    q_h = W.queries(wl)
    g = wl.group_tokens
    for s, page in ((0, 0), (bad_seq, bad_page)):
        ref = OracleSeq(wl, s, 1100)
        _, _, k_hat = ref.attend(q_h[s], cache.sm_scale)
        keep = np.ones(1100, bool)
        keep[page * g:(page + 1) * g] = False
        v = W.values_for_seq(wl, s, 1100).astype(np.float64)
        _, want = attention.attend(q_h[s].astype(np.float64), k_hat[keep], v[keep], cache.sm_scale)
        assert np.abs(out[s] - want).max() <= OUT_ABS


@pytest.mark.parametrize("n_q_heads", [32, 64])
def test_masked_pages_in_a_large_grid(n_q_heads):
    """Block-table entries outside the pool (too large, negative) in a launch served by the
    role-specialised kernel: those pages count as masked, for either wavefront pair of a
    work-group and for first, middle and last pages of a chunk."""
    from oracle import attention
    from paper_2502_00527_amd import pq_decode_kernel_name
    from paper_2502_00527_amd.cache import build_device_cache

    wl = WL["gqa"].scaled(n_seqs=32, n_q_heads=n_q_heads, n_kv_heads=8, max_len=1100, min_len=1100)
    cache = build_device_cache(wl)
    assert pq_decode_kernel_name(cache.layout, wl.n_seqs, wl.n_q_heads, cache.max_seq_len) == "pq_decode_roles_kernel"
    # sequence 20 loses the whole of its first chunk (8 pages), sequence 21 every page
    masked = {0: [0], 1: [3], 2: [1, 2], 5: [8], 9: [4, 7], 17: [0, 1, 2, 3], 20: list(range(8)),
              21: list(range(9)), 31: [5]}
    bt = cache.block_table.clone()
    for k, (s, pages) in enumerate(masked.items()):
        for p in pages:
            bt[s, p] = (cache.n_pool_pages + 7 + p) if (k + p) % 2 == 0 else -1 - p
    cache.block_table = bt
    _say("[parity] masked_pages_large_grid: decode launch")
    out = cache.decode().cpu().numpy()
    torch.cuda.synchronize()
    q_h = W.queries(wl)
    g = wl.group_tokens
    worst = 0.0
    assert not out[21].any(), "a sequence whose pages are all masked must give a zero output row"
    for s in sorted((set(masked) - {21}) | {3, 30}):
        ref = OracleSeq(wl, s, 1100)
        _, _, k_hat = ref.attend(q_h[s], cache.sm_scale)
        keep = np.ones(1100, bool)
        for p in masked.get(s, []):
            keep[p * g:(p + 1) * g] = False
        v = W.values_for_seq(wl, s, 1100).astype(np.float64)
        _, want = attention.attend(q_h[s].astype(np.float64), k_hat[keep], v[keep], cache.sm_scale)
        worst = max(worst, float(np.abs(out[s] - want).max()))
    _say(f"[parity] masked_pages_large_grid: max_out_err={worst:.3e}")
    assert worst <= OUT_ABS


# ---- full-size launch configurations (what the benchmark times), sampled sequences ----

FULL = {
    "gqa": [0, 11],          # the headline configuration
    "mha": [5],
    "long33": [0],
    "ragged": [0, 37],
    "gqa_grouped_angles": [6],
}


@pytest.mark.parametrize("name", list(FULL))
def test_full_size_sampled(name):
    wl = WL["gqa"].scaled(grouped_angles=True) if name == "gqa_grouped_angles" else WL[name]
    _check_workload(name + "_full", wl, None, sample_seqs=FULL[name])


# ---- sizes near the ends of the supported range ----

def test_one_million_token_sequence():
    """A single 1 Mi-token sequence (8193 pages, 257 chunks): index arithmetic at the long end."""
    wl = WL["gqa"].scaled(n_seqs=1, n_q_heads=4, n_kv_heads=1, max_len=(1 << 20) + 77, min_len=(1 << 20) + 77)
    _check_workload("one_million_tokens", wl, None)


def test_many_short_sequences():
    """1500 sequences of 1..300 tokens (grid of 1500 x 1 chunk, most work-groups nearly empty)."""
    wl = WL["ragged"].scaled(n_seqs=1500, n_q_heads=2, n_kv_heads=1, max_len=300, min_len=1)
    _check_workload("many_short_sequences", wl, None, sample_seqs=list(range(0, 1500, 7)))


# ---- streams and graphs: the library keeps no state and allocates nothing ----

def test_decode_under_hip_graph_replay():
    """pq_decode_attention captured into a HIP graph and replayed, with eager work and
    synchronisations between the replays, reproduces the eager result bit for bit; new inputs
    written into the captured buffers are picked up by the next replay."""
    from paper_2502_00527_amd.cache import build_device_cache

    wl = WL["gqa"].scaled(n_seqs=3, n_q_heads=8, n_kv_heads=2, max_len=2500, min_len=900)
    cache = build_device_cache(wl)
    eager = cache.decode().clone()
    torch.cuda.synchronize()
    out = torch.zeros_like(eager)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        cache.decode(out)                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    _say("[graph] capture")
    with torch.cuda.graph(graph, stream=side):
        cache.decode(out)
    q0 = cache.q.clone()
    for rep in range(4):
        out.fill_(float("nan"))
        _say(f"[graph] replay {rep}")
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager), f"replay {rep} differs from the eager result"
        # eager work between replays, on other buffers
        other = cache.decode()
        torch.cuda.synchronize()
        assert torch.equal(other, eager)
    # a new query in the captured input buffer
    cache.q.copy_(torch.flip(q0, dims=[0]))
    want = cache.decode().clone()
    torch.cuda.synchronize()
    out.fill_(float("nan"))
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, want) and not torch.equal(want, eager)
    cache.q.copy_(q0)


def test_two_streams_with_their_own_workspaces():
    """Two decode calls in flight on two streams (separate workspaces and outputs) give what
    each gives alone."""
    from paper_2502_00527_amd.cache import build_device_cache

    wl_a = WL["gqa"].scaled(n_seqs=4, n_q_heads=8, n_kv_heads=2, max_len=6000, min_len=3000)
    wl_b = WL["mha"].scaled(n_seqs=3, n_q_heads=4, n_kv_heads=4, max_len=5000, min_len=5000)
    a, b = build_device_cache(wl_a), build_device_cache(wl_b)
    ref_a, ref_b = a.decode().clone(), b.decode().clone()
    torch.cuda.synchronize()
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    out_a, out_b = torch.zeros_like(ref_a), torch.zeros_like(ref_b)
    for rep in range(5):
        with torch.cuda.stream(sa):
            a.decode(out_a)
        with torch.cuda.stream(sb):
            b.decode(out_b)
        torch.cuda.synchronize()
        assert torch.equal(out_a, ref_a) and torch.equal(out_b, ref_b)


def test_random_shapes():
    """Seeded sweep over shapes the fixed cases do not name: random batch sizes, query-group
    sizes, bit allocations, angle quantizers and ragged lengths (lengths of 0 included)."""
    rng = np.random.default_rng(20250299)
    bit_choices = [(4, 4), (3, 3), (5, 3), (3, 5), (4, 2), (2, 4)]
    for case in range(20):
        n_kv = int(rng.choice([1, 2, 3, 5]))
        group = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 16]))
        grouped = bool(rng.random() < 0.4)
        r, t = bit_choices[int(rng.integers(6))]
        n_seqs = int(rng.integers(1, 7))
        max_len = int(rng.integers(1, 1400))
        base = WL["ragged"] if rng.random() < 0.5 else WL["mha"]
        wl = base.scaled(n_seqs=n_seqs, n_q_heads=n_kv * group, n_kv_heads=n_kv, max_len=max_len, min_len=1,
                         r_bits=r, t_bits=t, grouped_angles=grouped, index=100 + case,
                         shuffled_pages=bool(rng.random() < 0.5),
                         key_dtype="f32" if rng.random() < 0.3 else "f16")
        lens = rng.integers(0, max_len + 1, n_seqs).astype(np.int32)
        lens[int(rng.integers(n_seqs))] = max_len
        _check_workload(f"random_{case}", wl, lens)


def test_random_shapes_many_units():
    """The same kind of sweep with enough (sequence, KV head) units that the launches cross the
    256-work-group line: fp16 values with the uniform grid then run the role-specialised kernel."""
    from paper_2502_00527_amd import pq_decode_kernel_name
    from paper_2502_00527_amd.cache import make_layout

    rng = np.random.default_rng(20250298)
    bit_choices = [(4, 4), (3, 3), (5, 3), (3, 5), (4, 2), (2, 4)]
    n_roles = 0
    for case in range(10):
        n_kv = int(rng.choice([4, 8, 6]))
        group = int(rng.choice([1, 2, 3, 4, 5, 8]))
        r, t = bit_choices[int(rng.integers(6))]
        n_seqs = int(rng.integers(256 // n_kv, 400 // n_kv))
        max_len = int(rng.integers(300, 900))
        base = WL["ragged"] if rng.random() < 0.5 else WL["mha"]
        wl = base.scaled(n_seqs=n_seqs, n_q_heads=n_kv * group, n_kv_heads=n_kv, max_len=max_len, min_len=1,
                         r_bits=r, t_bits=t, index=200 + case, shuffled_pages=bool(rng.random() < 0.5),
                         key_dtype="f32" if rng.random() < 0.3 else "f16")
        lens = rng.integers(0, max_len + 1, n_seqs).astype(np.int32)
        lens[int(rng.integers(n_seqs))] = max_len
        n_roles += pq_decode_kernel_name(make_layout(wl), n_seqs, wl.n_q_heads, max_len) == "pq_decode_roles_kernel"
        _check_workload(f"random_many_{case}", wl, lens, sample_seqs=list(range(0, n_seqs, 3)))
    assert n_roles >= 8
