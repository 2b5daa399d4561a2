"""Multi-step generation through the C ABI: pq_append_keys keeps new keys in the fp16 residual
buffer and encodes a group when it fills; pq_decode_attention scores packed groups through the
lookup table and the residual group by plain dot products.  Checked against the oracle at several
points of a 260-step run that crosses page boundaries."""
import sys

import numpy as np
import pytest
import torch

from oracle import attention, cache_format, polar
from paper_2502_00527_amd import workloads as W

from parity import OUT_ABS, SCORE_REL, score_errors

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.mark.parametrize("bits", [(4, 4, False), (3, 3, False), (4, 4, True), (3, 3, True)])
def test_append_then_decode_with_residual(bits):
    r, t, grouped = bits
    wl = W.WORKLOADS["gqa"].scaled(n_seqs=3, n_q_heads=8, n_kv_heads=2, max_len=1024, min_len=1024,
                                   r_bits=r, t_bits=t, shuffled_pages=True, grouped_angles=grouped)
    _generate(wl, np.array([300, 128, 5], np.int32), 260, (1, 84, 123, 124, 200, 260))


@pytest.mark.parametrize("bits", [(4, 4, 4, "f16"), (3, 3, 2, "f16"), (5, 3, 1, "f16"), (2, 4, 4, "f32"),
                                  (3, 5, 6, "f16"), (4, 2, 2, "f32"), (4, 4, 8, "f16"), (3, 3, 8, "f32")])
def test_append_then_decode_large_batch(bits):
    """The same run with 256 (sequence, KV head) units, which the role-specialised attention kernel
    serves: residual groups of every fill level at once (the start lengths differ by 5 tokens from
    sequence to sequence), on first, middle and last pages of a chunk and on either wavefront pair."""
    from paper_2502_00527_amd import pq_decode_kernel_name
    from paper_2502_00527_amd.cache import make_layout

    r, t, group, dt = bits
    S, H = 64, 4
    wl = W.WORKLOADS["gqa"].scaled(n_seqs=S, n_q_heads=H * group, n_kv_heads=H, max_len=1024, min_len=1024,
                                   r_bits=r, t_bits=t, shuffled_pages=True, key_dtype=dt)
    start = (300 + 5 * np.arange(S)).astype(np.int32)          # 300 .. 615: residual groups on pages 2 .. 5
    start[10], start[11], start[12], start[20], start[21] = 128, 256, 127, 3, 0
    steps = 131
    assert pq_decode_kernel_name(make_layout(wl), S, wl.n_q_heads, int(start.max()) + steps) == "pq_decode_roles_kernel"
    _generate(wl, start, steps, (1, 64, 131), sample=list(range(0, S, 3)) + [10, 11, 12])


def _generate(wl, start, steps, check_at, sample=None):
    import paper_2502_00527_amd as pq
    from paper_2502_00527_amd.cache import make_layout

    r, t, grouped = wl.r_bits, wl.t_bits, wl.grouped_angles
    layout = make_layout(wl)
    g, H, d, S = wl.group_tokens, wl.n_kv_heads, wl.head_dim, wl.n_seqs
    sample = list(range(S)) if sample is None else sorted(set(sample))
    final = start + steps
    table, total = W.page_table(wl, final)
    dev = "cuda:0"
    # keys are fp16 values (the residual buffer keeps fp16 rows); with an fp32 workload they are
    # handed over as fp32 numbers that fp16 represents exactly, the queries stay genuine fp32
    keys_all = [W.keys_for_seq(wl, s, int(final[s])).astype(np.float16).astype(wl.np_key_dtype) for s in range(S)]
    vals_all = [W.values_for_seq(wl, s, int(final[s])) for s in range(S)]
    q_h = W.queries(wl)
    ub = 2 * (r + t)
    codes = torch.full((total, H, d // 32, g, ub), 0x5A, dtype=torch.uint8, device=dev)
    params = torch.full((total, H, 2, d // 2, 2) if grouped else (total, H, d // 2, 2), float("nan"),
                        dtype=torch.float16, device=dev)
    values = torch.zeros((total, H, g, d), dtype=torch.float16, device=dev)
    residual = torch.full((S, H, g, d), float("nan"), dtype=torch.float16, device=dev)
    bt = torch.from_numpy(np.maximum(table, 0)).to(dev)
    for s in range(S):
        L0 = int(start[s])
        n_full = L0 // g
        if n_full:
            ids = torch.from_numpy(table[s, :n_full].copy()).to(dev)
            pq.pq_encode_keys(layout, torch.from_numpy(keys_all[s][: n_full * g]).to(dev), ids, codes, params)
        if L0 % g:
            residual[s, :, : L0 - n_full * g] = torch.from_numpy(keys_all[s][n_full * g: L0]).to(dev).permute(1, 0, 2)
        n_pages = (int(final[s]) + g - 1) // g
        v = np.zeros((n_pages * g, H, d), np.float16)
        v[: final[s]] = vals_all[s]
        values[torch.from_numpy(table[s, :n_pages].astype(np.int64)).to(dev)] = \
            torch.from_numpy(v.reshape(n_pages, g, H, d).transpose(0, 2, 1, 3).copy()).to(dev)
    lens = torch.from_numpy(start.copy()).to(dev)
    q = torch.from_numpy(q_h).to(dev)
    max_len = int(final.max())
    ws = torch.empty(pq.pq_decode_workspace_bytes(layout, S, wl.n_q_heads, max_len), dtype=torch.uint8, device=dev)
    out = torch.empty((S, wl.n_q_heads, d), dtype=torch.float32, device=dev)
    scores = torch.zeros((S, wl.n_q_heads, max_len), dtype=torch.float32, device=dev)
    sm_scale = 1.0 / np.sqrt(d)

    def check(step_no):
        cur = lens.cpu().numpy()
        pq.pq_decode_attention(layout, q, codes, params, values, bt, lens, max_len, sm_scale, out, ws, scores, residual)
        qk = torch.full_like(scores, float("nan"))
        pq.pq_score_keys(layout, q, codes, params, bt, lens, max_len, qk, residual)     # the product alone, same keys
        torch.cuda.synchronize()
        for s in range(S):
            assert torch.equal(qk[s, :, : int(cur[s])], scores[s, :, : int(cur[s])])
            assert torch.isnan(qk[s, :, int(cur[s]):]).all()
        worst_s = worst_o = 0.0
        for s in sample:
            L = int(cur[s])
            if L == 0:
                assert not out[s].cpu().numpy().any(), "empty sequence must give a zero output row"
                continue
            n_full = L // g
            parts = []
            if n_full:
                enc = polar.encode_keys(keys_all[s][: n_full * g], r, t, g, grouped_angles=grouped)
                parts.append(polar.dequant_keys(enc["a"], enc["c"], enc["scale"], enc["zero"], t, g,
                                                enc.get("t_scale"), enc.get("t_zero")))
            if L % g:
                parts.append(keys_all[s][n_full * g: L].astype(np.float64))
            k_ref = np.concatenate(parts)
            ref_scores, ref_out = attention.attend(q_h[s].astype(np.float64), k_ref, vals_all[s][:L].astype(np.float64), sm_scale)
            err = score_errors(scores[s, :, :L].cpu().numpy(), ref_scores, q_h[s], k_ref)
            worst_s = max(worst_s, float(err.max()))
            worst_o = max(worst_o, float(np.abs(out[s].cpu().numpy() - ref_out).max()))
        _say(f"[generation r{r}t{t}{' grouped angles' if grouped else ''}] step {step_no}: lens {cur.tolist()[:8]}{'...' if S > 8 else ''} score err {worst_s:.2e} out err {worst_o:.2e}")
        assert worst_s <= SCORE_REL and worst_o <= OUT_ABS

    check(0)
    for i in range(steps):
        new = np.stack([keys_all[s][int(start[s]) + i] for s in range(S)])           # [S, H, d]
        pq.pq_append_keys(layout, torch.from_numpy(new).to(dev), residual, lens, bt, codes, params)
        lens += 1
        if i + 1 in check_at:
            check(i + 1)

    # every group completed on the way is encoded bit-exactly as the oracle encodes it
    for s in sample:
        n_full = int(final[s]) // g
        if n_full == 0:
            continue
        enc = polar.encode_keys(keys_all[s][: n_full * g], r, t, g, grouped_angles=grouped)
        want_codes, want_params = cache_format.pack_sequence(enc["a"], enc["c"], enc["scale"], enc["zero"], r, t, g,
                                                             enc.get("t_scale"), enc.get("t_zero"))
        ids = torch.from_numpy(table[s, :n_full].astype(np.int64)).to(dev)
        np.testing.assert_array_equal(codes[ids].cpu().numpy(), want_codes)
        np.testing.assert_array_equal(params[ids].cpu().numpy().view(np.uint16), want_params.view(np.uint16))
