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
    import paper_2502_00527_amd as pq
    from paper_2502_00527_amd.cache import make_layout

    r, t, grouped = bits
    wl = W.WORKLOADS["gqa"].scaled(n_seqs=3, n_q_heads=8, n_kv_heads=2, max_len=1024, min_len=1024,
                                   r_bits=r, t_bits=t, shuffled_pages=True, grouped_angles=grouped)
    layout = make_layout(wl)
    g, H, d, S = wl.group_tokens, wl.n_kv_heads, wl.head_dim, wl.n_seqs
    start = np.array([300, 128, 5], np.int32)
    steps = 260
    final = start + steps
    table, total = W.page_table(wl, final)
    dev = "cuda:0"
    keys_all = [W.keys_for_seq(wl, s, int(final[s])) for s in range(S)]          # fp16 [L, H, d]
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
        for s in range(S):
            L = int(cur[s])
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
        _say(f"[generation r{r}t{t}{' grouped angles' if grouped else ''}] step {step_no}: lens {cur.tolist()} score err {worst_s:.2e} out err {worst_o:.2e}")
        assert worst_s <= SCORE_REL and worst_o <= OUT_ABS

    check(0)
    for i in range(steps):
        new = np.stack([keys_all[s][int(start[s]) + i] for s in range(S)])           # [S, H, d]
        pq.pq_append_keys(layout, torch.from_numpy(new).to(dev), residual, lens, bt, codes, params)
        lens += 1
        if i + 1 in (1, 84, 123, 124, 200, 260):
            check(i + 1)

    # every group completed on the way is encoded bit-exactly as the oracle encodes it
    for s in range(S):
        n_full = int(final[s]) // g
        enc = polar.encode_keys(keys_all[s][: n_full * g], r, t, g, grouped_angles=grouped)
        want_codes, want_params = cache_format.pack_sequence(enc["a"], enc["c"], enc["scale"], enc["zero"], r, t, g,
                                                             enc.get("t_scale"), enc.get("t_zero"))
        ids = torch.from_numpy(table[s, :n_full].astype(np.int64)).to(dev)
        np.testing.assert_array_equal(codes[ids].cpu().numpy(), want_codes)
        np.testing.assert_array_equal(params[ids].cpu().numpy().view(np.uint16), want_params.view(np.uint16))
