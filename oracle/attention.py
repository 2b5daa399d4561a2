"""Decode attention over a polar-quantized, paged key cache (oracle; test infrastructure only).

The method's lookup-table product is an exact re-ordering of "dequantize the
key, then take the inner product with the query" (Section 3.3; Appendix A), so
the oracle is that plain definition: unpack the stored bytes, reconstruct each
key with the mid-point dequantizer of Section 3.2, and take direct float64 dot
products.  Softmax and the fp16-value aggregation around it are standard
attention (Section 2); values stay fp16 as in the paper's experiments (Section
4.1, "General setup").

Query head h reads KV head h // (n_q_heads / n_kv_heads) (grouped-query
attention, Section 5.2).  `scores` are the raw q . k~ (no softmax scale).
"""
from __future__ import annotations

import numpy as np

from . import cache_format, polar, values


def dequant_sequence(codes_pool, params_pool, page_ids, length, r_bits, t_bits, group_tokens,
                     residual_seq=None):
    """Keys float64 [length, H, d] of one sequence as the decode step sees them.

    codes_pool uint8 [n_pool_pages, H, P/16, g, 2w]; params_pool fp16 [n_pool_pages, H, P, 2], or
    [n_pool_pages, H, 2, P, 2] when the angles were quantized group-wise (radius, then angle
    parameters: the angle levels are then the group's own);
    page_ids: the sequence's pages in order.  Without a residual buffer every token is
    reconstructed from the packed pages.  With one (fp16 [H, g, d]; Appendix B.1: recent keys
    stay un-quantized until a full group exists) only the complete groups are, and the keys of
    the last, incomplete group are the residual rows themselves.
    """
    g = group_tokens
    if residual_seq is None:
        n_pages = (length + g - 1) // g
        ids = np.asarray(page_ids[:n_pages], np.int64)
        a, c, *par = cache_format.unpack_pages(codes_pool[ids], params_pool[ids], length, r_bits, t_bits)
        return polar.dequant_keys(a, c, par[0], par[1], t_bits, g, *par[2:])
    n_full = length // g
    rest = length - n_full * g
    parts = []
    if n_full:
        ids = np.asarray(page_ids[:n_full], np.int64)
        a, c, *par = cache_format.unpack_pages(codes_pool[ids], params_pool[ids], n_full * g, r_bits, t_bits)
        parts.append(polar.dequant_keys(a, c, par[0], par[1], t_bits, g, *par[2:]))
    if rest:
        parts.append(np.asarray(residual_seq)[:, :rest, :].transpose(1, 0, 2).astype(np.float64))
    return np.concatenate(parts, axis=0)


def gather_values(v_pool, page_ids, length, group_tokens):
    """Values float64 [length, H, d] of one sequence; v_pool fp16 [n_pool_pages, H, g, d]."""
    n_pages = (length + group_tokens - 1) // group_tokens
    ids = np.asarray(page_ids[:n_pages], np.int64)
    v = v_pool[ids].transpose(0, 2, 1, 3)                                  # [n_pages, g, H, d]
    return v.reshape(n_pages * group_tokens, v.shape[2], v.shape[3])[:length].astype(np.float64)


def gather_quantized_values(vq_pool, vq_params, page_ids, length, group_tokens, bits):
    """Dequantized values float64 [length, H, d] of one sequence.

    vq_pool uint8 [n_pool_pages, H, g/T, d/8, 16]; vq_params fp16 [n_pool_pages, H, g, 2] = (scale, zero).
    """
    g = group_tokens
    n_pages = (length + g - 1) // g
    ids = np.asarray(page_ids[:n_pages], np.int64)
    codes = cache_format.unpack_value_pages(vq_pool[ids], length, bits)               # [L, H, d]
    par = vq_params[ids].transpose(0, 2, 1, 3).reshape(n_pages * g, vq_params.shape[1], 2)[:length]
    return values.dequant_values(codes, par[..., 0], par[..., 1])


def attend(q, k_hat, v, sm_scale):
    """q float64 [Hq, d]; k_hat, v float64 [L, Hkv, d] -> (scores [Hq, L], out [Hq, d])."""
    n_q, n_kv = q.shape[0], k_hat.shape[1]
    assert n_q % n_kv == 0
    rep = n_q // n_kv
    scores = np.empty((n_q, k_hat.shape[0]), np.float64)
    out = np.empty((n_q, v.shape[2]), np.float64)
    for h in range(n_q):
        kh = h // rep
        s = k_hat[:, kh, :] @ q[h]
        scores[h] = s
        e = np.exp(sm_scale * s - np.max(sm_scale * s))
        out[h] = (e / e.sum()) @ v[:, kh, :]
    return scores, out


def decode_attention(q, codes_pool, params_pool, v_pool, block_table, seq_lens,
                     r_bits, t_bits, group_tokens, sm_scale, seqs=None, residual=None,
                     vq_params=None, v_bits=16):
    """One decode step per sequence.

    q [S, Hq, d] (any float dtype); pools as in dequant_sequence / gather_values;
    block_table int [S, max_pages]; seq_lens int [S]; residual optional fp16 [S, H, g, d].
    With v_bits 4 or 2, v_pool holds quantized value pages and vq_params their (scale, zero).
    `seqs` restricts the work to some sequences.
    Returns {seq: (scores float64 [Hq, L_seq], out float64 [Hq, d])}.
    """
    res = {}
    for s in (range(q.shape[0]) if seqs is None else seqs):
        L = int(seq_lens[s])
        k_hat = dequant_sequence(codes_pool, params_pool, block_table[s], L, r_bits, t_bits, group_tokens,
                                 None if residual is None else residual[s])
        if v_bits == 16:
            v = gather_values(v_pool, block_table[s], L, group_tokens)
        else:
            v = gather_quantized_values(v_pool, vq_params, block_table[s], L, group_tokens, v_bits)
        res[s] = attend(q[s].astype(np.float64), k_hat, v, sm_scale)
    return res
