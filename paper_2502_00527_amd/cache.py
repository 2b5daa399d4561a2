"""Device-side pools of a paged polar-quantized cache: allocation and filling.

Plumbing around the C ABI for tests, the smoke check and the benchmark: torch
allocates the pools, `pq_encode_keys` (HIP) packs the keys, and value rows are
copied into their pages.  No arithmetic of the method happens here.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np
import torch

from . import (Layout, pq_codes_bytes_per_page, pq_decode_attention, pq_decode_workspace_bytes,
               pq_encode_keys, pq_encode_values, pq_params_bytes_per_page, pq_vq_bytes_per_page)
from . import workloads as W


@dataclasses.dataclass
class DeviceCache:
    layout: Layout
    wl: W.Workload
    lens: np.ndarray                 # host int32 [S]
    table: np.ndarray                # host int32 [S, width]
    n_pool_pages: int
    codes: torch.Tensor              # uint8 [pages, H, P/16, g, 2w]
    params: torch.Tensor             # fp16  [pages, H, P, 2], or [pages, H, 2, P, 2] with grouped angles
    values: torch.Tensor             # fp16  [pages, H, g, d], or uint8 [pages, H, g/T, d/8, 16] when quantized
    v_bits: int                      # 16, 4 or 2
    v_params: Optional[torch.Tensor] # fp16 [pages, H, g, 2] (scale, zero) when quantized
    block_table: torch.Tensor        # int32 [S, width] (device; -1 replaced by 0)
    seq_lens: torch.Tensor           # int32 [S]
    q: torch.Tensor                  # [S, Hq, d]
    workspace: torch.Tensor
    max_seq_len: int

    @property
    def sm_scale(self) -> float:
        return 1.0 / float(np.sqrt(self.wl.head_dim))

    def decode(self, out: Optional[torch.Tensor] = None, scores: Optional[torch.Tensor] = None,
               residual: Optional[torch.Tensor] = None):
        if out is None:
            out = torch.empty((self.wl.n_seqs, self.wl.n_q_heads, self.wl.head_dim), dtype=torch.float32,
                              device=self.q.device)
        pq_decode_attention(self.layout, self.q, self.codes, self.params, self.values, self.block_table,
                            self.seq_lens, self.max_seq_len, self.sm_scale, out, self.workspace, scores, residual,
                            self.v_bits, self.v_params)
        return out


def make_layout(wl: W.Workload) -> Layout:
    return Layout(wl.head_dim, wl.r_bits, wl.t_bits, wl.group_tokens, wl.n_kv_heads, 1 if wl.grouped_angles else 0)


def build_device_cache(wl: W.Workload, device="cuda:0", lens: Optional[np.ndarray] = None,
                       progress=None, v_bits: int = 16) -> DeviceCache:
    """Generates the workload's inputs on the host (seeded), uploads them, encodes the keys
    with pq_encode_keys and files the value rows into their pages (fp16, or quantized by
    pq_encode_values when v_bits is 4 or 2)."""
    layout = make_layout(wl)
    if lens is None:
        lens = W.seq_lengths(wl)
    lens = np.asarray(lens, np.int32)
    table, total = W.page_table(wl, np.maximum(lens, 1))
    g, H, d = wl.group_tokens, wl.n_kv_heads, wl.head_dim
    ub = 2 * (wl.r_bits + wl.t_bits)
    assert pq_codes_bytes_per_page(layout) == H * (d // 32) * g * ub
    par_shape = (total, H, 2, d // 2, 2) if wl.grouped_angles else (total, H, d // 2, 2)
    assert pq_params_bytes_per_page(layout) == int(np.prod(par_shape[1:])) * 2
    # poison the pools so that a slot the encoder should have written shows up
    codes = torch.full((total, H, d // 32, g, ub), 0xA5, dtype=torch.uint8, device=device)
    params = torch.full(par_shape, float("nan"), dtype=torch.float16, device=device)
    v_params = None
    if v_bits == 16:
        values = torch.full((total, H, g, d), float("nan"), dtype=torch.float16, device=device)
    else:
        t_per_unit = 16 // v_bits
        assert pq_vq_bytes_per_page(layout, v_bits) == H * g * d * v_bits // 8
        values = torch.full((total, H, g // t_per_unit, d // 8, 16), 0xC3, dtype=torch.uint8, device=device)
        v_params = torch.full((total, H, g, 2), float("nan"), dtype=torch.float16, device=device)
    for s in range(wl.n_seqs):
        L = int(lens[s])
        if L <= 0:
            continue
        n_pages = (L + g - 1) // g
        ids = torch.from_numpy(table[s, :n_pages].copy()).to(device)
        keys = torch.from_numpy(W.keys_for_seq(wl, s, L)).to(device)
        pq_encode_keys(layout, keys, ids, codes, params)
        vals = torch.from_numpy(W.values_for_seq(wl, s, L)).to(device)
        if v_bits == 16:
            full = n_pages * g
            if full != L:
                vals = torch.cat([vals, torch.full((full - L, H, d), float("nan"), dtype=torch.float16,
                                                   device=device)])
            values[ids.long()] = vals.view(n_pages, g, H, d).permute(0, 2, 1, 3)
        else:
            pq_encode_values(layout, v_bits, vals, ids, values, v_params)
        del keys, vals
        if progress:
            progress(s)
    max_len = int(max(1, lens.max()))
    ws_bytes = pq_decode_workspace_bytes(layout, wl.n_seqs, wl.n_q_heads, max_len)
    assert ws_bytes > 0
    bt = torch.from_numpy(np.maximum(table, 0)).to(device)
    return DeviceCache(
        layout=layout, wl=wl, lens=lens, table=table, n_pool_pages=total, codes=codes, params=params,
        values=values, v_bits=v_bits, v_params=v_params, block_table=bt, seq_lens=torch.from_numpy(lens).to(device),
        q=torch.from_numpy(W.queries(wl)).to(device),
        workspace=torch.empty(ws_bytes, dtype=torch.uint8, device=device), max_seq_len=max_len)
