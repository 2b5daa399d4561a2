"""pq_decode_attention_static (the entry point that allocates nothing: its chunk partials live in a
static device array inside the library) against pq_decode_attention with a caller's workspace,
through the C ABI: two calls in a row, the second with a smaller input, then the size limit."""
import ctypes
import sys

import numpy as np
import pytest
import torch

import paper_2502_00527_amd as pq
from paper_2502_00527_amd import workloads as W

from parity import OUT_ABS, OracleSeq

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _raw_static_call(lib, cache, out, scores=None):
    """The C entry point itself, with plain pointers and sizes."""
    null = ctypes.c_void_p(0)
    wl = cache.wl
    st = lib.pq_decode_attention_static(
        ctypes.byref(cache.layout), cache.q.data_ptr(), pq.PQ_F16 if cache.q.dtype == torch.float16 else pq.PQ_F32,
        wl.n_seqs, wl.n_q_heads, cache.codes.data_ptr(), cache.params.data_ptr(), cache.values.data_ptr(), 16, null,
        cache.n_pool_pages, cache.block_table.data_ptr(), cache.block_table.shape[1], cache.seq_lens.data_ptr(),
        cache.max_seq_len, ctypes.c_float(cache.sm_scale), out.data_ptr(),
        null if scores is None else scores.data_ptr(), 0 if scores is None else scores.shape[-1], null,
        ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return st


def test_static_scratch_entry_point_matches_the_workspace_one():
    from paper_2502_00527_amd.cache import build_device_cache

    lib = pq.load_library()
    # first call: several chunks per sequence, ragged; second call: a smaller batch of shorter
    # sequences, which uses a prefix of the same static array while the rest keeps the first
    # call's partials
    big = W.WORKLOADS["ragged"].scaled(n_seqs=24, n_q_heads=16, n_kv_heads=4, max_len=6000, min_len=100)
    small = W.WORKLOADS["gqa"].scaled(n_seqs=3, n_q_heads=8, n_kv_heads=2, max_len=700, min_len=700, r_bits=3, t_bits=3)
    for name, wl in (("first call (24 ragged sequences)", big), ("second call (3 short sequences)", small)):
        cache = build_device_cache(wl)
        assert pq.pq_decode_workspace_bytes(cache.layout, wl.n_seqs, wl.n_q_heads, cache.max_seq_len) <= pq.PQ_STATIC_SCRATCH_BYTES
        want = cache.decode().clone()
        want_scores = torch.full((wl.n_seqs, wl.n_q_heads, cache.max_seq_len), float("nan"), dtype=torch.float32, device="cuda:0")
        cache.decode(scores=want_scores)
        torch.cuda.synchronize()
        got = torch.full_like(want, float("nan"))
        got_scores = torch.full_like(want_scores, float("nan"))
        _say(f"[static scratch] {name}: launch")
        assert _raw_static_call(lib, cache, got, got_scores) == 0
        torch.cuda.synchronize()
        assert torch.equal(got, want), "static-scratch result differs from the workspace result"
        assert torch.equal(got_scores.nan_to_num(nan=-7.0), want_scores.nan_to_num(nan=-7.0))
        # and against the oracle directly, for one sequence
        s = wl.n_seqs - 1
        L = int(cache.lens[s])
        _, ref_out, _ = OracleSeq(wl, s, L).attend(W.queries(wl)[s], cache.sm_scale)
        assert np.abs(got[s].cpu().numpy() - ref_out).max() <= OUT_ABS
        # the binding's wrapper reaches the same entry point
        again = torch.full_like(want, float("nan"))
        pq.pq_decode_attention_static(cache.layout, cache.q, cache.codes, cache.params, cache.values, cache.block_table,
                                      cache.seq_lens, cache.max_seq_len, cache.sm_scale, again)
        torch.cuda.synchronize()
        assert torch.equal(again, want)


def test_static_scratch_rejects_shapes_beyond_its_size():
    """A shape that needs more than PQ_STATIC_SCRATCH_BYTES is refused on the host, before any launch."""
    lib = pq.load_library()
    lay = pq.Layout(128, 4, 4, 128, 8)
    assert pq.pq_decode_workspace_bytes(lay, 512, 32, 16384) > pq.PQ_STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(4096)
    null = ctypes.c_void_p(0)
    st = lib.pq_decode_attention_static(ctypes.byref(lay), fake, 0, 512, 32, fake, fake, fake, 16, null, 4, fake, 128, fake,
                                        16384, ctypes.c_float(0.1), fake, null, 0, null, null)
    assert st == -5 and "static" in pq.pq_strerror(st)
