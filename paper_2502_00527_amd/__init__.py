"""Python binding of libpolarquant (include/polarquant.h): argument marshalling only.

Every step of the path -- encoding keys into the polar-quantized cache (paper
Section 3.2) and decode attention through the per-query lookup table (Section
3.3, Appendix A) -- runs in the HIP kernels behind the C ABI.  This module
turns torch tensors into device pointers and sizes, passes torch's current HIP
stream, and raises on any non-zero status.  There is no fallback: if the
shared library has not been built (`python -m paper_2502_00527_amd.build`),
the first call raises.

The functions carry the names of the C entry points.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_float, c_int, c_int32, c_int64, c_size_t, c_void_p
from typing import Optional

__all__ = [
    "Layout", "PQ_F16", "PQ_F32", "PolarQuantError", "lib_path", "load_library",
    "pq_version", "pq_strerror", "pq_codes_bytes_per_page", "pq_params_bytes_per_page",
    "pq_values_bytes_per_page", "pq_decode_workspace_bytes", "pq_encode_keys",
    "pq_decode_attention", "pq_decode_partials", "pq_decode_merge", "pq_score_keys", "pq_append_keys",
    "pq_vq_bytes_per_page", "pq_vq_params_bytes_per_page", "pq_encode_values",
    "pq_probe_read_stream", "pq_decode_kernel_name", "pq_decode_merges_in_kernel",
    "pq_decode_attention_static", "PQ_STATIC_SCRATCH_BYTES",
]

PQ_F16, PQ_F32 = 0, 1
PQ_STATIC_SCRATCH_BYTES = 8 << 20
_LIB_NAME = "libpolarquant.so"
_lib = None


class PolarQuantError(RuntimeError):
    pass


class Layout(ctypes.Structure):
    """pq_layout: head_dim, r_bits, t_bits, group_tokens, n_kv_heads, angle_quantizer
    (0 = uniform grid, 1 = the paper's grouped min/scale quantizer)."""

    _fields_ = [("head_dim", c_int32), ("r_bits", c_int32), ("t_bits", c_int32),
                ("group_tokens", c_int32), ("n_kv_heads", c_int32), ("angle_quantizer", c_int32)]


def lib_path() -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), _LIB_NAME)


# name -> (restype, argtypes); mirrors include/polarquant.h
_LP = ctypes.POINTER(Layout)
_SIGNATURES = {
    "pq_version": (c_int, []),
    "pq_strerror": (ctypes.c_char_p, [c_int]),
    "pq_last_hip_error": (c_int, []),
    "pq_codes_bytes_per_page": (c_size_t, [_LP]),
    "pq_params_bytes_per_page": (c_size_t, [_LP]),
    "pq_values_bytes_per_page": (c_size_t, [_LP]),
    "pq_decode_workspace_bytes": (c_size_t, [_LP, c_int32, c_int32, c_int32]),
    "pq_encode_keys": (c_int, [_LP, c_void_p, c_int, c_int64, c_int64, c_int64, c_void_p, c_void_p,
                               c_void_p, c_int64, c_void_p]),
    "pq_decode_attention": (c_int, [_LP, c_void_p, c_int, c_int32, c_int32, c_void_p, c_void_p, c_void_p,
                                    c_int32, c_void_p, c_int64, c_void_p, c_int32, c_void_p, c_int32, c_float, c_void_p,
                                    c_void_p, c_int64, c_void_p, c_void_p, c_size_t, c_void_p]),
    "pq_decode_attention_static": (c_int, [_LP, c_void_p, c_int, c_int32, c_int32, c_void_p, c_void_p, c_void_p,
                                           c_int32, c_void_p, c_int64, c_void_p, c_int32, c_void_p, c_int32, c_float,
                                           c_void_p, c_void_p, c_int64, c_void_p, c_void_p]),
    "pq_decode_partials": (c_int, [_LP, c_void_p, c_int, c_int32, c_int32, c_void_p, c_void_p, c_void_p,
                                   c_int32, c_void_p, c_int64, c_void_p, c_int32, c_void_p, c_int32, c_float, c_void_p,
                                   c_int64, c_void_p, c_void_p, c_size_t, c_void_p]),
    "pq_vq_bytes_per_page": (c_size_t, [_LP, c_int32]),
    "pq_vq_params_bytes_per_page": (c_size_t, [_LP]),
    "pq_encode_values": (c_int, [_LP, c_int32, c_void_p, c_int64, c_int64, c_int64, c_void_p, c_void_p, c_void_p,
                                 c_int64, c_void_p]),
    "pq_append_keys": (c_int, [_LP, c_void_p, c_int, c_int32, c_void_p, c_void_p, c_void_p, c_int32,
                               c_void_p, c_void_p, c_int64, c_void_p]),
    "pq_decode_merge": (c_int, [_LP, c_int32, c_int32, c_void_p, c_int32, c_void_p, c_void_p, c_size_t,
                                c_void_p]),
    "pq_score_keys": (c_int, [_LP, c_void_p, c_int, c_int32, c_int32, c_void_p, c_void_p, c_int64, c_void_p,
                              c_int32, c_void_p, c_int32, c_void_p, c_int64, c_void_p, c_void_p]),
    "pq_decode_kernel_name": (ctypes.c_char_p, [_LP, c_int32, c_int32, c_int32, c_int32]),
    "pq_decode_merges_in_kernel": (c_int32, [_LP, c_int32, c_int32, c_int32, c_int32]),
    "pq_probe_read_stream": (c_int, [c_void_p, c_size_t, c_void_p, c_void_p]),
}


def load_library():
    """Loads libpolarquant.so from the package directory; raises if it is not built."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise PolarQuantError(
                f"{path} is missing: build it with `python -m paper_2502_00527_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(path)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _check(status: int, what: str) -> None:
    if status != 0:
        lib = load_library()
        msg = lib.pq_strerror(status).decode()
        extra = f" (hipError_t {lib.pq_last_hip_error()})" if status == -4 else ""
        raise PolarQuantError(f"{what}: {msg}{extra}")


def _dev_ptr(t, name: str, dtypes=None) -> int:
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise PolarQuantError(f"{name} must be a device tensor")
    if dtypes is not None and t.dtype not in dtypes:
        raise PolarQuantError(f"{name} has dtype {t.dtype}, expected one of {dtypes}")
    if not t.is_contiguous():
        raise PolarQuantError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _float_kind(t, name: str) -> int:
    import torch
    if t.dtype == torch.float16:
        return PQ_F16
    if t.dtype == torch.float32:
        return PQ_F32
    raise PolarQuantError(f"{name} must be float16 or float32")


def pq_version() -> int:
    return load_library().pq_version()


def pq_strerror(status: int) -> str:
    return load_library().pq_strerror(status).decode()


def pq_codes_bytes_per_page(layout: Layout) -> int:
    return load_library().pq_codes_bytes_per_page(ctypes.byref(layout))


def pq_params_bytes_per_page(layout: Layout) -> int:
    return load_library().pq_params_bytes_per_page(ctypes.byref(layout))


def pq_values_bytes_per_page(layout: Layout) -> int:
    return load_library().pq_values_bytes_per_page(ctypes.byref(layout))


def pq_decode_workspace_bytes(layout: Layout, n_seqs: int, n_q_heads: int, max_seq_len: int) -> int:
    return load_library().pq_decode_workspace_bytes(ctypes.byref(layout), n_seqs, n_q_heads, max_seq_len)


def pq_decode_merges_in_kernel(layout: Layout, n_seqs: int, n_q_heads: int, max_seq_len: int, v_bits: int = 16) -> bool:
    st = load_library().pq_decode_merges_in_kernel(ctypes.byref(layout), n_seqs, n_q_heads, max_seq_len, v_bits)
    if st < 0:
        _check(st, "pq_decode_merges_in_kernel")
    return bool(st)


def pq_decode_kernel_name(layout: Layout, n_seqs: int, n_q_heads: int, max_seq_len: int, v_bits: int = 16) -> str:
    return load_library().pq_decode_kernel_name(ctypes.byref(layout), n_seqs, n_q_heads, max_seq_len, v_bits).decode()


def _key_pool_pages(layout: Layout, codes_pool, params_pool) -> int:
    """Pages the codes pool holds; the parameter pool must hold as many (its page size doubles
    with the grouped angle quantizer)."""
    n = codes_pool.numel() * codes_pool.element_size() // max(1, pq_codes_bytes_per_page(layout))
    if params_pool.numel() * params_pool.element_size() < n * pq_params_bytes_per_page(layout):
        raise PolarQuantError("params pool holds fewer pages than the codes pool")
    return n


def pq_encode_keys(layout: Layout, keys, page_ids, codes_pool, params_pool) -> None:
    """keys [n_tokens, n_kv_heads, d] (last dim contiguous, fp16/fp32, device); page_ids int32
    [ceil(n_tokens/g)] device; pools uint8 device tensors holding whole pages."""
    import torch
    if keys.dim() != 3 or keys.shape[1] != layout.n_kv_heads or keys.shape[2] != layout.head_dim:
        raise PolarQuantError("keys must be [n_tokens, n_kv_heads, head_dim]")
    if keys.stride(2) != 1 or not keys.is_cuda:
        raise PolarQuantError("keys must be a device tensor with a contiguous last dimension")
    n_pool_pages = _key_pool_pages(layout, codes_pool, params_pool)
    st = load_library().pq_encode_keys(
        ctypes.byref(layout), keys.data_ptr(), _float_kind(keys, "keys"), keys.stride(0), keys.stride(1),
        keys.shape[0], _dev_ptr(page_ids, "page_ids", (torch.int32,)), _dev_ptr(codes_pool, "codes_pool"),
        _dev_ptr(params_pool, "params_pool"), n_pool_pages, _stream())
    _check(st, "pq_encode_keys")


def _decode_common(layout, q, codes_pool, params_pool, v_pool, block_table, seq_lens, v_bits=16, v_params=None):
    import torch
    if q.dim() != 3 or q.shape[2] != layout.head_dim:
        raise PolarQuantError("q must be [n_seqs, n_q_heads, head_dim]")
    n_pool_pages = _key_pool_pages(layout, codes_pool, params_pool)
    if v_bits == 16:
        v_ptr, vp_ptr = _dev_ptr(v_pool, "v_pool", (torch.float16,)), None
        n_v_pages = v_pool.numel() * v_pool.element_size() // max(1, pq_values_bytes_per_page(layout))
    else:
        v_ptr, vp_ptr = _dev_ptr(v_pool, "v_pool", (torch.uint8,)), _dev_ptr(v_params, "v_params", (torch.float16,))
        n_v_pages = v_pool.numel() // max(1, pq_vq_bytes_per_page(layout, v_bits))
    if n_v_pages < n_pool_pages:
        raise PolarQuantError("value pool holds fewer pages than the codes pool")
    return dict(
        q=_dev_ptr(q, "q"), qk=_float_kind(q, "q"), n_seqs=q.shape[0], n_q=q.shape[1],
        codes=_dev_ptr(codes_pool, "codes_pool"), params=_dev_ptr(params_pool, "params_pool"),
        v=v_ptr, vbits=v_bits, vpar=vp_ptr, n_pool=n_pool_pages,
        bt=_dev_ptr(block_table, "block_table", (torch.int32,)), width=block_table.shape[1],
        lens=_dev_ptr(seq_lens, "seq_lens", (torch.int32,)))


def pq_decode_attention(layout: Layout, q, codes_pool, params_pool, v_pool, block_table, seq_lens,
                        max_seq_len: int, sm_scale: float, out, workspace, scores=None, residual=None,
                        v_bits: int = 16, v_params=None) -> None:
    """One decode step per sequence; see include/polarquant.h.  `out` fp32 [n_seqs, n_q_heads, d];
    `scores` optional fp32 [n_seqs, n_q_heads, stride >= max_seq_len]; `workspace` a uint8 device
    tensor of at least pq_decode_workspace_bytes(...) bytes."""
    import torch
    c = _decode_common(layout, q, codes_pool, params_pool, v_pool, block_table, seq_lens, v_bits, v_params)
    st = load_library().pq_decode_attention(
        ctypes.byref(layout), c["q"], c["qk"], c["n_seqs"], c["n_q"], c["codes"], c["params"], c["v"],
        c["vbits"], c["vpar"], c["n_pool"], c["bt"], c["width"], c["lens"], max_seq_len, sm_scale,
        _dev_ptr(out, "out", (torch.float32,)),
        None if scores is None else _dev_ptr(scores, "scores", (torch.float32,)),
        0 if scores is None else scores.shape[-1],
        None if residual is None else _dev_ptr(residual, "residual", (torch.float16,)),
        _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream())
    _check(st, "pq_decode_attention")


def pq_decode_attention_static(layout: Layout, q, codes_pool, params_pool, v_pool, block_table, seq_lens,
                               max_seq_len: int, sm_scale: float, out, scores=None, residual=None,
                               v_bits: int = 16, v_params=None) -> None:
    """pq_decode_attention without a workspace argument (the library's static scratch array)."""
    import torch
    c = _decode_common(layout, q, codes_pool, params_pool, v_pool, block_table, seq_lens, v_bits, v_params)
    st = load_library().pq_decode_attention_static(
        ctypes.byref(layout), c["q"], c["qk"], c["n_seqs"], c["n_q"], c["codes"], c["params"], c["v"],
        c["vbits"], c["vpar"], c["n_pool"], c["bt"], c["width"], c["lens"], max_seq_len, sm_scale,
        _dev_ptr(out, "out", (torch.float32,)),
        None if scores is None else _dev_ptr(scores, "scores", (torch.float32,)),
        0 if scores is None else scores.shape[-1],
        None if residual is None else _dev_ptr(residual, "residual", (torch.float16,)),
        _stream())
    _check(st, "pq_decode_attention_static")


def pq_decode_partials(layout: Layout, q, codes_pool, params_pool, v_pool, block_table, seq_lens,
                       max_seq_len: int, sm_scale: float, workspace, scores=None, residual=None,
                       v_bits: int = 16, v_params=None) -> None:
    import torch
    c = _decode_common(layout, q, codes_pool, params_pool, v_pool, block_table, seq_lens, v_bits, v_params)
    st = load_library().pq_decode_partials(
        ctypes.byref(layout), c["q"], c["qk"], c["n_seqs"], c["n_q"], c["codes"], c["params"], c["v"],
        c["vbits"], c["vpar"], c["n_pool"], c["bt"], c["width"], c["lens"], max_seq_len, sm_scale,
        None if scores is None else _dev_ptr(scores, "scores", (torch.float32,)),
        0 if scores is None else scores.shape[-1],
        None if residual is None else _dev_ptr(residual, "residual", (torch.float16,)),
        _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size(), _stream())
    _check(st, "pq_decode_partials")


def pq_decode_merge(layout: Layout, n_seqs: int, n_q_heads: int, seq_lens, max_seq_len: int, out,
                    workspace) -> None:
    import torch
    st = load_library().pq_decode_merge(
        ctypes.byref(layout), n_seqs, n_q_heads, _dev_ptr(seq_lens, "seq_lens", (torch.int32,)), max_seq_len,
        _dev_ptr(out, "out", (torch.float32,)), _dev_ptr(workspace, "workspace"),
        workspace.numel() * workspace.element_size(), _stream())
    _check(st, "pq_decode_merge")


def pq_vq_bytes_per_page(layout: Layout, v_bits: int) -> int:
    return load_library().pq_vq_bytes_per_page(ctypes.byref(layout), v_bits)


def pq_vq_params_bytes_per_page(layout: Layout) -> int:
    return load_library().pq_vq_params_bytes_per_page(ctypes.byref(layout))


def pq_encode_values(layout: Layout, v_bits: int, values, page_ids, vq_pool, vq_params) -> None:
    """values fp16 [n_tokens, n_kv_heads, d] (last dim contiguous, device); vq_pool uint8, vq_params fp16
    device tensors holding whole pages."""
    import torch
    if values.dim() != 3 or values.shape[1] != layout.n_kv_heads or values.shape[2] != layout.head_dim:
        raise PolarQuantError("values must be [n_tokens, n_kv_heads, head_dim]")
    if values.dtype != torch.float16 or values.stride(2) != 1 or not values.is_cuda:
        raise PolarQuantError("values must be a device fp16 tensor with a contiguous last dimension")
    n_pool_pages = vq_pool.numel() // max(1, pq_vq_bytes_per_page(layout, v_bits))
    st = load_library().pq_encode_values(
        ctypes.byref(layout), v_bits, values.data_ptr(), values.stride(0), values.stride(1), values.shape[0],
        _dev_ptr(page_ids, "page_ids", (torch.int32,)), _dev_ptr(vq_pool, "vq_pool", (torch.uint8,)),
        _dev_ptr(vq_params, "vq_params", (torch.float16,)), n_pool_pages, _stream())
    _check(st, "pq_encode_values")


def pq_append_keys(layout: Layout, new_keys, residual, seq_lens, block_table, codes_pool, params_pool) -> None:
    """new_keys [n_seqs, n_kv_heads, d] fp16/fp32; residual fp16 [n_seqs, n_kv_heads, g, d]; seq_lens int32
    [n_seqs] = lengths before the append (the caller increments them afterwards)."""
    import torch
    if new_keys.dim() != 3 or new_keys.shape[1] != layout.n_kv_heads or new_keys.shape[2] != layout.head_dim:
        raise PolarQuantError("new_keys must be [n_seqs, n_kv_heads, head_dim]")
    n_pool_pages = _key_pool_pages(layout, codes_pool, params_pool)
    st = load_library().pq_append_keys(
        ctypes.byref(layout), _dev_ptr(new_keys, "new_keys"), _float_kind(new_keys, "new_keys"), new_keys.shape[0],
        _dev_ptr(residual, "residual", (torch.float16,)), _dev_ptr(seq_lens, "seq_lens", (torch.int32,)),
        _dev_ptr(block_table, "block_table", (torch.int32,)), block_table.shape[1],
        _dev_ptr(codes_pool, "codes_pool"), _dev_ptr(params_pool, "params_pool"), n_pool_pages, _stream())
    _check(st, "pq_append_keys")


def pq_score_keys(layout: Layout, q, codes_pool, params_pool, block_table, seq_lens, max_seq_len: int,
                  scores, residual=None) -> None:
    """Raw q . k~ of every cached token; `scores` fp32 [n_seqs, n_q_heads, stride >= max_seq_len];
    `residual` optional fp16 [n_seqs, n_kv_heads, g, d] (the un-quantized keys of the last group)."""
    import torch
    if q.dim() != 3 or q.shape[2] != layout.head_dim:
        raise PolarQuantError("q must be [n_seqs, n_q_heads, head_dim]")
    n_pool_pages = _key_pool_pages(layout, codes_pool, params_pool)
    st = load_library().pq_score_keys(
        ctypes.byref(layout), _dev_ptr(q, "q"), _float_kind(q, "q"), q.shape[0], q.shape[1],
        _dev_ptr(codes_pool, "codes_pool"), _dev_ptr(params_pool, "params_pool"), n_pool_pages,
        _dev_ptr(block_table, "block_table", (torch.int32,)), block_table.shape[1],
        _dev_ptr(seq_lens, "seq_lens", (torch.int32,)), max_seq_len,
        _dev_ptr(scores, "scores", (torch.float32,)), scores.shape[-1],
        None if residual is None else _dev_ptr(residual, "residual", (torch.float16,)), _stream())
    _check(st, "pq_score_keys")


def pq_probe_read_stream(src, sink) -> None:
    """Streams `src` (device tensor, byte size a multiple of 16) once; `sink` int32/uint32 [64] device."""
    st = load_library().pq_probe_read_stream(_dev_ptr(src, "src"), src.numel() * src.element_size(),
                                             _dev_ptr(sink, "sink"), _stream())
    _check(st, "pq_probe_read_stream")
