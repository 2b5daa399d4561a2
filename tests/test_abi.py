"""The C-ABI library loads, exports every symbol the public header declares, and its
host-side logic (sizes, chunk plan, argument checks) behaves -- no GPU needed: every
call here returns before anything is launched."""
import ctypes
import os
import re

import pytest

import paper_2502_00527_amd as pq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(pq.lib_path()):
        from paper_2502_00527_amd import build
        build.build(verbose=False)
    return pq.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "polarquant.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pq_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"pq_encode_keys", "pq_decode_attention"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in polarquant.h but not exported"
    assert set(names) == set(pq._SIGNATURES), "binding and header disagree on the entry points"


def test_page_sizes_and_bit_accounting(lib):
    lay = pq.Layout(128, 4, 4, 128, 8)
    assert pq.pq_codes_bytes_per_page(lay) == 8 * 128 * 64          # one byte per pair
    assert pq.pq_params_bytes_per_page(lay) == 8 * 64 * 4
    assert pq.pq_values_bytes_per_page(lay) == 8 * 128 * 128 * 2
    # (r+t)/2 bits per element + 16/g bits of parameters (Appendix B.1, uniform angle grid)
    bits = 8 * (pq.pq_codes_bytes_per_page(lay) + pq.pq_params_bytes_per_page(lay)) / (8 * 128 * 128)
    assert bits == 4.125
    # grouped angle quantizer: a second (scale, zero) per pair and group, 32/g bits in all (Appendix B.1)
    grouped = pq.Layout(128, 4, 4, 128, 8, 1)
    assert pq.pq_params_bytes_per_page(grouped) == 2 * 8 * 64 * 4
    assert pq.pq_codes_bytes_per_page(grouped) == pq.pq_codes_bytes_per_page(lay)
    assert 8 * (pq.pq_codes_bytes_per_page(grouped) + pq.pq_params_bytes_per_page(grouped)) / (8 * 128 * 128) == 4.25
    assert pq.pq_params_bytes_per_page(pq.Layout(128, 3, 3, 128, 8, 1)) == 2 * 8 * 64 * 4
    assert pq.pq_params_bytes_per_page(pq.Layout(128, 5, 3, 128, 8, 1)) == 2 * 8 * 64 * 4     # any bit allocation
    assert pq.pq_params_bytes_per_page(pq.Layout(128, 4, 4, 128, 8, 2)) == 0     # unknown quantizer
    lay33 = pq.Layout(128, 3, 3, 128, 8)
    assert pq.pq_codes_bytes_per_page(lay33) == 8 * 128 * 48
    for bad in (pq.Layout(64, 4, 4, 128, 8), pq.Layout(128, 4, 3, 128, 8), pq.Layout(128, 4, 4, 64, 8),
                pq.Layout(128, 6, 2, 128, 8), pq.Layout(128, 4, 4, 128, 0)):
        assert pq.pq_codes_bytes_per_page(bad) == 0


def test_workspace_size_follows_the_chunk_plan(lib):
    lay = pq.Layout(128, 4, 4, 128, 8)
    # 16 seqs x 8 kv heads, 256 pages: chunks of 32 pages -> 8 chunks per sequence (grid launches);
    # balanced launches need (768 work-groups + 128 units) x 4 heads slots, which is fewer; plus
    # 8-byte arrival words: one per unit and one per segment slot
    n = pq.pq_decode_workspace_bytes(lay, 16, 32, 32768)
    assert n == 16 * 32 * 8 * 128 * 4 + 16 * 32 * 8 * 2 * 4 + (128 + 768 + 128) * 8
    # one sequence x 8 kv heads, 1024 pages: (768 + 8) x 4 balanced slots exceed the 32 x 64 chunk slots
    n = pq.pq_decode_workspace_bytes(pq.Layout(128, 3, 3, 128, 8), 1, 32, 131072)
    assert n == 776 * 4 * 128 * 4 + 776 * 4 * 2 * 4 + (8 + 768 + 8) * 8 + 128      # rounded up to 256
    assert pq.pq_decode_workspace_bytes(lay, 1, 32, 1) > 0
    assert pq.pq_decode_workspace_bytes(lay, 0, 32, 128) == 0
    assert pq.pq_decode_workspace_bytes(lay, 1, 12, 128) == 0      # 12 query heads over 8 kv heads
    assert pq.pq_decode_workspace_bytes(lay, 1, 64, 128) > 0       # group of 8: two passes of 4
    assert pq.pq_decode_workspace_bytes(lay, 1, 8 * 17, 128) == 0  # group of 17 not served
    # the chunk count is a grid dimension: 2^31 - 1 tokens would need more than 65535 chunks of 32 pages
    assert pq.pq_decode_workspace_bytes(lay, 64, 32, 2 ** 31 - 1) == 0
    assert pq.pq_decode_workspace_bytes(lay, 64, 32, 65535 * 32 * 128) > 0


def test_dispatch_queries(lib):
    """Which kernel serves a shape, and whether it merges itself, are host decisions the library reports."""
    lay = pq.Layout(128, 4, 4, 128, 8)
    # the headline shape: role-specialised kernel, launch shared out evenly, merge in the kernel
    assert pq.pq_decode_kernel_name(lay, 16, 32, 32768) == "pq_decode_roles_kernel"
    assert pq.pq_decode_merges_in_kernel(lay, 16, 32, 32768) is True
    # one long sequence: same kernel, but one work-group per chunk and the merge kernel
    lay33 = pq.Layout(128, 3, 3, 128, 8)
    assert pq.pq_decode_kernel_name(lay33, 1, 32, 131072) == "pq_decode_roles_kernel"
    assert pq.pq_decode_merges_in_kernel(lay33, 1, 32, 131072) is False
    # small launches and 4-bit values at four query heads per KV head: the alternating-phase kernel
    assert pq.pq_decode_kernel_name(lay, 2, 32, 1024) == "pq_decode_partials_kernel"
    assert pq.pq_decode_merges_in_kernel(lay, 2, 32, 1024) is False
    assert pq.pq_decode_kernel_name(lay, 16, 32, 32768, 4) == "pq_decode_partials_kernel"
    assert pq.pq_decode_kernel_name(lay, 16, 16, 32768, 4) == "pq_decode_roles_kernel"
    assert pq.pq_decode_kernel_name(lay, 0, 32, 128) == ""
    with pytest.raises(pq.PolarQuantError):
        pq.pq_decode_merges_in_kernel(lay, 0, 32, 128)


def test_argument_errors_are_reported_before_any_launch(lib):
    lay = pq.Layout(128, 4, 4, 128, 8)
    null = ctypes.c_void_p(0)
    st = lib.pq_encode_keys(ctypes.byref(lay), null, 0, 1024, 128, 10, null, null, null, 4, null)
    assert st == -1 and pq.pq_strerror(st) == "invalid argument"
    assert lib.pq_encode_keys(ctypes.byref(lay), null, 0, 1024, 128, 0, null, null, null, 4, null) == 0
    bad = pq.Layout(128, 7, 1, 128, 8)
    assert lib.pq_encode_keys(ctypes.byref(bad), null, 0, 1024, 128, 10, null, null, null, 4, null) == -2
    st = lib.pq_decode_attention(ctypes.byref(lay), null, 0, 1, 32, null, null, null, 16, null, 4, null, 1, null, 128,
                                 0.1, null, null, 0, null, null, 0, null)
    assert st == -1
    fake = ctypes.c_void_p(4096)
    st = lib.pq_decode_partials(ctypes.byref(lay), fake, 0, 1, 32, fake, fake, fake, 16, null, 4, fake, 1, fake, 128,
                                0.1, null, 0, null, null, 0, null)
    assert st == -3 and "workspace" in pq.pq_strerror(st)
    # more pages needed than the block table is wide
    st = lib.pq_decode_partials(ctypes.byref(lay), fake, 0, 1, 32, fake, fake, fake, 16, null, 4, fake, 1, fake, 129,
                                0.1, null, 0, null, fake, 1 << 20, null)
    assert st == -1
    # quantized values need their parameter pool; 3-bit values are not built
    st = lib.pq_decode_partials(ctypes.byref(lay), fake, 0, 1, 32, fake, fake, fake, 4, null, 4, fake, 1, fake, 128,
                                0.1, null, 0, null, fake, 1 << 20, null)
    assert st == -1
    st = lib.pq_decode_partials(ctypes.byref(lay), fake, 0, 1, 32, fake, fake, fake, 3, fake, 4, fake, 1, fake, 128,
                                0.1, null, 0, null, fake, 1 << 20, null)
    assert st == -2
    assert pq.pq_vq_bytes_per_page(lay, 4) == 8 * 128 * 64 and pq.pq_vq_bytes_per_page(lay, 2) == 8 * 128 * 32
    assert pq.pq_vq_bytes_per_page(lay, 3) == 0 and pq.pq_vq_params_bytes_per_page(lay) == 8 * 128 * 4
    st = lib.pq_encode_values(ctypes.byref(lay), 4, null, 1024, 128, 10, null, null, null, 4, null)
    assert st == -1
    st = lib.pq_append_keys(ctypes.byref(lay), null, 0, 4, null, null, null, 8, null, null, 16, null)
    assert st == -1
    # r + t must be 6 or 8, with either angle quantizer
    odd = pq.Layout(128, 5, 4, 128, 8, 1)
    st = lib.pq_decode_partials(ctypes.byref(odd), fake, 0, 1, 32, fake, fake, fake, 16, null, 4, fake, 1, fake, 128,
                                0.1, null, 0, null, fake, 1 << 20, null)
    assert st == -2
    # the allocation-free variant refuses, on the host, shapes beyond its static scratch array
    st = lib.pq_decode_attention_static(ctypes.byref(lay), fake, 0, 512, 32, fake, fake, fake, 16, null, 4, fake, 128,
                                        fake, 16384, 0.1, fake, null, 0, null, null)
    assert st == -5 and "static" in pq.pq_strerror(st)
    assert pq.pq_version() >= 102


def test_bench_refuses_more_than_one_gpu():
    """bench.py is single-GPU by construction: --gpus 2 exits with a message before touching the device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
