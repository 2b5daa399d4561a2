#!/usr/bin/env python3
"""Benchmark of decode attention over the polar-quantized key cache on one MI355X.

A step is one pass of the whole decode hot path -- table build, table-lookup
scoring of every cached key, online softmax, fp16 value aggregation, chunk
merge -- over one batch of synthetic sequences (one decode step per sequence).
The cache is encoded beforehand by pq_encode_keys and is resident in HBM when
the timed region starts.  The metric is keys scored per second (query-head x
cached-token scores); the roofline object prices the dominant kernel
(the attention kernel behind pq_decode_partials) against the 8 TB/s HBM peak using the algorithmic bytes of
the packed cache: per (KV head, token) 64*w/8 B of codes + 2 B of radius
parameters + 256 B of fp16 values.

Prints ONE JSON line.  `--gpus` above 1 is refused: this build is single-GPU.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0


def algorithmic_bytes(wl, lens, v_bits: int = 16) -> int:
    """Bytes the method must move per launch: codes + radius params + values (fp16, or b-bit codes
    plus 4 bytes of scale / zero-point per token) of every cached (KV head, token)."""
    w = wl.r_bits + wl.t_bits
    v_bytes = wl.head_dim * 2 if v_bits == 16 else wl.head_dim * v_bits // 8 + 4
    param_sets = 2 if wl.grouped_angles else 1      # radius (and angle) scale / zero-point per pair and group
    per_token = (wl.head_dim // 2) * w // 8 + (wl.head_dim // 2) * 4 * param_sets / wl.group_tokens + v_bytes
    return int(round(float(lens.astype("int64").sum()) * wl.n_kv_heads * per_token))


def time_region(fn, n, torch):
    """Average milliseconds of n back-to-back calls of fn on torch's current stream (HIP events)."""
    start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    start.record()
    for _ in range(n):
        fn()
    stop.record()
    torch.cuda.synchronize()
    return start.elapsed_time(stop) / n


def _cpu_worker(wl, lens, my_seqs, budget_s, barrier, result_q):
    """One host core's share of the oracle baseline: prepare its sequences (untimed: that is
    prefill), wait for the others, then run the oracle's decode over them again and again until
    `budget_s` seconds have passed.  Reports (scores computed, start, end) on the shared clock."""
    import numpy as np
    from threadpoolctl import threadpool_limits

    from oracle import attention, cache_format, polar
    from paper_2502_00527_amd import workloads as W

    g = wl.group_tokens
    with threadpool_limits(limits=1):
        q = W.queries(wl)
        prepared = []
        for s in my_seqs:
            L = int(lens[s])
            keys = W.keys_for_seq(wl, s, L)
            enc = polar.encode_keys(keys, wl.r_bits, wl.t_bits, g, grouped_angles=wl.grouped_angles)
            codes, params = cache_format.pack_sequence(enc["a"], enc["c"], enc["scale"], enc["zero"],
                                                       wl.r_bits, wl.t_bits, g, enc.get("t_scale"), enc.get("t_zero"))
            n_pages = codes.shape[0]
            vals = np.zeros((n_pages * g, wl.n_kv_heads, wl.head_dim), np.float16)
            vals[:L] = W.values_for_seq(wl, s, L)
            v_pool = np.ascontiguousarray(vals.reshape(n_pages, g, wl.n_kv_heads, wl.head_dim).transpose(0, 2, 1, 3))
            prepared.append((s, L, codes, params, v_pool, np.arange(n_pages, dtype=np.int32)[None, :]))
            del keys, enc, vals
        barrier.wait()
        t0 = time.perf_counter()
        scored = 0
        while True:
            for s, L, codes, params, v_pool, table in prepared:
                attention.decode_attention(q[s:s + 1], codes, params, v_pool, table, np.array([L]), wl.r_bits,
                                           wl.t_bits, g, 1.0 / np.sqrt(wl.head_dim))
                scored += L * wl.n_q_heads
                if time.perf_counter() - t0 >= budget_s:
                    break
            if time.perf_counter() - t0 >= budget_s:
                break
        result_q.put((scored, t0, time.perf_counter()))


def cpu_baseline(wl, lens, budget_s: float = 10.0):
    """The oracle's decode (unpack -> dequantize -> dot -> softmax -> P.V, float64) on the host
    cores this process may use: one worker process per core (BLAS held to one thread each, so the
    core count is exact), sequences of the same workload dealt round-robin, each worker decoding
    its sequences repeatedly for about `budget_s` seconds.  Rate = all scores computed / wall time
    between the first worker's start and the last one's end.  Must run before this process touches
    the GPU: the workers are forked."""
    import multiprocessing as mp

    cores = len(os.sched_getaffinity(0))
    n_workers = max(1, min(cores, wl.n_seqs))
    ctx = mp.get_context("fork")
    barrier = ctx.Barrier(n_workers)
    result_q = ctx.Queue()
    procs = []
    for w in range(n_workers):
        my = list(range(w, wl.n_seqs, n_workers))[:2]     # at most two sequences per worker: bounded set-up time
        procs.append(ctx.Process(target=_cpu_worker, args=(wl, lens, my, budget_s, barrier, result_q)))
        procs[-1].start()
    got = [result_q.get() for _ in procs]
    for p in procs:
        p.join()
    scored = sum(g[0] for g in got)
    wall = max(g[2] for g in got) - min(g[1] for g in got)
    used = sorted({s for w in range(n_workers) for s in list(range(w, wl.n_seqs, n_workers))[:2]})
    return {"value": scored / wall, "unit": "keys/s", "cores": n_workers, "kind": "oracle",
            "host_cores_available": cores,
            "sample": f"{len(used)} of {wl.n_seqs} sequences of the same workload, decoded repeatedly by {n_workers} "
                      f"worker processes (one per host core, one BLAS thread each) for {wall:.1f} s: {scored} scores "
                      f"of NumPy float64 decode; encode not timed"}


def read_traffic_note(workload: str, kernel: str):
    """(HBM bytes per launch, source) of the dominant kernel as measured with rocprofv3 --pmc, if a
    committed summary for this workload states it for the kernel that runs
    (profiles/decode_attention_<workload>_pmc.txt); counters cannot be read inside a timed run, so
    this is a recorded figure, not one measured by this process."""
    rel = os.path.join("profiles", f"decode_attention_{workload}_pmc.txt")
    try:
        with open(os.path.join(ROOT, rel)) as f:
            text = f.read()
    except OSError:
        return None, None
    if kernel not in text:
        return None, None
    for line in text.splitlines():
        if line.startswith("traffic_bytes_per_launch:"):
            return int(float(line.split(":", 1)[1].split()[0])), rel + " (recorded with rocprofv3 --pmc, not measured in this run)"
    return None, None


def preheat(fn, torch, min_busy_ms: float = 60.0, window: int = 20, tol: float = 0.02, max_busy_ms: float = 2000.0):
    """Untimed steps until the device runs at its steady clocks: windows of `window` steps until at
    least `min_busy_ms` of load have passed and two consecutive windows agree within `tol` (an idle
    device takes some tens of milliseconds of load to raise its clocks).  Returns what was done."""
    busy, n, first, prev = 0.0, 0, None, None
    while True:
        ms = time_region(fn, window, torch)
        busy += ms * window
        n += window
        if first is None:
            first = ms
        if busy >= min_busy_ms and prev is not None and abs(ms - prev) <= tol * prev:
            break
        if busy >= max_busy_ms:
            break
        prev = ms
    return {"steps": n, "busy_ms": busy, "first_window_ms_per_step": first, "last_window_ms_per_step": ms}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10, help="untimed steps before anything else")
    ap.add_argument("--no-preheat", action="store_true",
                    help="skip the disclosed, untimed pre-heat that follows the warm-up steps (an idle device needs "
                         "some tens of milliseconds of load to reach its steady clocks; see `preheat` in the output)")
    ap.add_argument("--workload", default="gqa", choices=["gqa", "mha", "long33", "ragged", "tiny"])
    ap.add_argument("--v-bits", type=int, default=16, choices=[16, 4, 2],
                    help="value precision: 16 = fp16 values (the headline configuration), 4 / 2 = token-wise quantized")
    ap.add_argument("--grouped-angles", action="store_true",
                    help="the paper's per-group min/scale angle quantizer instead of the uniform grid (the headline)")
    ap.add_argument("--copies", type=int, default=4,
                    help="independent copies of the packed cache that successive steps rotate over, so that the "
                         "256 MB memory-side cache cannot serve a step from the previous step's reads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=10.0,
                    help="seconds every host core spends in the oracle's decode")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np

    from paper_2502_00527_amd import workloads as W

    wl = W.WORKLOADS[args.workload]
    if args.grouped_angles:
        wl = wl.scaled(grouped_angles=True)

    # The oracle on the host cores comes first: its worker processes are forked, which has to
    # happen before this process initialises the GPU.
    cpu = None
    if not args.no_cpu_baseline:
        print("[bench] oracle baseline on the host cores ...", file=sys.stderr, flush=True)
        t0 = time.time()
        cpu = cpu_baseline(wl, W.seq_lengths(wl), args.cpu_budget)
        print(f"[bench] oracle baseline done in {time.time() - t0:.1f} s on {cpu['cores']} cores", file=sys.stderr, flush=True)

    import torch

    import paper_2502_00527_amd as pq
    from paper_2502_00527_amd.cache import build_device_cache

    pq.load_library()          # raises if libpolarquant.so is not built: there is no fallback
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    t0 = time.time()
    cache = build_device_cache(wl, v_bits=args.v_bits,
                               progress=lambda s: print(f"[bench] encoded sequence {s + 1}/{wl.n_seqs}",
                                                        file=sys.stderr, flush=True))
    torch.cuda.synchronize()
    print(f"[bench] inputs ready in {time.time() - t0:.1f} s", file=sys.stderr, flush=True)
    lens = cache.lens
    out = torch.empty((wl.n_seqs, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device="cuda:0")

    # N copies of the pools in one N-times larger pool; copy k is reached through block table k
    n_copies = max(1, args.copies)
    if n_copies > 1:
        import dataclasses
        rep = lambda t: None if t is None else torch.cat([t] * n_copies, dim=0)
        big = dataclasses.replace(cache, codes=rep(cache.codes), params=rep(cache.params), values=rep(cache.values),
                                  v_params=rep(cache.v_params), n_pool_pages=cache.n_pool_pages * n_copies)
        views = [dataclasses.replace(big, block_table=cache.block_table + k * cache.n_pool_pages)
                 for k in range(n_copies)]
        del big
    else:
        views = [cache]
    turn = [0]

    def next_view():
        turn[0] = (turn[0] + 1) % n_copies
        return views[turn[0]]

    def step():
        next_view().decode(out)

    def partials_only():
        c = next_view()
        pq.pq_decode_partials(c.layout, c.q, c.codes, c.params, c.values, c.block_table,
                              c.seq_lens, c.max_seq_len, c.sm_scale, c.workspace,
                              v_bits=c.v_bits, v_params=c.v_params)

    def merge_only():
        pq.pq_decode_merge(cache.layout, wl.n_seqs, wl.n_q_heads, cache.seq_lens, cache.max_seq_len, out,
                           cache.workspace)

    # buffers of the read-stream probe, allocated now so that nothing idles the device between the
    # timed regions below
    probe = torch.empty(2 << 30, dtype=torch.uint8, device="cuda:0").fill_(1)
    sink = torch.zeros(64, dtype=torch.int32, device="cuda:0")

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # Disclosed pre-heat, untimed and independent of --warmup: an idle device runs its first tens of
    # milliseconds of load at lower clocks (the first window's time is reported as the cold figure).
    heat = None if args.no_preheat else preheat(step, torch)
    t_start = time.perf_counter()
    ms_step = time_region(step, args.steps, torch)
    wall = time.perf_counter() - t_start
    # the dominant kernel alone, same launch configuration, same stream, same clock state.  The
    # role-specialised kernel merges inside the kernel: the step IS that one kernel, timed again
    # here in a region of its own; the other kernels are followed by a separate merge kernel.
    kernel = pq.pq_decode_kernel_name(cache.layout, wl.n_seqs, wl.n_q_heads, cache.max_seq_len, args.v_bits)
    one_kernel_step = pq.pq_decode_merges_in_kernel(cache.layout, wl.n_seqs, wl.n_q_heads, cache.max_seq_len, args.v_bits)
    ms_partials = time_region(step if one_kernel_step else partials_only, args.steps, torch)
    ms_merge = 0.0 if one_kernel_step else time_region(merge_only, args.steps, torch)
    # what this device streams with bare non-temporal 128-bit loads (context for the roofline
    # fraction), timed right behind the kernel so that both see the same clocks
    for _ in range(5):
        pq.pq_probe_read_stream(probe, sink)
    ms_probe = time_region(lambda: pq.pq_probe_read_stream(probe, sink), 20, torch)
    read_stream_gbps = probe.numel() / (ms_probe * 1e-3) / 1e9
    del probe

    # the query-key product alone (pq_score_keys): the one operation the paper itself times
    # (Section 5.2, batch 8); context beside the headline, not part of `value`
    qk = None
    if wl.n_seqs >= 8:
        scores = torch.empty((8, wl.n_q_heads, cache.max_seq_len), dtype=torch.float32, device="cuda:0")
        q8, bt8, sl8 = cache.q[:8].contiguous(), cache.block_table[:8].contiguous(), cache.seq_lens[:8].contiguous()

        def qk_only():
            pq.pq_score_keys(cache.layout, q8, cache.codes, cache.params, bt8, sl8, cache.max_seq_len, scores)

        for _ in range(args.warmup):
            qk_only()
        if not args.no_preheat:
            preheat(qk_only, torch, min_busy_ms=20.0)
        ms_qk = time_region(qk_only, args.steps, torch)
        n_scores = int(lens[:8].astype(np.int64).sum()) * wl.n_q_heads
        qk = {"entry_point": "pq_score_keys", "batch": 8, "ms_per_call": ms_qk,
              "scores_per_s": n_scores / (ms_qk * 1e-3),
              "note": "paper Table 2 (hardware not stated): PolarQuant44 at batch 8 x 32K = 1.49 s per 10K calls"}
        del scores

    # the prefill-time encoder on the 32768-token x 8-head fp16 prefill of the ragged configuration
    # (context: it runs once per prompt, not per decode step, and is no part of `value`)
    enc = None
    if True:
        pre = W.WORKLOADS["prefill"].scaled(grouped_angles=wl.grouped_angles, r_bits=wl.r_bits, t_bits=wl.t_bits)
        from paper_2502_00527_amd.cache import make_layout
        lay = make_layout(pre)
        n_tok = pre.max_len
        n_pg = n_tok // pre.group_tokens
        keys = torch.from_numpy(W.keys_for_seq(pre, 0, n_tok)).to("cuda:0")
        e_codes = torch.empty(n_pg * pq.pq_codes_bytes_per_page(lay), dtype=torch.uint8, device="cuda:0")
        e_params = torch.empty(n_pg * pq.pq_params_bytes_per_page(lay), dtype=torch.uint8, device="cuda:0")
        ids = torch.arange(n_pg, dtype=torch.int32, device="cuda:0")

        def encode_only():
            pq.pq_encode_keys(lay, keys, ids, e_codes, e_params)

        for _ in range(10):
            encode_only()
        if not args.no_preheat:
            preheat(encode_only, torch, min_busy_ms=20.0)
        ms_enc = time_region(encode_only, 50, torch)
        enc_bytes = keys.numel() * keys.element_size() + e_codes.numel() + e_params.numel()
        enc = {"entry_point": "pq_encode_keys", "tokens": n_tok, "kv_heads": pre.n_kv_heads, "ms_per_call": ms_enc,
               "pairs_per_s": n_tok * pre.n_kv_heads * (pre.head_dim // 2) / (ms_enc * 1e-3),
               "GBps": enc_bytes / (ms_enc * 1e-3) / 1e9, "bound": "alu",
               "note": "exactly rounded fp32 radius chain and exact angle classification; not HBM-bound"}
        del keys, e_codes, e_params

    traffic, traffic_source = read_traffic_note(wl.name, kernel) if args.v_bits == 16 and not wl.grouped_angles else (None, None)
    keys_scored = int(lens.astype(np.int64).sum()) * wl.n_q_heads
    alg_bytes = algorithmic_bytes(wl, lens, args.v_bits)
    achieved = alg_bytes / (ms_partials * 1e-3) / 1e9
    result = {
        "metric": "decode keys scored/sec on polar-quantized cache",
        "value": keys_scored / (ms_step * 1e-3),
        "unit": "keys/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: {wl.n_seqs} seqs x {wl.n_q_heads} q heads over {wl.n_kv_heads} kv heads, "
                               f"head_dim {wl.head_dim}, context {wl.min_len}..{wl.max_len}, r{wl.r_bits}/t{wl.t_bits}, "
                               f"group {wl.group_tokens}, {'grouped' if wl.grouped_angles else 'uniform'} angle quantizer, {'fp16' if args.v_bits == 16 else str(args.v_bits) + '-bit'} values, "
                               f"RoPE base {wl.rope_base:g}",
                   "cache_copies_rotated": n_copies,
                   "keys_scored_per_step": keys_scored,
                   "kv_tokens_per_step": int(lens.astype(np.int64).sum()) * wl.n_kv_heads},
        "roofline": {"bound": "hbm",
                     "kernel": kernel, "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes": alg_bytes,
                     "ms_per_launch": ms_partials, "ms_merge_kernel": ms_merge, "merge_in_kernel": one_kernel_step,
                     "read_stream_GBps": read_stream_gbps,
                     "frac_of_read_stream": achieved / read_stream_gbps,
                     "whole_step_GBps": alg_bytes / (ms_step * 1e-3) / 1e9},
        "wall_s_timed_region": wall,
        "preheat": heat,
    }
    if qk is not None:
        result["qk_only"] = qk
    if enc is not None:
        result["encode"] = enc
    if cpu is not None:
        result["cpu_baseline"] = cpu
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
