#!/usr/bin/env python3
"""Benchmark of the paged KV-cache data path on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input, all inputs
resident in HBM: paged decode attention over the batch (partition kernel + merge kernel), then
pack of the step's dirty blocks into a contiguous replica, then restore of a replica (the one
packed a step earlier) into a second pool under fresh block ids.  The timed workload is the
long-context case (the largest decode working set); the other cases are reported under "extra":
a full 200k-block restore and pack (the copy-bandwidth figure), the replication mix with pack on a
side stream beside decode (overlap cost), and the 8B-layer case (cache-resident, latency only).

Prints ONE JSON line.  `value` is decode KV bytes per second: valid cached tokens x K/V bytes per
token, divided by the mean time of the decode call measured with HIP events inside the timed steps.
"""
import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X published dense bf16 matrix-core peak

# HBM traffic per decode launch from two `rocprofv3 --pmc` runs of this file (FETCH_SIZE, then
# WRITE_SIZE), scaled by the same counters on a plain copy of known size; see profiles/.  Valid
# only for the kernel sources (kv_decode.hip + kv_decode_common.h) the counters were taken with.
DECODE_TRAFFIC = {"kernel_sha256": "3472378714227b721abb12222d69300c8cdb5d05e02425179b5562a100ae2f66",
                  "fetch_bytes": 1290203005, "write_bytes": 2371422}

PAPER_CONTEXT = {
    "note": "end-to-end serving figures from the paper, other hardware, context only",
    "hardware": "8/16 nodes, one NVIDIA A10 24GB per node, 1 Gbps Ethernet, Llama-3.1-8B, 4-stage pipeline",
    "mttr_s": [35, 30, 29], "mttr_baseline_s": 600,
    "tpot_ms_avg_p99": [163, 203],
    "best_avg_latency_improvement": 3.12, "best_p99_latency_improvement": 2.85,
    "best_avg_ttft_improvement": 378.91, "best_p99_ttft_improvement": 574.56,
    "replication_overhead_pct_avg_p99": {"8_nodes": [2.3, 2.8], "16_nodes": [4.0, 3.6]},
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def bf16_dev(bits):
    import torch
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


class Decode:
    """Device-resident inputs of one decode case plus its output and workspace."""

    def __init__(self, case, pool, kvflow, out_dtype=None):
        import torch
        g = case.geom
        self.case, self.kvflow, self.pool = case, kvflow, pool
        self.q = bf16_dev(case.q)
        self.table = torch.from_numpy(case.block_table).cuda()
        self.lens = torch.from_numpy(case.context_lens).cuda()
        self.out = torch.empty((case.batch, g.num_q_heads, g.head_dim), device="cuda",
                               dtype=out_dtype or torch.bfloat16)
        self.max_len = case.max_context_len
        nbytes = kvflow.kv_decode_workspace_bytes(case.batch, g.num_q_heads, g.num_kv_heads, g.head_dim,
                                                  self.max_len, 0)
        self.ws = torch.empty(nbytes // 4, dtype=torch.float32, device="cuda")
        self.workgroups = kvflow.kv_decode_workgroups(case.batch, g.num_kv_heads, self.max_len, 0)
        self.scale = float(g.scale)

    def run(self, stream=None):
        self.kvflow.kv_decode_attn(self.out, self.q, self.pool, self.table, self.lens, self.max_len,
                                   self.scale, 0, self.ws, stream)


def event_ms(pairs):
    return [a.elapsed_time(b) for a, b in pairs]


def stats(ms):
    a = np.asarray(ms, dtype=np.float64)
    return {"mean_ms": float(a.mean()), "median_ms": float(np.median(a)), "min_ms": float(a.min())}


def time_calls(fn, iters, warmup):
    """Mean/median/min duration of fn() on the current stream, one HIP event pair per call."""
    import torch
    for _ in range(warmup):
        fn()
    pairs = []
    for _ in range(iters):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        fn()
        b.record()
        pairs.append((a, b))
    torch.cuda.synchronize()
    return stats(event_ms(pairs))


def copy_rates(payload_bytes, ms):
    gbps = payload_bytes / (ms * 1e-3) / 1e9
    return {"payload_GBps": gbps, "traffic_GBps": 2 * gbps, "frac_hbm_peak": 2 * gbps / HBM_PEAK_GBPS}


def bench_long_context(args, kvflow, W):
    """The timed workload: K steps of decode -> pack -> restore on one stream."""
    import torch
    t0 = time.time()
    case = W.long_context()
    g = case.geom
    log(f"[bench] long_context generated in {time.time() - t0:.1f}s: lens={case.context_lens.tolist()} "
        f"pool={case.num_blocks} blocks, dirty={len(case.dirty_ids)}")
    pool = bf16_dev(case.pool)
    dec = Decode(case, pool, kvflow)
    n = len(case.dirty_ids)
    ids = torch.from_numpy(case.dirty_ids).cuda()
    replicas = [torch.empty((n,) + pool.shape[1:], dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    # the recovery target: a second pool and fresh ids for the restored blocks
    target = torch.zeros_like(pool)
    fresh = np.random.default_rng(12345).permutation(case.num_blocks)[:n].astype(np.int32)
    fresh_ids = torch.from_numpy(fresh).cuda()
    kvflow.kv_pack_blocks(replicas[1], pool, ids)          # the replica the first restore consumes

    def step(i, evs=None):
        if evs is not None:
            evs[0].record()
        dec.run()
        if evs is not None:
            evs[1].record()
        kvflow.kv_pack_blocks(replicas[i & 1], pool, ids)
        if evs is not None:
            evs[2].record()
        kvflow.kv_restore_blocks(target, replicas[(i + 1) & 1], fresh_ids)
        if evs is not None:
            evs[3].record()

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    all_evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, all_evs[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # the same steps captured once into a HIP graph and replayed (no host launch cost between kernels)
    graph_ms = None
    try:
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(cap):
            with torch.cuda.graph(graph, stream=cap):
                step(0)
                step(1)
        torch.cuda.synchronize()
        for _ in range(3):
            graph.replay()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = max(1, args.steps // 2)
        g0.record()
        for _ in range(reps):
            graph.replay()
        g1.record()
        torch.cuda.synchronize()
        graph_ms = g0.elapsed_time(g1) / (2 * reps)
    except Exception as exc:                                  # graph capture is a convenience figure only
        log(f"[bench] graph replay skipped: {exc}")
    d_ms = stats([e[0].elapsed_time(e[1]) for e in all_evs])
    p_ms = stats([e[1].elapsed_time(e[2]) for e in all_evs])
    r_ms = stats([e[2].elapsed_time(e[3]) for e in all_evs])
    kv_bytes = case.kv_bytes
    payload = n * g.block_bytes
    # what the timed steps wrote, kept on the host for the parity figures printed beside the rate
    written = {"out": dec.out.double().cpu().numpy(),
               "replicas": [r.view(torch.int16).cpu().numpy().view(np.uint16) for r in replicas],
               "target": target.view(torch.int16).cpu().numpy().view(np.uint16), "fresh_ids": fresh}
    del target
    res = {
        "case": case, "dec": dec, "pool": pool, "ids": ids, "replica": replicas[0], "written": written,
        "ms_per_step": wall / args.steps * 1e3, "graph_ms_per_step": graph_ms,
        "decode": d_ms, "pack": p_ms, "restore": r_ms,
        "kv_bytes": kv_bytes, "payload": payload,
        "decode_GBps": kv_bytes / (d_ms["mean_ms"] * 1e-3) / 1e9,
    }
    return res


def cpu_baseline(case, oracle, n_seqs=None):
    """The oracle as it stands, timed on this host: all query heads of the first n_seqs sequences."""
    g = case.geom
    n_seqs = case.batch if n_seqs is None else n_seqs
    rows = np.array([(b, h) for b in range(n_seqs) for h in range(g.num_q_heads)], np.int32)
    t0 = time.perf_counter()
    want, threads = oracle.decode_attn(case.q, case.pool, case.block_table, case.context_lens, g.scale,
                                       rows=rows, return_threads=True)
    dt = time.perf_counter() - t0
    sample_bytes = int(case.context_lens[:n_seqs].astype(np.int64).sum()) * g.kv_bytes_per_token
    t0 = time.perf_counter()
    rep, _ = oracle.pack_blocks(case.pool, case.dirty_ids, return_threads=True)
    dt_pack = time.perf_counter() - t0
    return want.reshape(n_seqs, g.num_q_heads, g.head_dim), rep, {
        "value": sample_bytes / dt / 1e9, "unit": "GB/s", "cores": int(threads), "kind": "oracle",
        "sample": f"fp64 decode of all {g.num_q_heads} query heads of the first {n_seqs} of {case.batch} "
                  f"sequences of the timed workload ({sample_bytes / 1e6:.0f} MB of KV, {dt:.1f} s); "
                  f"pack of the full dirty list by memcpy: {rep.nbytes / dt_pack / 1e9:.2f} GB/s payload",
        "seconds": dt, "pack_payload_GBps": rep.nbytes / dt_pack / 1e9,
        "cpu_model": cpu_model(), "host_cores": os.cpu_count(),
    }


def parity_of_timed_buffers(case, written, want_out, want_replica, oracle):
    """The buffers the timed steps wrote against the oracle: decode output element by element, the packed
    replicas and the restored pool byte for byte."""
    err = np.abs(written["out"][:len(want_out)] - want_out)
    want_target = np.zeros_like(case.pool)
    oracle.restore_blocks(want_target, want_replica, written["fresh_ids"])
    return {"decode_max_abs": float(err.max()), "decode_mean_abs": float(err.mean()),
            "decode_rows_checked": int(err.shape[0] * err.shape[1]), "decode_finite": bool(np.isfinite(written["out"]).all()),
            "pack_bit_exact": bool(all(np.array_equal(r, want_replica) for r in written["replicas"])),
            "restore_bit_exact": bool(np.array_equal(written["target"], want_target)),
            "tolerance": {"max_abs": 2e-2, "mean_abs": 2e-3}}


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def bench_recovery(args, kvflow, W, num_blocks):
    """Full-replica restore (and the symmetric pack) of num_blocks 64 KiB blocks, then a decode."""
    import torch
    t0 = time.time()
    rc = W.recovery(num_blocks=num_blocks)
    g = rc.geom
    shape = (num_blocks, 2, g.num_kv_heads, g.block_size, g.head_dim)
    replica = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    step = 16 * W.REPLICA_CHUNK_BLOCKS
    for first in range(0, num_blocks, step):
        nb = min(step, num_blocks - first)
        replica[first:first + nb] = bf16_dev(rc.replica_chunk(first, nb))
    log(f"[bench] recovery replica ({num_blocks} blocks, {replica.numel() * 2 / 1e9:.2f} GB) generated "
        f"and uploaded in {time.time() - t0:.1f}s")
    pool = torch.empty(shape, dtype=torch.bfloat16, device="cuda")
    ids = torch.from_numpy(rc.restore_ids).cuda()
    payload = num_blocks * g.block_bytes
    r = time_calls(lambda: kvflow.kv_restore_blocks(pool, replica, ids), args.copy_iters, 2)
    back = torch.empty_like(replica)
    p = time_calls(lambda: kvflow.kv_pack_blocks(back, pool, ids), args.copy_iters, 2)
    same = bool(torch.equal(back, replica))
    del back
    dec = Decode(rc.decode, pool, kvflow)
    d = time_calls(dec.run, 10, 3)
    out = {
        "blocks": num_blocks, "payload_GB": payload / 1e9,
        "restore": {**r, **copy_rates(payload, r["mean_ms"])},
        "pack": {**p, **copy_rates(payload, p["mean_ms"])},
        "pack_of_restore_is_identity": same,
        "decode_after_restore": {**d, "kv_GB": rc.decode.kv_bytes / 1e9, "workgroups": dec.workgroups,
                                 "kv_GBps": rc.decode.kv_bytes / (d["mean_ms"] * 1e-3) / 1e9,
                                 "frac_hbm_peak": rc.decode.kv_bytes / (d["mean_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS},
    }
    # plain device-to-device copy of the same bytes, as a yardstick of what a copy reaches here
    dst = torch.empty_like(replica)
    c = time_calls(lambda: dst.copy_(replica), args.copy_iters, 2)
    out["plain_copy_same_bytes"] = {**c, **copy_rates(payload, c["mean_ms"])}
    return out


def bench_replication_mix(args, kvflow, W):
    """Decode alone, pack alone, and pack on a side stream beside decode."""
    import torch
    case = W.replication_mix()
    g = case.geom
    pool = bf16_dev(case.pool)
    dec = Decode(case, pool, kvflow)
    ids = torch.from_numpy(case.dirty_ids).cuda()
    n = len(case.dirty_ids)
    replica = torch.empty((n,) + pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    d = time_calls(dec.run, 20, 5)
    p = time_calls(lambda: kvflow.kv_pack_blocks(replica, pool, ids), 20, 5)
    side = torch.cuda.Stream()
    main = torch.cuda.current_stream()
    # token-granular replication ships the new K/V rows only: their gather is the whole device-side cost
    positions = torch.from_numpy(np.maximum(case.context_lens - 1, 0).astype(np.int32)).cuda()  # the newest slot
    k_out = torch.empty((case.batch, g.num_kv_heads, g.head_dim), dtype=torch.bfloat16, device="cuda")
    v_out = torch.empty_like(k_out)

    def train(n_iter, with_pack):
        """n_iter decode steps back to back on the main stream.  with_pack = "side": every step also
        starts a pack on the side stream, ordered after the previous step by an event (as a pack of
        freshly written blocks has to be); "same": the pack follows the decode on the main stream.
        Returns ms per step."""
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0.record(main)
        for _ in range(n_iter):
            if with_pack in ("side", "fork_only"):
                ev = torch.cuda.Event()
                ev.record(main)
                side.wait_event(ev)
                if with_pack == "side":
                    kvflow.kv_pack_blocks(replica, pool, ids, stream=side)
            dec.run()
            if with_pack == "same":
                kvflow.kv_pack_blocks(replica, pool, ids)
            if with_pack == "tokens":
                kvflow.kv_gather_tokens(k_out, v_out, pool, dec.table, positions)
        if with_pack in ("side", "fork_only"):
            done = torch.cuda.Event()
            done.record(side)
            main.wait_event(done)
        t1.record(main)
        torch.cuda.synchronize()
        return t0.elapsed_time(t1) / n_iter

    train(5, "side")
    alone_ms = min(train(30, None) for _ in range(3))
    both_ms = min(train(30, "side") for _ in range(3))
    same_ms = min(train(30, "same") for _ in range(3))
    fork_ms = min(train(30, "fork_only") for _ in range(3))
    tok_ms = min(train(30, "tokens") for _ in range(3))
    o = {"ms_per_step_decode_only": alone_ms, "ms_per_step_with_pack_on_side_stream": both_ms,
         "ms_per_step_with_pack_on_same_stream": same_ms,
         "ms_per_step_with_token_rows_gathered_on_same_stream": tok_ms,
         "ms_per_step_with_the_fork_event_but_no_pack": fork_ms,
         "note": "eager launches; the side-stream figure includes one event record/wait per step between the two "
                 "streams, whose cost alone is the fork-event figure (it is paid once per fork, here once per "
                 "150 us decode call; a serving step forks once per token step of all layers)"}

    # The same three trains captured once into HIP graphs: the fork and join between the streams become graph
    # dependencies, so a replay makes no host-side event call.  `steps` steps per graph.
    def graph_train(with_pack, steps=20):
        cap, side2 = torch.cuda.Stream(), torch.cuda.Stream()
        cap.wait_stream(main)
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.stream(cap):
            with torch.cuda.graph(gr, stream=cap):
                for _ in range(steps):
                    if with_pack == "side":
                        side2.wait_stream(cap)
                        kvflow.kv_pack_blocks(replica, pool, ids, stream=side2)
                    dec.run(stream=cap)
                    if with_pack == "same":
                        kvflow.kv_pack_blocks(replica, pool, ids, stream=cap)
                    if with_pack == "side":
                        cap.wait_stream(side2)
        torch.cuda.synchronize()
        gr.replay()
        torch.cuda.synchronize()
        best = None
        for _ in range(5):
            t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            t0.record(main)
            gr.replay()
            t1.record(main)
            torch.cuda.synchronize()
            ms = t0.elapsed_time(t1) / steps
            best = ms if best is None else min(best, ms)
        return best

    graphs = None
    try:
        g_alone, g_side, g_same = graph_train(None), graph_train("side"), graph_train("same")
        graphs = {"ms_per_step_decode_only": g_alone, "ms_per_step_with_pack_on_side_stream": g_side,
                  "ms_per_step_with_pack_on_same_stream": g_same,
                  "side_stream_slowdown_pct": 100.0 * (g_side / g_alone - 1.0),
                  "same_stream_slowdown_pct": 100.0 * (g_same / g_alone - 1.0),
                  "added_traffic_pct": 100.0 * 2 * n * g.block_bytes / case.kv_bytes,
                  "note": "20 steps per graph; decode is bound by HBM bandwidth, so the pack's own read+write traffic "
                          "(added_traffic_pct of the decode's) is the floor of any slowdown"}
    except Exception as exc:                                  # capture across two streams is a convenience figure
        log(f"[bench] two-stream graph skipped: {exc}")
    # the on-device replication loop of one step: append the new tokens, collect the dirty list, pack it
    rs = np.random.SeedSequence(4242).spawn(2)
    k_new = bf16_dev(W.normal_bf16(rs[0], (case.batch, g.num_kv_heads, g.head_dim)))
    v_new = bf16_dev(W.normal_bf16(rs[1], (case.batch, g.num_kv_heads, g.head_dim)))
    bitmap = torch.zeros((case.num_blocks + 31) // 32, dtype=torch.int32, device="cuda")
    ids_dev = torch.empty(case.batch, dtype=torch.int32, device="cuda")
    cnt_dev = torch.zeros(1, dtype=torch.int32, device="cuda")
    a_t = time_calls(lambda: kvflow.kv_append_tokens(pool, k_new, v_new, dec.table, positions, bitmap), 20, 5)
    c_t = time_calls(lambda: kvflow.kv_collect_dirty(bitmap, case.num_blocks, ids_dev, cnt_dev, False), 20, 5)
    p_t = time_calls(lambda: kvflow.kv_pack_blocks_counted(replica, pool, ids_dev, cnt_dev), 20, 5)
    g_t = time_calls(lambda: kvflow.kv_gather_tokens(k_out, v_out, pool, dec.table, positions), 20, 5)
    loop = {"gather_tokens_us": g_t["mean_ms"] * 1e3,
            "bytes_per_step_block_granular": n * g.block_bytes,
            "bytes_per_step_token_granular": case.batch * g.kv_bytes_per_token,
            "append_us": a_t["mean_ms"] * 1e3, "collect_dirty_us": c_t["mean_ms"] * 1e3,
            "pack_counted_us": p_t["mean_ms"] * 1e3, "dirty_found": int(cnt_dev.item()),
            "note": "latency-bound helpers (KB to MB of traffic); times include launch and event overhead"}
    # pack into pinned host memory (a transport buffer on the far side of PCIe): rate, and what a
    # decode step costs while such a pack is running beside it.  The list is long enough (2048
    # blocks, 268 MB) for the pack to outlast the measured decode steps.
    n_host = min(2048, len(case.in_use_ids))
    host_ids = torch.from_numpy(case.in_use_ids[:n_host].copy()).cuda()
    host_replica = torch.empty((n_host,) + pool.shape[1:], dtype=torch.bfloat16).pin_memory()
    host_payload = n_host * g.block_bytes

    def decode_steps_beside(launch_pack, steps=40):
        """`steps` decode steps on the main stream while launch_pack() runs on the side stream.
        Returns (median ms of the steps after the first four, total ms of all steps, side-stream ms)."""
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        if launch_pack is not None:
            ev = torch.cuda.Event()
            ev.record(main)
            side.wait_event(ev)
            s0.record(side)
            launch_pack()
            s1.record(side)
        for i in range(steps):
            evs[i].record(main)
            dec.run()
        evs[steps].record(main)
        torch.cuda.synchronize()
        ms = [evs[i].elapsed_time(evs[i + 1]) for i in range(steps)]
        return float(np.median(ms[4:])), float(sum(ms)), (s0.elapsed_time(s1) if launch_pack is not None else 0.0)

    dev_staging = torch.empty((n_host,) + pool.shape[1:], dtype=torch.bfloat16, device="cuda")

    def direct():
        kvflow.kv_pack_blocks(host_replica, pool, host_ids, stream=side)

    def staged():
        kvflow.kv_pack_blocks(dev_staging, pool, host_ids, stream=side)
        with torch.cuda.stream(side):
            host_replica.copy_(dev_staging, non_blocking=True)       # DMA engine, not the compute units

    chunk_blocks = max(1, (32 << 20) // g.block_bytes)                  # two staging halves of 32 MiB
    small_staging = torch.empty((2 * chunk_blocks,) + pool.shape[1:], dtype=torch.bfloat16, device="cuda")
    copy_stream = torch.cuda.Stream()

    def double_buffered():
        copy_stream.wait_stream(side)
        kvflow.kv_pack_blocks_staged(host_replica, pool, host_ids, small_staging, chunk_blocks, side, copy_stream)
        side.wait_stream(copy_stream)                                   # the side-stream timer closes after the last copy

    host = {"blocks": n_host, "payload_MB": host_payload / 1e6, "decode_steps": 40,
            "double_buffer_staging_MB": 2 * chunk_blocks * g.block_bytes / 1e6}
    decode_steps_beside(None)
    base_med, base_sum, _ = decode_steps_beside(None)
    host["decode_alone"] = {"median_step_ms": base_med, "total_ms": base_sum}
    for label, fn in (("pack_kernel_writes_host_memory", direct), ("pack_to_device_staging_then_dma", staged),
                      ("pack_staged_double_buffered", double_buffered)):
        decode_steps_beside(fn)
        med, tot, side_ms = decode_steps_beside(fn)
        host[label] = {"transfer_ms": side_ms, "payload_GBps": host_payload / (side_ms * 1e-3) / 1e9,
                       "median_step_ms_meanwhile": med, "steady_slowdown_pct": 100.0 * (med / base_med - 1.0),
                       "total_delay_of_the_steps_ms": tot - base_sum}
    kv = case.kv_bytes
    return {
        "kv_GB": kv / 1e9, "dirty_blocks": n, "replication_loop": loop, "pack_to_host": host, "pack_payload_MB": n * g.block_bytes / 1e6,
        "workgroups": dec.workgroups,
        "decode_alone": {**d, "kv_GBps": kv / (d["mean_ms"] * 1e-3) / 1e9,
                         "frac_hbm_peak": kv / (d["mean_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS},
        "pack_alone": {**p, **copy_rates(n * g.block_bytes, p["mean_ms"])},
        "back_to_back_steps": o,
        "back_to_back_steps_replayed_from_hip_graphs": graphs,
        "decode_slowdown_pct": 100.0 * (both_ms / alone_ms - 1.0),
        "same_stream_slowdown_pct": 100.0 * (same_ms / alone_ms - 1.0),
        "fork_event_alone_slowdown_pct": 100.0 * (fork_ms / alone_ms - 1.0),
        "token_rows_same_stream_slowdown_pct": 100.0 * (tok_ms / alone_ms - 1.0),
        "added_traffic_floor_pct": 100.0 * 2 * n * g.block_bytes / case.kv_bytes,
    }


def bench_long_context_fp8(args, kvflow, W):
    """The timed workload's decode again with an FP8 (E4M3) pool: half the KV bytes per token."""
    import torch
    case = W.long_context(kv_elt_bytes=1)
    pool = kvflow.Fp8Pool(torch.from_numpy(case.pool).cuda(), W.FP8_KV_SCALE, W.FP8_KV_SCALE)
    dec = Decode(case, pool, kvflow)
    d = time_calls(dec.run, 50, 10)
    kv = case.kv_bytes
    return {"kv_GB": kv / 1e9, "workgroups": dec.workgroups, **d, "kv_GBps": kv / (d["mean_ms"] * 1e-3) / 1e9,
            "frac_hbm_peak": kv / (d["mean_ms"] * 1e-3) / 1e9 / HBM_PEAK_GBPS,
            "tokens_per_s": float(case.context_lens.sum()) / (d["mean_ms"] * 1e-3)}


def bench_llama_layer(args, kvflow, W):
    case = W.llama8b_layer()
    pool = bf16_dev(case.pool)
    dec = Decode(case, pool, kvflow)
    d = time_calls(dec.run, 50, 10)
    kv = case.kv_bytes
    return {"kv_GB": kv / 1e9, "workgroups": dec.workgroups, **d,
            "kv_GBps": kv / (d["mean_ms"] * 1e-3) / 1e9,
            "note": "working set near the last-level cache size: latency figure, not an HBM measurement"}


def bench_recompute(args, kvflow, W):
    """Recomputation (causal prefill over the paged pool): whole sequences, and a 2048-token chunk over a
    long restored prefix.  A dense contraction: reported against the bf16 matrix-core peak; flops count the
    (query, key) pairs inside the causal mask only."""
    import torch
    out = {}
    for label, maker in (("recompute", W.recompute), ("chunked_recompute", W.chunked_recompute),
                         ("recompute_fp8_pool", lambda: W.recompute(kv_elt_bytes=1)),
                         ("short_chunk", W.short_chunk_recompute)):
        case = maker()
        kv, g = case.kv, case.geom
        q = torch.from_numpy(case.q.view(np.int16)).cuda().view(torch.bfloat16)
        if kv.pool.dtype == np.uint8:
            pool = kvflow.Fp8Pool(torch.from_numpy(kv.pool).cuda(), W.FP8_KV_SCALE, W.FP8_KV_SCALE)
        else:
            pool = torch.from_numpy(kv.pool.view(np.int16)).cuda().view(torch.bfloat16)
        table = torch.from_numpy(kv.block_table).cuda()
        lens = torch.from_numpy(kv.context_lens).cuda()
        starts = torch.from_numpy(case.q_starts).cuda()
        o = torch.empty((case.total_q, g.num_q_heads, g.head_dim), dtype=torch.bfloat16, device="cuda")
        ks = kvflow.kv_prefill_key_splits(case.batch, g.num_q_heads, g.num_kv_heads, case.max_q_len,
                                          kv.max_context_len)
        nbytes = kvflow.kv_prefill_workspace_bytes(case.total_q, g.num_q_heads, g.head_dim, ks)
        ws = torch.empty(max(nbytes, 4) // 4, dtype=torch.float32, device="cuda")
        d = time_calls(lambda: kvflow.kv_prefill_attn(o, q, pool, table, lens, starts, case.max_q_len, float(g.scale),
                                                      ks, ws), 20, 5)
        tflops = case.flops / (d["mean_ms"] * 1e-3) / 1e12
        out[label] = {
            "context_lens": kv.context_lens.tolist(), "q_lens": case.q_lens.tolist(),
            "flops_in_mask": case.flops, "key_splits": ks, **d, "TFLOPps": tflops,
            "roofline": {"bound": "mfma", "kernel": f"prefill_kernel<128, 2, {str(kv.pool.dtype == np.uint8).lower()}>",
                         "achieved": tflops,
                         "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tflops / MFMA_BF16_PEAK_TFLOPS,
                         "traffic": None},
            "query_tokens_per_s": case.total_q / (d["mean_ms"] * 1e-3),
        }
        del q, pool, o
        torch.cuda.empty_cache()
    return out


def bench_yardsticks(args, kvflow, W):
    """What plain streaming kernels reach on this device: the practical ceilings next to the 8 TB/s peak.
    Three designs of each: the library's two probe kernels and torch's own fill / copy / sum-free read."""
    import torch
    nbytes = 4 << 30
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    b = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    b.random_(0, 255)
    sink = torch.zeros(16, dtype=torch.uint8, device="cuda")
    out = {"bytes": nbytes}
    a32, b32 = a.view(torch.int32), b.view(torch.int32)
    runs = (
        ("read_only", lambda: kvflow.kv_probe_stream(0, sink, b, nbytes), nbytes),
        ("write_only", lambda: kvflow.kv_probe_stream(1, a, None, nbytes), nbytes),
        ("contiguous_copy", lambda: kvflow.kv_probe_stream(2, a, b, nbytes), 2 * nbytes),
        ("read_only_second_design", lambda: kvflow.kv_probe_stream(3, sink, b, nbytes), nbytes),
        ("write_only_second_design", lambda: kvflow.kv_probe_stream(4, a, None, nbytes), nbytes),
        ("contiguous_copy_second_design", lambda: kvflow.kv_probe_stream(5, a, b, nbytes), 2 * nbytes),
        ("write_only_torch_fill", lambda: a32.fill_(7), nbytes),
        ("contiguous_copy_torch", lambda: a32.copy_(b32), 2 * nbytes),
    )
    for name, fn, traffic in runs:
        d = time_calls(fn, 10, 3)
        gbps = traffic / (d["mean_ms"] * 1e-3) / 1e9
        out[name] = {**d, "traffic_GBps": gbps, "frac_hbm_peak": gbps / HBM_PEAK_GBPS}
    del a, b, a32, b32
    torch.cuda.empty_cache()
    out["matrix_core"] = bench_matrix_yardsticks(kvflow)
    return out


def bench_matrix_yardsticks(kvflow):
    """What bounds the recomputation kernel: the MFMA rate on registers alone with zero and with random operands
    (the device lowers its clock under random data), the vector work of a softmax step, and how much of it
    hides under the matrix work of the wavefront that shares the SIMD."""
    import torch
    sink = torch.empty(kvflow.KV_PROBE_MATRIX_SINK_BYTES // 4, dtype=torch.float32, device="cuda")
    iters = 20000
    waves, mfma_per_block = 256 * 8, 32
    res = {"iterations": iters,
           "blocks": "matrix block = 32 MFMA 16x16x32 bf16 on registers; vector block = 80 fma + 16 exp2; "
                     "256 workgroups of 8 wavefronts, wavefronts w and w + 4 share a SIMD"}
    cyc = lambda ms: ms * 1e-3 * 2.4e9 / iters           # cycles per iteration at the nominal 2.4 GHz
    for mode, name, active_waves in ((0, "matrix_only_zero_operands", waves), (1, "matrix_only_random_operands", waves),
                                     (4, "matrix_on_half_the_wavefronts_partners_idle", waves // 2)):
        d = time_calls(lambda: kvflow.kv_probe_matrix(mode, iters, sink), 5, 2)
        tflops = active_waves * iters * mfma_per_block * 16384 / (d["mean_ms"] * 1e-3) / 1e12
        res[name] = {"mean_ms": d["mean_ms"], "TFLOPps": tflops, "frac_mfma_peak": tflops / MFMA_BF16_PEAK_TFLOPS,
                     "cycles_per_iteration_at_2p4GHz": cyc(d["mean_ms"])}
    for mode, name in ((2, "vector_only_all_wavefronts"), (5, "vector_on_half_the_wavefronts_partners_idle"),
                       (3, "matrix_wavefronts_beside_vector_partners")):
        d = time_calls(lambda: kvflow.kv_probe_matrix(mode, iters, sink), 5, 2)
        res[name] = {"mean_ms": d["mean_ms"], "cycles_per_iteration_at_2p4GHz": cyc(d["mean_ms"])}
    m, v = (res["matrix_on_half_the_wavefronts_partners_idle"]["cycles_per_iteration_at_2p4GHz"],
            res["vector_on_half_the_wavefronts_partners_idle"]["cycles_per_iteration_at_2p4GHz"])
    both = res["matrix_wavefronts_beside_vector_partners"]["cycles_per_iteration_at_2p4GHz"]
    res["vector_work_hidden_under_matrix_work_frac"] = (m + v - both) / min(m, v)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--copy-iters", type=int, default=5)
    ap.add_argument("--recovery-blocks", type=int, default=200_000)
    ap.add_argument("--only-timed", action="store_true", help="skip the extra cases and the CPU baseline")
    ap.add_argument("--extras", default="yardsticks,replication_mix,long_context_fp8_pool,llama8b_layer,recovery,recompute",
                    help="comma-separated extra cases to run after the timed workload")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after timing, run one plain device copy of the pool (known size) so that a "
                         "counter-collecting profiler run has a yardstick for FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU only: this data path uses no second GPU; run with --gpus 1")

    import torch
    from paper_2601_22438_amd import kvflow
    from paper_2601_22438_amd import workloads as W
    kvflow.load()                                     # fails loudly when the HIP library is missing
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)

    main_res = bench_long_context(args, kvflow, W)
    case = main_res["case"]
    g = case.geom
    d = main_res["decode"]
    achieved = main_res["decode_GBps"]
    # everything the decode kernels are built from: their sources, the shared constants, the compile flags
    src = b"".join(open(os.path.join(ROOT, "paper_2601_22438_amd", f), "rb").read()
                   for f in ("csrc/kv_decode.hip", "csrc/kv_decode_common.h", "csrc/kv_internal.h", "build.py"))
    traffic = None
    if DECODE_TRAFFIC["kernel_sha256"] == hashlib.sha256(src).hexdigest():
        traffic = DECODE_TRAFFIC["fetch_bytes"] + DECODE_TRAFFIC["write_bytes"]
    roofline = {"bound": "hbm", "kernel": "decode_partition_kernel<128> + decode_merge_kernel<128> (one decode call)",
                "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBPS, "traffic": traffic,
                "algorithmic_bytes_per_launch": main_res["kv_bytes"], "mean_launch_ms": d["mean_ms"]}
    extra = {
        "timed_workload": {
            "decode": {**d, "kv_GBps": achieved, "frac_hbm_peak": achieved / HBM_PEAK_GBPS,
                       "tokens_per_s": float(case.context_lens.sum()) / (d["mean_ms"] * 1e-3),
                       "workgroups": main_res["dec"].workgroups},
            "pack": {**main_res["pack"], **copy_rates(main_res["payload"], main_res["pack"]["mean_ms"])},
            "restore": {**main_res["restore"], **copy_rates(main_res["payload"], main_res["restore"]["mean_ms"])},
            "dirty_blocks": len(case.dirty_ids), "payload_MB": main_res["payload"] / 1e6,
            "ms_per_step_replayed_from_a_hip_graph": main_res["graph_ms_per_step"],
        },
        "paper_context": PAPER_CONTEXT,
    }
    cpu = parity = None
    if not args.only_timed:
        import oracle
        oracle.build()
        want_out, want_replica, cpu = cpu_baseline(case, oracle)
        log(f"[bench] cpu baseline done: {cpu['value']:.3f} GB/s on {cpu['cores']} threads")
        parity = parity_of_timed_buffers(case, main_res["written"], want_out, want_replica, oracle)
        log(f"[bench] parity of the timed buffers: {parity}")
        if not (parity["decode_max_abs"] <= 2e-2 and parity["decode_mean_abs"] <= 2e-3 and parity["decode_finite"]
                and parity["pack_bit_exact"] and parity["restore_bit_exact"]):
            sys.exit(f"bench.py: the timed steps' results do not match the oracle: {parity}")
    if args.calibration_copy:
        src_pool = main_res["pool"]
        dst_pool = torch.empty_like(src_pool)
        dst_pool.copy_(src_pool)
        torch.cuda.synchronize()
        extra["calibration_copy_bytes"] = src_pool.numel() * 2
        del dst_pool
    # free the timed workload before the large cases
    for k in ("dec", "pool", "ids", "replica", "written"):
        main_res.pop(k)
    torch.cuda.empty_cache()
    if not args.only_timed:
        runners = {
            "yardsticks": lambda: bench_yardsticks(args, kvflow, W),
            "replication_mix": lambda: bench_replication_mix(args, kvflow, W),
            "long_context_fp8_pool": lambda: bench_long_context_fp8(args, kvflow, W),
            "llama8b_layer": lambda: bench_llama_layer(args, kvflow, W),
            "recovery": lambda: bench_recovery(args, kvflow, W, args.recovery_blocks),
            "recompute": lambda: bench_recompute(args, kvflow, W),
        }
        for name in [x for x in args.extras.split(",") if x]:
            if name not in runners:
                sys.exit(f"unknown extra case {name!r}; known: {', '.join(runners)}")
            extra[name] = runners[name]()
            log(f"[bench] {name} done")
            torch.cuda.empty_cache()

    line = {
        "metric": "paged decode KV GB/s (pack/restore GB/s under extra), % of HBM peak, 1 MI355X",
        "value": achieved, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": main_res["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "long_context: batch 8, 32 query heads, 8 KV heads, head_dim 128, block_size 16, "
                               "context lengths uniform in [16384, 65536] (seed 2), pool 1.25x needed blocks with "
                               "shuffled block tables; step = decode, pack 10% of in-use blocks, restore them",
                   "kv_bytes_per_step": main_res["kv_bytes"], "pack_payload_bytes": main_res["payload"]},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity": parity,
        "extra": extra,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
