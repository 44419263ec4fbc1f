#!/usr/bin/env python3
"""Benchmark of the decode-attention hot path on one MI355X.

Workload (the configuration the metric is quoted on): Llama-3.2-3B attention
layer shape, bf16 -- batch 16, 24 query heads, 8 key/value heads, head_dim 128,
key/value blocks of 256 -- causal decode at step t = 4095.  One "step" is one
pass of the whole path for one layer through tempo_decode_step_causal: the
block-store write of step t's key/value, partial attention over keys 0..t, and
the split combine.  (The same step through the separate entry points
tempo_kv_append + tempo_attn_decode_causal is timed too and reported as
"separate_calls".)  Successive steps rotate over several layers' pools (a decode
step of a real model visits every layer's keys/values once), so the key/value
bytes of a step are not left in the last-level cache by the previous one (4 to 8
pools of 256 MiB: no more than the warm-up steps, so that warm-up visits each once).

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Prints ONE JSON line.  Timing protocol: W untimed warm-up steps, then exactly K
steps issued back to back on the launch stream with a HIP event recorded every few
steps (GPU timestamps on that stream, so the host's final synchronize is not in the
figure and the result does not move with K).  ms_per_step is the MEDIAN over those
chunks of (chunk time / steps in the chunk); the mean over all K steps, the fastest
chunk and the host wall-clock mean are reported beside it.  value = key/value GB/s =
algorithmic key/value bytes read per step (batch * (t+1) * 2 * Hkv * D * 2 bytes) /
ms_per_step, inputs resident in HBM.  "roofline" prices the dominant kernel (partial
attention) against the 8 TB/s HBM peak from its own HIP-event-timed launches inside
the same run; "cpu_baseline" is the fp64 oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0

# HBM bytes per launch of the partial-attention kernel at the benchmark workload come from the
# committed counter summary (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of `bench.py --counters`,
# each scaled by what the same counter reads for the 256 MiB copy kernel); the line
# "traffic_bytes_per_launch = N" of that file is what "roofline.traffic" reports.
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "attn_partial_bf16_llama_t4095_hbm_traffic.txt")


def measured_traffic_bytes():
    try:
        with open(TRAFFIC_PROFILE) as f:
            m = re.search(r"^traffic_bytes_per_launch\s*=\s*(\d+)", f.read(), re.M)
        return int(m.group(1)) if m else None
    except OSError:
        return None


def gpu_timed(torch, fn, n, warm, chunk=None):
    """`warm` untimed calls fn(i), then exactly n calls back to back on the current stream, with
    a HIP event recorded on that stream before the first call and after every `chunk` calls.
    Returns per-call seconds: median and min over the chunks, mean over all n calls (first to
    last event), and the host wall-clock mean around a final synchronize."""
    if chunk is None:
        chunk = 10 if n >= 100 else max(1, n // 4)
    for i in range(warm):
        fn(i)
    bounds = list(range(0, n, chunk)) + [n]
    events = [torch.cuda.Event(enable_timing=True) for _ in bounds]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    events[0].record()
    k = 1
    for i in range(n):
        fn(i)
        if i + 1 == bounds[k]:
            events[k].record()
            k += 1
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / n
    in_order = [events[j].elapsed_time(events[j + 1]) * 1e-3 / (bounds[j + 1] - bounds[j])
                for j in range(len(bounds) - 1)]
    per_call = sorted(in_order)
    mean = events[0].elapsed_time(events[-1]) * 1e-3 / n
    return {"median": per_call[len(per_call) // 2] if len(per_call) % 2 else
            0.5 * (per_call[len(per_call) // 2 - 1] + per_call[len(per_call) // 2]),
            "min": per_call[0], "mean": mean, "wall": wall, "chunk": chunk, "chunks": len(per_call),
            "first_chunks": in_order[:8]}


def graph_timed(torch, fn, group, replays, warm=3):
    """Capture `group` consecutive calls fn(0) .. fn(group-1) in one HIP graph and replay it;
    an event pair around every replay.  Returns per-call seconds (median and min over replays)."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for i in range(group):
            fn(i)                                         # warm-up on a capture-capable stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(group):
            fn(i)
    for _ in range(warm):
        graph.replay()
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(replays)]
    torch.cuda.synchronize()
    for a, b in pairs:
        a.record()
        graph.replay()
        b.record()
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) * 1e-3 / group for a, b in pairs)
    return {"median": ts[len(ts) // 2], "min": ts[0]}


def hbm_roofline(kernel, nbytes, seconds, what="whole call (all launches of the step)"):
    gbs = nbytes / seconds / 1e9
    return {"kernel": kernel, "bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(gbs / HBM_PEAK_GBS, 4), "timed": what}


def us(x):
    return round(x * 1e6, 2)


def launch_bound_legs(torch, T, BlockStore, synth, dev, kv_bytes_per_token):
    """The regimes where the fixed cost of a launch shows (short causal ranges, the 512-key window,
    one long sequence): the step issued eagerly (one C-ABI call per step from Python) and replayed
    from a HIP graph of 16 steps over 8 rotated layer pools.  Ideal = bytes / 8 TB/s."""
    Hq, Hkv, D, Z, R = 24, 8, 128, 256, 8
    out = {}
    q16 = synth.device_normal((16, Hq, D), 71, torch.bfloat16, dev)
    k16 = synth.device_normal((16, Hkv, D), 72, torch.bfloat16, dev)
    v16 = synth.device_normal((16, Hkv, D), 73, torch.bfloat16, dev)

    def layers(batch, max_t, ring=0):
        sts = []
        for _ in range(R):
            st = BlockStore(batch, Hq, Hkv, D, Z, max_t, T.TEMPO_BF16, device=dev, ring_blocks=ring)
            st.k_pool.normal_()
            st.v_pool.normal_()
            sts.append(st)
        return sts

    def leg(name, fn, nbytes, plan):
        eager = gpu_timed(torch, fn, 200, 20)
        graph = graph_timed(torch, fn, 16, 30)
        best = min(eager["median"], graph["median"])
        out[name] = {"eager_us_per_step": us(eager["median"]), "graph_us_per_step": us(graph["median"]),
                     "graph_min_us": us(graph["min"]), "ideal_us": us(nbytes / (HBM_PEAK_GBS * 1e9)),
                     "kv_bytes_per_step": nbytes, "splits": plan.num_splits,
                     "tokens_per_split": plan.tokens_per_split, "waves": plan.waves,
                     "roofline": hbm_roofline("attn_partial_bf16<128, false>", nbytes, best,
                                              "whole step, the faster of eager and graph replay")}

    sts = layers(16, 4095)
    o = sts[0].new_out()
    for t in (255, 511, 1023, 2047):
        leg(f"causal_b16_t{t}", lambda i: sts[i % R].step_causal(q16, k16, v16, o, t), 16 * (t + 1) * kv_bytes_per_token,
            T.tempo_attn_plan(sts[0].kv, 16, Hq, t, 0))
    del sts
    torch.cuda.empty_cache()
    # the other head size (32 query heads in groups of 4, head_dim 64: half the bytes per key)
    sts64 = []
    for _ in range(R):
        st = BlockStore(16, 32, 8, 64, Z, 8191, T.TEMPO_BF16, device=dev)
        st.k_pool.normal_()
        st.v_pool.normal_()
        sts64.append(st)
    q64 = synth.device_normal((16, 32, 64), 74, torch.bfloat16, dev)
    k64 = synth.device_normal((16, 8, 64), 75, torch.bfloat16, dev)
    v64 = synth.device_normal((16, 8, 64), 76, torch.bfloat16, dev)
    o64 = sts64[0].new_out()
    for t in (4095, 8191):
        leg(f"head_dim64_hq32_b16_t{t}", lambda i: sts64[i % R].step_causal(q64, k64, v64, o64, t),
            16 * (t + 1) * 2 * 8 * 64 * 2, T.tempo_attn_plan(sts64[0].kv, 16, 32, t, 0))
        out[f"head_dim64_hq32_b16_t{t}"]["roofline"]["kernel"] = "attn_partial_bf16<64, false>"
    del sts64
    torch.cuda.empty_cache()
    sts = layers(16, 16383)
    leg("window512_b16_t8191", lambda i: sts[i % R].step_window(q16, k16, v16, o, 8191, 512),
        16 * 512 * kv_bytes_per_token, T.tempo_attn_plan(sts[0].kv, 16, Hq, 8191, 512))
    del sts
    torch.cuda.empty_cache()
    # the window store: every sequence of every layer owns a ring of 4 blocks, drawn at random from ONE pool
    # that holds exactly those rings (8 layers x 16 sequences x 4 blocks), as an allocator would hand them out
    ring_perm = synth.permutation(31, 1, R * 16 * 4)
    ring_k = torch.empty((R * 16 * 4, Hkv, Z * D), dtype=torch.bfloat16, device=dev).normal_()
    ring_v = torch.empty((R * 16 * 4, Hkv, Z * D), dtype=torch.bfloat16, device=dev).normal_()
    sts = [BlockStore(16, Hq, Hkv, D, Z, 2 ** 30, T.TEMPO_BF16, device=dev, ring_blocks=4, num_blocks=R * 16 * 4,
                      block_table=torch.from_numpy(ring_perm[l * 64:(l + 1) * 64].reshape(16, 4).copy()),
                      pools=(ring_k, ring_v)) for l in range(R)]
    leg("window512_ring4_b16_t1000000", lambda i: sts[i % R].step_window(q16, k16, v16, o, 1000000, 512),
        16 * 512 * kv_bytes_per_token, T.tempo_attn_plan(sts[0].kv, 16, Hq, 1000000, 512))
    out["window512_ring4_b16_t1000000"]["pool_mib_per_layer"] = round(2 * ring_k.numel() * 2 / R / 2 ** 20, 1)
    out["window512_ring4_b16_t1000000"]["linear_store_would_need_mib"] = round(
        16 * (1000000 // Z + 1) * Hkv * Z * D * 2 * 2 / 2 ** 20, 1)
    del sts, ring_k, ring_v
    torch.cuda.empty_cache()
    sts = layers(1, 65535)
    q1, k1, v1 = q16[:1].contiguous(), k16[:1].contiguous(), v16[:1].contiguous()
    o1 = sts[0].new_out()
    for t in (8191, 32767, 65535):
        plan = T.tempo_attn_plan(sts[0].kv, 1, Hq, t, 0)
        leg(f"long_b1_t{t}", lambda i: sts[i % R].step_causal(q1, k1, v1, o1, t), (t + 1) * kv_bytes_per_token, plan)
        out[f"long_b1_t{t}"]["work_items"] = plan.num_splits * Hkv
    del sts
    torch.cuda.empty_cache()
    return out


def whole_run_rotated(torch, T, BlockStore, synth, dev, kv_bytes_per_token):
    """The whole causal decode t = 0 .. 4095 of 8 layers, as a decoder runs it: at every step, one
    fused call (append + attention) per layer, each on its own pool, so no step finds its bytes in
    the last-level cache.  8 x 4096 calls; aggregate = all key/value bytes read / GPU time."""
    B, Hq, Hkv, D, Z, T_len, R = 16, 24, 8, 128, 256, 4096, 8
    sts = [BlockStore(B, Hq, Hkv, D, Z, T_len - 1, T.TEMPO_BF16, device=dev) for _ in range(R)]
    q = synth.device_normal((B, Hq, D), 91, torch.bfloat16, dev)
    Kt = synth.device_normal((T_len, B, Hkv, D), 92, torch.bfloat16, dev)
    Vt = synth.device_normal((T_len, B, Hkv, D), 93, torch.bfloat16, dev)
    outs = [st.new_out() for st in sts]
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    c0 = time.perf_counter()
    e0.record()
    for t in range(T_len):
        k_t, v_t = Kt[t], Vt[t]
        for r in range(R):
            sts[r].step_causal(q, k_t, v_t, outs[r], t)
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - c0
    gpu = e0.elapsed_time(e1) * 1e-3
    total_bytes = R * B * kv_bytes_per_token * T_len * (T_len + 1) // 2
    return {"layer_steps": R * T_len, "gpu_seconds": round(gpu, 4), "wall_seconds": round(wall, 4),
            "layer_steps_per_s": round(R * T_len / gpu, 1), "kv_gbs": round(total_bytes / gpu / 1e9, 1),
            "pct_of_hbm_peak": round(100.0 * total_bytes / gpu / 1e9 / HBM_PEAK_GBS, 2),
            "note": "t = 0..4095, 8 layer pools visited at every step (real per-step appends); GPU time "
                    "between two events around all 32768 calls, issued from Python one C-ABI call each"}


def other_workloads(torch, T, BlockStore, synth, dev, kv_bytes_per_token):
    """Blocks of queries, the prompt, the rotary producer and the ragged 28-layer step, at their real
    shapes.  Pools are filled directly with N(0,1) (any layout of i.i.d. values is i.i.d.), fresh
    keys/values are appended by the step itself; each step visits a different layer's pool."""
    Hq, Hkv, D, Z = 24, 8, 128, 256
    out = {}
    q16 = synth.device_normal((16, Hq, D), 71, torch.bfloat16, dev)
    k16 = synth.device_normal((16, Hkv, D), 72, torch.bfloat16, dev)
    v16 = synth.device_normal((16, Hkv, D), 73, torch.bfloat16, dev)

    def layers(n, batch, max_t):
        sts = []
        for layer in range(n):
            st = BlockStore(batch, Hq, Hkv, D, Z, max_t, T.TEMPO_BF16, device=dev)
            st.k_pool.normal_()
            st.v_pool.normal_()
            sts.append(st)
        return sts

    # blocks of query steps over the headline shape: append C steps, then one attention call answers
    # steps 4096-C .. 4095.  5 steps (15 of the 16 tile columns) ride in the single-step kernel;
    # 10, 21 and 42 steps (30, 63 and 126 columns) go through the LDS-staged kernel.
    sts = layers(8, 16, 4095)
    block_bytes = 16 * 4096 * kv_bytes_per_token
    for C in (5, 10, 21, 42):
        qc = synth.device_normal((16, C, Hq, D), 177, torch.bfloat16, dev)
        kc = synth.device_normal((16, C, Hkv, D), 178, torch.bfloat16, dev)
        vc = synth.device_normal((16, C, Hkv, D), 179, torch.bfloat16, dev)
        oc = torch.empty_like(qc)

        def block_step(i):
            sts[i % 8].append_block(kc, vc, 4096 - C, C)
            sts[i % 8].attend_block(qc, oc, 4096 - C, C)

        dt = gpu_timed(torch, block_step, 200, 20)["median"]
        plan = T.tempo_attn_block_plan(sts[0].kv, 16, Hq, C, 4096 - C, 0)
        kernel = "attn_partial_bf16<128, false>" if C * (Hq // Hkv) <= 16 else "attn_prefill_bf16<128, NW, false, true>"
        out[f"block{C}_b16_t{4096 - C}"] = {"us_per_call": us(dt), "us_per_query_step": us(dt / C),
                                            "kv_gbs": round(block_bytes / dt / 1e9, 1),
                                            "splits": plan.num_splits, "tokens_per_split": plan.tokens_per_split,
                                            "waves": plan.waves,
                                            "roofline": hbm_roofline(kernel, block_bytes, dt,
                                                                     "whole call: block-store write + attention + combine")}
    # prompt processing: 4096 steps of 16 sequences in one tempo_prefill_causal call
    P = 4096
    qp = synth.device_normal((16, P, Hq, D), 277, torch.bfloat16, dev)
    kp = synth.device_normal((16, P, Hkv, D), 278, torch.bfloat16, dev)
    vp = synth.device_normal((16, P, Hkv, D), 279, torch.bfloat16, dev)
    op = torch.empty_like(qp)
    dt = gpu_timed(torch, lambda i: sts[i % 8].prefill_attend(qp, kp, vp, op, 0, P), 6, 2, chunk=1)["median"]
    pairs = P * (P + 1) // 2                                             # (query, key) pairs per sequence
    tflops = 16 * pairs * 4 * D * Hq / dt / 1e12
    out["prompt_b16_t4096"] = {"ms": round(dt * 1e3, 3), "tokens_per_s": round(16 * P / dt, 1),
                               "tflops": round(tflops, 1),
                               "roofline": {"kernel": "attn_prefill_bf16<128, 8, false, false>", "bound": "mfma",
                                            "achieved": round(tflops, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                                            "unit": "TFLOP/s", "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4)},
                               "note": "one tempo_prefill_causal call (block-store write + prompt kernel); "
                                       "algorithmic flops = 4*D*Hq per visible (query, key) pair, whole call timed"}
    del qp, kp, vp, op
    del sts
    torch.cuda.empty_cache()

    # producer fused in: unrotated q and k in, rotary embedding + block-store write + attention
    # in the launches of the plain step, against the same work as separate launches
    sts = layers(8, 16, 4095)
    ang = torch.arange(4096, device=dev, dtype=torch.float64)[:, None] * \
        (500000.0 ** (-torch.arange(0, D, 2, device=dev, dtype=torch.float64) / D))[None, :]
    cos_t, sin_t = torch.cos(ang).float().contiguous(), torch.sin(ang).float().contiguous()
    for st in sts:
        st.set_rope(cos_t, sin_t)
    o = sts[0].new_out()
    qr = torch.empty_like(q16)
    dt = gpu_timed(torch, lambda i: sts[i % 8].rope_step(q16, k16, v16, o, 4095), 200, 20)["median"]

    def rope_separate(i):
        st = sts[i % 8]
        st.rope_rotate(q16, qr, 4095)
        st.rope_append(k16, v16, 4095)
        st.attend_causal(qr, o, 4095)

    dt3 = gpu_timed(torch, rope_separate, 200, 20)["median"]
    out["rope_step_b16_t4095"] = {"us_per_step": us(dt), "kv_gbs": round(block_bytes / dt / 1e9, 1),
                                  "separate_launches_us": us(dt3),
                                  "roofline": hbm_roofline("attn_partial_bf16<128, true>", block_bytes, dt),
                                  "note": "fused: rotate q,k + append + attend in 2 launches; separate: 4 launches"}
    # the same for a block of 21 steps: one rotating block write + one block call with raw queries
    C = 21
    qc = synth.device_normal((16, C, Hq, D), 277, torch.bfloat16, dev)
    kc = synth.device_normal((16, C, Hkv, D), 278, torch.bfloat16, dev)
    vc = synth.device_normal((16, C, Hkv, D), 279, torch.bfloat16, dev)
    oc = torch.empty_like(qc)

    def rope_block(i):
        sts[i % 8].rope_append_block(kc, vc, 4096 - C, C)
        sts[i % 8].attend_block(qc, oc, 4096 - C, C, rope=True)

    dt = gpu_timed(torch, rope_block, 200, 20)["median"]
    out[f"rope_block{C}_b16_t{4096 - C}"] = {"us_per_call": us(dt), "us_per_query_step": us(dt / C),
                                             "roofline": hbm_roofline("attn_prefill_bf16<128, 4, true, true>", block_bytes, dt),
                                             "note": "rotating block write + block attention with unrotated queries"}
    del qc, kc, vc, oc
    del sts
    torch.cuda.empty_cache()

    out["ragged_28layers_b64"] = ragged_step_bench(torch, T, BlockStore, synth, dev, kv_bytes_per_token)

    # the anti-causal window reduction of the paper's reinforcement-learning example (Section 3,
    # Algorithm 1): returns over t : min(t+5, T) and over t : T, batch 64, T = 200 and 1000
    for T_len in (200, 1000):
        r = torch.empty((64, T_len), dtype=torch.float32, device=dev).normal_()
        g = torch.empty_like(r)
        for n in (5, 0):
            dt = graph_timed(torch, lambda i: T.tempo_discounted_sum(r, g, 64, T_len, n, 0.95), 16, 30)["median"]
            nbytes = 2 * r.numel() * 4
            out[f"discounted_sum_b64_T{T_len}_{'future' if n == 0 else 'n' + str(n)}"] = {
                "us_per_call": us(dt), "bytes_per_call": nbytes,
                "roofline": dict(hbm_roofline("discounted_suffix" if n == 0 else "discounted_window", nbytes, dt,
                                              "one launch, graph replay"),
                                 note="a few hundred KB per call: bound by launch latency (an empty kernel's "
                                      "period is 1.9 us), not by HBM")}
    return out


def ragged_step_bench(torch, T, BlockStore, synth, dev, kv_bytes_per_token, repeats=10):
    """Ragged multi-layer decode step: 28 layers, batch 64, lengths uniform in [1, 8192], one shared
    pool with exactly the blocks the sequences need, a random block table per layer; one step = per
    layer one fused call (block-store write + attention over each sequence's own range)."""
    import numpy as np
    Hq, Hkv, D, Z = 24, 8, 128, 256
    n_layers, B = 28, 64
    lengths = synth.integers(24, 1, B, 1, 8192)
    need = (lengths.astype(np.int64) + Z - 1) // Z                       # blocks per sequence
    per_layer = int(need.sum())
    nb = n_layers * per_layer
    k_pool = torch.empty((nb, Hkv, Z * D), dtype=torch.bfloat16, device=dev).normal_()
    v_pool = torch.empty((nb, Hkv, Z * D), dtype=torch.bfloat16, device=dev).normal_()
    perm = synth.permutation(24, 2, nb)
    sts = []
    for layer in range(n_layers):
        table = np.zeros((B, 8192 // Z), dtype=np.int32)
        ids = perm[layer * per_layer:(layer + 1) * per_layer]
        pos = 0
        for b in range(B):
            table[b, :need[b]] = ids[pos:pos + need[b]]
            pos += int(need[b])
        sts.append(BlockStore(B, Hq, Hkv, D, Z, 8191, T.TEMPO_BF16, device=dev, num_blocks=nb,
                              block_table=torch.from_numpy(table), pools=(k_pool, v_pool)))
    tps = torch.from_numpy(lengths - 1).to(dev).to(torch.int32)
    q64 = synth.device_normal((B, Hq, D), 74, torch.bfloat16, dev)
    k64 = synth.device_normal((B, Hkv, D), 75, torch.bfloat16, dev)
    v64 = synth.device_normal((B, Hkv, D), 76, torch.bfloat16, dev)
    o = sts[0].new_out()

    def ragged_step(_):
        for st in sts:
            st.step_causal(q64, k64, v64, o, 8191, t_per_seq=tps)

    def ragged_step_listed(_):
        # the work list depends on the steps only: built once per decode step, used by all 28 layers
        worklist = sts[0].build_worklist(8191, tps)
        for st in sts:
            st.step_ragged(q64, k64, v64, o, 8191, tps, worklist)

    dense = gpu_timed(torch, ragged_step, repeats, 2, chunk=1)["median"]
    listed = gpu_timed(torch, ragged_step_listed, repeats, 2, chunk=1)["median"]
    dt = min(dense, listed)
    gdt = graph_timed(torch, ragged_step, 1, repeats)["median"]
    step_bytes = n_layers * int(lengths.astype(np.int64).sum()) * kv_bytes_per_token
    plan = T.tempo_attn_plan(sts[0].kv, B, Hq, 8191, 0, True)
    return {"ms_per_step": round(dt * 1e3, 3), "ms_per_step_work_list": round(listed * 1e3, 3),
            "ms_per_step_dense_grid": round(dense * 1e3, 3), "graph_ms_per_step": round(gdt * 1e3, 3),
            "kv_gbs": round(step_bytes / dt / 1e9, 1), "kv_bytes_per_step": step_bytes,
            "pool_gib": round(2 * k_pool.numel() * 2 / 2**30, 1),
            "splits": plan.num_splits, "tokens_per_split": plan.tokens_per_split, "waves": plan.waves,
            "roofline": hbm_roofline("attn_partial_bf16<128, false>", step_bytes, min(dt, gdt),
                                     "all 28 layers (block-store write, attention, combine each, plus one work-list "
                                     "launch per step when listed); the fastest of dense grid, work list and one "
                                     "graph of the 28 dense layers"),
            "lengths": [int(x) for x in lengths]}


def prompt_only(torch, T, BlockStore, synth, dev, repeats):
    """The prompt-processing workload alone (for profiling its kernel): 4096 steps x 16
    sequences of the headline shape through one tempo_prefill_causal call, `repeats` times."""
    B, Hq, Hkv, D, Z, P = 16, 24, 8, 128, 256, 4096
    st = BlockStore(B, Hq, Hkv, D, Z, P - 1, T.TEMPO_BF16, device=dev)
    q = synth.device_normal((B, P, Hq, D), 277, torch.bfloat16, dev)
    k = synth.device_normal((B, P, Hkv, D), 278, torch.bfloat16, dev)
    v = synth.device_normal((B, P, Hkv, D), 279, torch.bfloat16, dev)
    o = torch.empty_like(q)
    dt = gpu_timed(torch, lambda i: st.prefill_attend(q, k, v, o, 0, P), repeats, 2, chunk=1)["median"]
    flops = B * (P * (P + 1) // 2) * 4 * D * Hq
    return {"workload": "prompt of 4096 steps x 16 sequences, llama-3.2-3b attention shape, one tempo_prefill_causal call",
            "ms": round(dt * 1e3, 3), "tokens_per_s": round(B * P / dt, 1), "algorithmic_flops_per_call": flops,
            "roofline": {"kernel": "attn_prefill_bf16<128, 8, false, false>", "bound": "mfma",
                         "achieved": round(flops / dt / 1e12, 1), "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": round(flops / dt / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}}


def block_only(torch, T, BlockStore, synth, dev, C, repeats):
    """One block workload alone (for profiling the split path of the LDS-staged kernel): C query
    steps of 16 sequences of the headline shape in front of 4096 - C stored steps, one block-store
    write and one tempo_attn_block_causal call per repeat, 8 layer pools rotated."""
    B, Hq, Hkv, D, Z = 16, 24, 8, 128, 256
    sts = []
    for layer in range(8):
        st = BlockStore(B, Hq, Hkv, D, Z, 4095, T.TEMPO_BF16, device=dev)
        st.k_pool.normal_()
        st.v_pool.normal_()
        sts.append(st)
    q = synth.device_normal((B, C, Hq, D), 177, torch.bfloat16, dev)
    k = synth.device_normal((B, C, Hkv, D), 178, torch.bfloat16, dev)
    v = synth.device_normal((B, C, Hkv, D), 179, torch.bfloat16, dev)
    o = torch.empty_like(q)

    def step(i):
        sts[i % 8].append_block(k, v, 4096 - C, C)
        sts[i % 8].attend_block(q, o, 4096 - C, C)

    dt = gpu_timed(torch, step, repeats, 10)["median"]
    plan = T.tempo_attn_block_plan(sts[0].kv, B, Hq, C, 4096 - C, 0)
    nbytes = B * 4096 * 2 * Hkv * D * 2
    return {"workload": f"block of {C} query steps x 16 sequences at t0={4096 - C}, llama-3.2-3b attention shape",
            "us_per_call": us(dt), "kv_gbs": round(nbytes / dt / 1e9, 1),
            "algorithmic_bytes_per_call": nbytes, "splits": plan.num_splits,
            "tokens_per_split": plan.tokens_per_split}


def step_only(torch, T, BlockStore, synth, dev, name, repeats):
    """One launch-bound step alone, `repeats` times over 8 rotated layer pools (for a kernel trace of
    where its microseconds go): "window512" = batch 16, 512-key window at t = 8191; "long8191" = one
    sequence at t = 8191; "t255" = batch 16, causal, t = 255."""
    Hq, Hkv, D, Z = 24, 8, 128, 256
    batch, max_t = (1, 8191) if name == "long8191" else (16, 8191)
    sts = []
    for layer in range(8):
        st = BlockStore(batch, Hq, Hkv, D, Z, max_t, T.TEMPO_BF16, device=dev)
        st.k_pool.normal_()
        st.v_pool.normal_()
        sts.append(st)
    q = synth.device_normal((batch, Hq, D), 71, torch.bfloat16, dev)
    k = synth.device_normal((batch, Hkv, D), 72, torch.bfloat16, dev)
    v = synth.device_normal((batch, Hkv, D), 73, torch.bfloat16, dev)
    o = sts[0].new_out()
    if name == "window512":
        fn, keys = (lambda i: sts[i % 8].step_window(q, k, v, o, 8191, 512)), 512
    elif name == "window512odd":   # the window starts inside a 32-slot group, as it does at most steps
        fn, keys = (lambda i: sts[i % 8].step_window(q, k, v, o, 8000, 512)), 512
    elif name == "t300":
        fn, keys = (lambda i: sts[i % 8].step_causal(q, k, v, o, 300)), 301
    elif name == "long8191":
        fn, keys = (lambda i: sts[i % 8].step_causal(q, k, v, o, 8191)), 8192
    elif name == "t255":
        fn, keys = (lambda i: sts[i % 8].step_causal(q, k, v, o, 255)), 256
    else:
        raise SystemExit(f"bench.py: unknown --step-only workload {name!r}")
    r = gpu_timed(torch, fn, repeats, 20)
    nbytes = batch * keys * 2 * Hkv * D * 2
    return {"workload": name, "us_per_step": us(r["median"]), "us_per_step_min": us(r["min"]),
            "kv_bytes_per_step": nbytes, "kv_gbs": round(nbytes / r["median"] / 1e9, 1)}


def plan_sweep(torch, T, BlockStore, synth, dev):
    """Every explicit split plan against the library's own choice: causal decode of the Llama head
    shape at batch 4, 16 and 64 and several steps; one attention call per step (the store already
    holds step t) through tempo_attn_block_with_plan, 8 rotated layer pools, median over chunks."""
    Hq, Hkv, D, Z = 24, 8, 128, 256
    out = {}
    for batch in (4, 16, 64):
        sts = []
        for layer in range(8):
            st = BlockStore(batch, Hq, Hkv, D, Z, 8191, T.TEMPO_BF16, device=dev)
            st.k_pool.normal_()
            st.v_pool.normal_()
            sts.append(st)
        q = synth.device_normal((batch, Hq, D), 61, torch.bfloat16, dev)
        o = sts[0].new_out()
        for t in (255, 1023, 1535, 2047, 2500, 3500, 4095, 5000, 8191):
            lib = T.tempo_attn_plan(sts[0].kv, batch, Hq, t, 0)
            rows = {}
            for k in range(7, 14):                                        # 128 .. 8192 keys per split
                tps = 1 << k
                splits = t // tps + 1
                if splits > 1024 or (splits == 1 and tps >= 2 * (t + 1)):
                    continue                                              # longer single splits are the same plan
                for waves in (4, 8):
                    if tps // 32 < waves:
                        continue
                    plan = T.tempo_plan(tps, splits, waves)
                    nbytes = T.tempo_attn_plan_workspace_bytes(sts[0].kv, batch, Hq, plan)
                    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)

                    def call(i):
                        T.tempo_attn_block_with_plan(sts[i % 8].kv, q, o, batch, Hq, 1, t, None, 0, sts[0].scale, plan,
                                                     ws, nbytes)

                    rows[f"{tps}x{waves}"] = us(gpu_timed(torch, call, 100, 10)["median"])
            lib_us = us(gpu_timed(torch, lambda i: sts[i % 8].attend_causal(q, o, t), 100, 10)["median"])
            out[f"b{batch}_t{t}"] = {"plans_us": rows, "library_plan": f"{lib.tokens_per_split}x{lib.waves}",
                                     "library_splits": lib.num_splits, "library_us": lib_us,
                                     "best_us": min(rows.values())}
        del sts
        torch.cuda.empty_cache()
    return out


def tile_sweep(torch, T, BlockStore, synth, dev):
    """Tile-size sweep and padded baseline at T = 16384 (the shape of the paper's block-size
    figure, Section 7.2): for batch 4 and 16 and tile sizes Z = 32 .. 8192, the mean time of a
    decode step over steps spread evenly over 0..T-1, (a) over the dynamic range (fused append +
    attention), (b) with every step padded to T and masked.  Pools are filled directly with
    N(0,1); 4 layer pools are rotated."""
    Hq, Hkv, D, T_len = 24, 8, 128, 16384
    kv_bytes_per_token = 2 * Hkv * D * 2
    steps = [T_len * (2 * i + 1) // 64 for i in range(32)]          # 32 evenly spread steps, mean = T/2
    out = {"T": T_len, "sampled_steps": len(steps), "unit": "us per decode step (mean over sampled steps)"}
    for batch in (4, 16):
        q = synth.device_normal((batch, Hq, D), 81, torch.bfloat16, dev)
        k = synth.device_normal((batch, Hkv, D), 82, torch.bfloat16, dev)
        v = synth.device_normal((batch, Hkv, D), 83, torch.bfloat16, dev)
        rows = {}
        for Z in (32, 64, 256, 1024, 2048, 8192):
            sts = []
            for layer in range(4):
                st = BlockStore(batch, Hq, Hkv, D, Z, T_len - 1, T.TEMPO_BF16, device=dev)
                st.k_pool.normal_()
                st.v_pool.normal_()
                sts.append(st)
            o = sts[0].new_out()
            dyn, pad = [], []
            for t in steps:
                dyn.append(gpu_timed(torch, lambda i: sts[i % 4].step_causal(q, k, v, o, t), 40, 8)["mean"])
                pad.append(gpu_timed(torch, lambda i: sts[i % 4].attend_padded(q, o, t, T_len - 1), 40, 8)["mean"])
            mean_dyn, mean_pad = sum(dyn) / len(dyn), sum(pad) / len(pad)
            mean_bytes = batch * (sum(steps) / len(steps) + 1) * kv_bytes_per_token
            rows[str(Z)] = {"dynamic_us": us(mean_dyn), "padded_us": us(mean_pad),
                            "padded_over_dynamic": round(mean_pad / mean_dyn, 2),
                            "dynamic_kv_gbs": round(mean_bytes / mean_dyn / 1e9, 1),
                            "last_step_dynamic_us": us(dyn[-1])}
            del sts
            torch.cuda.empty_cache()
        out[f"batch{batch}"] = rows
    return out


def cpu_baselines(torch, np, synth, oracle, dev, keep_flat, q, got_out, t, scale, step_bytes, kv_bytes_per_token):
    """The oracle as it stands, timed on this machine's host cores on bounded samples of the workloads
    (the only leg that touches it); its output at the headline step doubles as a parity spot check."""
    res = {}
    K0, V0 = keep_flat
    Kc = K0.float().cpu().numpy().astype(np.float64)
    Vc = V0.float().cpu().numpy().astype(np.float64)
    qc = q.float().cpu().numpy().astype(np.float64)
    sample_b = [0, 7, 15]
    got = got_out.float().cpu().numpy().astype(np.float64)
    ref = oracle.attend(qc, Kc, Vc, t, 0, scale)
    err = float(np.abs(got[sample_b] - ref[sample_b]).max())
    parity = {"max_abs_err": err, "ok": bool(err <= 2e-2 and err <= 1e-2 * np.abs(ref[sample_b]).max()),
              "sequences": sample_b}
    times = []
    budget_end = time.perf_counter() + 10.0
    while len(times) < 3 or (time.perf_counter() < budget_end and len(times) < 50):
        c0 = time.perf_counter()
        oracle.attend(qc, Kc, Vc, t, 0, scale)
        times.append(time.perf_counter() - c0)
    med = sorted(times)[len(times) // 2]
    res = {"value": round(step_bytes / med / 1e9, 3), "unit": "GB/s", "cores": oracle.threads(), "kind": "oracle",
           "sample": f"full batch of 16 sequences at t=4095 (one layer, attention only), "
                     f"median of {len(times)} runs, {med * 1e3:.1f} ms per step"}

    def best_of(fn, n=2):
        best = None
        for _ in range(n):
            c0 = time.perf_counter()
            fn()
            d = time.perf_counter() - c0
            best = d if best is None or d < best else best
        return best

    # the oracle at the steps of the per-t curve (two runs each, the faster one)
    per_t = {str(tt): round(best_of(lambda: oracle.attend(qc, Kc, Vc, tt, 0, scale)) * 1e3, 2)
             for tt in (255, 511, 1023, 2047)}
    per_t[str(t)] = round(med * 1e3, 2)
    res["ms_per_step_at_t"] = per_t
    others = {}
    # window 512, steady state: the same arrays, the window ending at t = 4095
    d = best_of(lambda: oracle.attend(qc, Kc, Vc, t, 512, scale), 3)
    others["window512_b16_steady_state"] = {"ms_per_step": round(d * 1e3, 3),
                                            "gbs": round(16 * 512 * kv_bytes_per_token / d / 1e9, 3)}
    # single core, headline step
    import ctypes
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        n_threads = oracle.threads()
        gomp.omp_set_num_threads(1)
        d = best_of(lambda: oracle.attend(qc, Kc, Vc, t, 0, scale), 1)
        gomp.omp_set_num_threads(n_threads)
        others["llama_causal_t4095_single_core"] = {"ms_per_step": round(d * 1e3, 1), "cores": 1,
                                                    "gbs": round(step_bytes / d / 1e9, 3)}
    except OSError:
        pass
    del Kc, Vc
    # one long sequence at t = 8191, 32767, 65535 (keys/values drawn on the GPU in fp64, values do not matter)
    Kl = torch.empty((1, 65536, 8, 128), dtype=torch.float64, device=dev).normal_().cpu().numpy()
    Vl = torch.empty((1, 65536, 8, 128), dtype=torch.float64, device=dev).normal_().cpu().numpy()
    for tt in (8191, 32767, 65535):
        d = best_of(lambda: oracle.attend(qc[:1], Kl, Vl, tt, 0, scale))
        others[f"long_b1_t{tt}"] = {"ms_per_step": round(d * 1e3, 2),
                                    "gbs": round((tt + 1) * kv_bytes_per_token / d / 1e9, 3)}
    del Kl, Vl
    # ragged 28-layer step: one layer (batch 64, the bench's own lengths) timed, times 28 identical-geometry layers
    lengths = synth.integers(24, 1, 64, 1, 8192)
    Kr = torch.empty((64, 8192, 8, 128), dtype=torch.float64, device=dev).normal_().cpu().numpy()
    Vr = torch.empty((64, 8192, 8, 128), dtype=torch.float64, device=dev).normal_().cpu().numpy()
    qr = np.ascontiguousarray(np.broadcast_to(qc[:1], (64,) + qc.shape[1:]))
    d = best_of(lambda: oracle.attend(qr, Kr, Vr, lengths - 1, 0, scale))
    layer_bytes = int(lengths.astype(np.int64).sum()) * kv_bytes_per_token
    others["ragged_28layers_b64"] = {"ms_per_step": round(28 * d * 1e3, 1), "gbs": round(layer_bytes / d / 1e9, 3),
                                     "sample": "one of the 28 identical-geometry layers timed, times 28"}
    del Kr, Vr
    res["other_workloads"] = others
    return res, parity


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--layers", type=int, default=8,
                    help="most pools rotated over (cache defeat); the run uses max(4, min(this, warmup))")
    ap.add_argument("--no-extras", action="store_true", help="skip the per-t curve, whole-run and other-workload legs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline")
    ap.add_argument("--counters", action="store_true",
                    help="short run to put under rocprofv3 --pmc: pools filled directly with N(0,1), "
                         "W+K decode steps, then 4 copy launches of 256 MiB (the known-size kernel the "
                         "traffic counters are scaled by); no timing, no oracle")
    ap.add_argument("--block-only", type=int, default=0, metavar="C",
                    help="instead of the headline run: a block of C query steps at t0 = 4096 - C alone, "
                         "--steps times, printed as one JSON line")
    ap.add_argument("--prompt-only", action="store_true",
                    help="instead of the headline run: the prompt-processing workload alone, --steps times "
                         "(use a small --steps), printed as one JSON line")
    ap.add_argument("--step-only", default="", metavar="NAME",
                    help="instead of the headline run: one launch-bound step alone, --steps times "
                         "(window512, long8191, t255, or ragged = the 28-layer ragged step), printed as one JSON line")
    ap.add_argument("--plan-sweep", action="store_true",
                    help="instead of the headline run: every explicit split plan against the library's choice at "
                         "batch 4, 16, 64, printed as one JSON line")
    ap.add_argument("--tile-sweep", action="store_true",
                    help="instead of the headline run: tile-size sweep and padded baseline at T=16384, "
                         "printed as one JSON line")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2501_05408_amd import synth
    from paper_2501_05408_amd import tempo as T
    from paper_2501_05408_amd.store import BlockStore

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    T.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.block_only:
        print(json.dumps({"block_of_queries": block_only(torch, T, BlockStore, synth, dev, args.block_only,
                                                         min(args.steps, 400))}))
        return 0
    if args.prompt_only:
        print(json.dumps({"prompt_processing": prompt_only(torch, T, BlockStore, synth, dev, min(args.steps, 50))}))
        return 0
    if args.step_only == "ragged":
        print(json.dumps({"ragged_step": ragged_step_bench(torch, T, BlockStore, synth, dev, 2 * 8 * 128 * 2,
                                                           min(args.steps, 100))}))
        return 0
    if args.step_only:
        print(json.dumps({"launch_bound_step": step_only(torch, T, BlockStore, synth, dev, args.step_only,
                                                         min(args.steps, 2000))}))
        return 0
    if args.plan_sweep:
        print(json.dumps({"plan_sweep": plan_sweep(torch, T, BlockStore, synth, dev)}))
        return 0
    if args.tile_sweep:
        print(json.dumps({"tile_size_sweep": tile_sweep(torch, T, BlockStore, synth, dev)}))
        return 0

    B, Hq, Hkv, D, Z, t = 16, 24, 8, 128, 256, 4095
    # Pools rotated over: at least 4 (4 x 256 MiB of keys/values, four times the last-level cache), at most
    # --layers, and no more than the warm-up steps, so that the W warm-up steps visit every pool once (a pool's
    # first step after set-up pays for cold address translation: 48-50 us instead of 46-47).
    R = max(4, min(args.layers, args.warmup))
    T_len = t + 1
    scale = 1.0 / math.sqrt(D)
    kv_bytes_per_token = 2 * Hkv * D * 2                      # K and V, bf16
    step_bytes = B * T_len * kv_bytes_per_token               # 256 MiB at t = 4095

    # --- build R layers: flat K/V drawn on the GPU, written through the ABI -------
    stores, keep_flat = [], None
    for layer in range(R if args.counters else 0):
        # hardware-counter mode: traffic does not depend on values, so skip the per-step appends
        perm = synth.permutation(7, layer, B * (T_len // Z))
        st = BlockStore(B, Hq, Hkv, D, Z, t, T.TEMPO_BF16, device=dev,
                        block_table=torch.from_numpy(perm.reshape(B, T_len // Z).copy()))
        st.k_pool.normal_()
        st.v_pool.normal_()
        st.k_last = synth.device_normal((B, Hkv, D), 500 + layer, torch.bfloat16, dev)
        st.v_last = synth.device_normal((B, Hkv, D), 600 + layer, torch.bfloat16, dev)
        stores.append(st)
    for layer in range(0 if args.counters else R):
        K = synth.device_normal((B, T_len, Hkv, D), 1000 + 2 * layer, torch.bfloat16, dev)
        V = synth.device_normal((B, T_len, Hkv, D), 1001 + 2 * layer, torch.bfloat16, dev)
        perm = synth.permutation(7, layer, B * (T_len // Z))
        table = torch.from_numpy(perm.reshape(B, T_len // Z).copy())
        st = BlockStore(B, Hq, Hkv, D, Z, t, T.TEMPO_BF16, device=dev, block_table=table)
        st.prefill(K, V, t - 1)
        st.k_last, st.v_last = K[:, t].contiguous(), V[:, t].contiguous()
        stores.append(st)
        if layer == 0:
            keep_flat = (K, V)
    q = synth.device_normal((B, Hq, D), 99, torch.bfloat16, dev)
    outs = [st.new_out() for st in stores]
    torch.cuda.synchronize()

    def step(i):
        st = stores[i % R]
        st.step_causal(q, st.k_last, st.v_last, outs[i % R], t)

    def step_separate(i):
        st = stores[i % R]
        st.append(st.k_last, st.v_last, t)
        st.attend_causal(q, outs[i % R], t)

    if args.counters:
        for i in range(args.warmup + args.steps):
            step(i)
        src = torch.empty(128 << 20, dtype=torch.bfloat16, device=dev).normal_()   # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(4):
            T.tempo_stream_copy(src, dst, 2 * src.numel(), 2048)
        torch.cuda.synchronize()
        print(json.dumps({"mode": "counters", "steps": args.warmup + args.steps,
                          "kv_bytes_per_step": step_bytes, "copy_bytes": 2 * src.numel(), "copies": 4}))
        return 0

    # --- the timed region: W warm-up steps, then exactly K steps -------------------
    head = gpu_timed(torch, step, args.steps, args.warmup)
    sec_per_step = head["median"]
    value = step_bytes / sec_per_step / 1e9

    # --- the same step through the separate append / attend entry points -----------
    sep = gpu_timed(torch, step_separate, args.steps, args.warmup)["median"]

    # --- the dominant kernel alone: the step's partial-attention launch (fused append
    # included), K launches back to back on the launch stream, timed with HIP events on
    # that stream exactly as the steps above.  Its mean period is what a kernel trace of
    # this command reports as that kernel's average duration (plus the dispatch gap).
    plan = T.tempo_attn_plan(stores[0].kv, B, Hq, t, 0)
    ws_bytes = stores[0].workspace_bytes

    def partial_only(i):
        st = stores[i % R]
        T.tempo_attn_decode_partial(st.kv, q, st.k_last, st.v_last, B, Hq, t, None, 0, scale, plan,
                                    st.workspace, ws_bytes)

    kern = gpu_timed(torch, partial_only, args.steps, args.warmup)
    kernel_s = kern["mean"]
    achieved = step_bytes / kernel_s / 1e9

    # --- the streaming-read yardstick over the same bytes (one layer's two pools) -----
    sink = torch.zeros(16, dtype=torch.int32, device=dev)

    def stream_only(i):
        st = stores[i % R]
        T.tempo_stream_read(st.k_pool, 2 * st.k_pool.numel(), sink, 512)
        T.tempo_stream_read(st.v_pool, 2 * st.v_pool.numel(), sink, 512)

    stream_s = gpu_timed(torch, stream_only, args.steps, args.warmup)["mean"]

    result = {
        "metric": "decode-attention KV GB/s (% of HBM peak) + steps/s, Llama-3.2-3B shape",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "llama-3.2-3b attention-layer shape, causal decode at t=4095 "
                        "(append + partial attention + split combine per step, one call)",
            "batch": B, "num_q_heads": Hq, "num_kv_heads": Hkv, "head_dim": D, "kv_block": Z,
            "t": t, "layers_rotated": R, "kv_bytes_per_step": step_bytes,
            "plan": {"tokens_per_split": plan.tokens_per_split, "num_splits": plan.num_splits,
                     "waves": plan.waves},
        },
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "timing": {"method": f"HIP events on the launch stream every {head['chunk']} steps; ms_per_step = median over "
                             f"{head['chunks']} chunks",
                   "ms_per_step_median": round(head["median"] * 1e3, 5),
                   "ms_per_step_min": round(head["min"] * 1e3, 5),
                   "ms_per_step_mean_gpu": round(head["mean"] * 1e3, 5),
                   "ms_per_step_mean_host_wall": round(head["wall"] * 1e3, 5),
                   "ms_per_step_first_chunks_in_order": [round(x * 1e3, 5) for x in head["first_chunks"]]},
        "separate_calls": {"ms_per_step": round(sep * 1e3, 5), "kv_gbs": round(step_bytes / sep / 1e9, 1),
                           "launches": "tempo_kv_append + tempo_attn_decode_causal"},
        "steps_per_s": round(1.0 / sec_per_step, 1),
        "roofline": {
            "kernel": "attn_partial_bf16<128, false>",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": measured_traffic_bytes(),
            "traffic_source": "profiles/attn_partial_bf16_llama_t4095_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE, "
                              "WRITE_SIZE of `bench.py --counters`, scaled by the copy kernel)",
            "kernel_avg_us": us(kernel_s),
            "kernel_avg_us_is": "mean launch period of K back-to-back launches of the kernel alone, HIP events on "
                                "the launch stream",
            "kernel_min_us": us(kern["min"]),
            "algorithmic_bytes_per_launch": step_bytes,
            "stream_read_same_bytes": {"us": us(stream_s), "gbs": round(step_bytes / stream_s / 1e9, 1),
                                       "note": "two plain read launches (K pool, V pool) of one layer"},
            "kernel_over_stream_read": round(stream_s / kernel_s, 4),
            "step_over_stream_read": round(stream_s / sec_per_step, 4),
        },
    }

    # --- CPU baseline: the oracle on this machine's host cores --------------------------------------
    if not args.no_cpu:
        from oracle import tempo_oracle as oracle

        result["cpu_baseline"], result["parity"] = cpu_baselines(torch, np, synth, oracle, dev, keep_flat, q, outs[0],
                                                                 t, scale, step_bytes, kv_bytes_per_token)

    # --- extras: graph replay of the headline step, single pool, per-t curve, whole run ---------
    if not args.no_extras:
        g = graph_timed(torch, step, 16, 20)
        result["graph_replay"] = {"ms_per_step": round(g["median"] * 1e3, 5), "kv_gbs": round(step_bytes / g["median"] / 1e9, 1),
                                  "note": "16 steps over the rotated pools captured in one HIP graph"}
        # the same step on ONE layer's pool (256 MiB of keys/values, the size of the last-level
        # cache): not the headline, reported so the effect of rotating pools is visible
        st0 = stores[0]
        dt1 = gpu_timed(torch, lambda i: st0.step_causal(q, st0.k_last, st0.v_last, outs[0], t), args.steps,
                        args.warmup)["median"]
        result["unrotated_single_pool"] = {"ms_per_step": round(dt1 * 1e3, 5),
                                           "kv_gbs": round(step_bytes / dt1 / 1e9, 1),
                                           "note": "one 256 MiB pool reused every step (partly cache resident)"}
        del stores, outs, keep_flat, st0
        torch.cuda.empty_cache()
        result["whole_run"] = whole_run_rotated(torch, T, BlockStore, synth, dev, kv_bytes_per_token)
        result["launch_bound"] = launch_bound_legs(torch, T, BlockStore, synth, dev, kv_bytes_per_token)
        result["other_workloads"] = other_workloads(torch, T, BlockStore, synth, dev, kv_bytes_per_token)

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
