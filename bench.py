#!/usr/bin/env python3
"""Benchmark of the decode-attention hot path on one MI355X.

Workload (the configuration the metric is quoted on): Llama-3.2-3B attention
layer shape, bf16 -- batch 16, 24 query heads, 8 key/value heads, head_dim 128,
key/value blocks of 256 -- causal decode at step t = 4095.  One "step" is one
pass of the whole path for one layer through tempo_decode_step_causal: the
block-store write of step t's key/value, partial attention over keys 0..t, and
the split combine, in one launch.  (The same step through the separate entry
points tempo_kv_append + tempo_attn_decode_causal is timed too and reported as
"separate_calls".)  Successive steps
rotate over several layers' pools (a decode step of a real model visits every
layer's keys/values once), so the key/value bytes of a step are not left in the
last-level cache by the previous one.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Prints ONE JSON line.  value = key/value GB/s = algorithmic key/value bytes read
per step (batch * (t+1) * 2 * Hkv * D * 2 bytes) / mean step time, inputs resident
in HBM.  "roofline" prices the dominant kernel (partial attention) against the
8 TB/s HBM peak from its own HIP-event durations inside the same run;
"cpu_baseline" is the fp64 oracle timed on this machine's host cores.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per launch of the partial-attention kernel at the benchmark workload,
# from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of `bench.py --counters`
# (profiles/attn_partial_bf16_llama_t4095_hbm_traffic.txt), each scaled by what the
# same counter reads for the 256 MiB copy kernel: 268,712,922 fetched + 1,711,861 written.
MEASURED_TRAFFIC_BYTES = 270424782


def _timed(torch, fn, n, warm):
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n):
        fn(i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / n


def other_workloads(torch, T, BlockStore, synth, dev, kv_bytes_per_token):
    """Sliding-window decode, a long single sequence, and the ragged 28-layer step, at their real
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

    # block of 5 query steps (5 x 3 heads = 15 of the 16 tile columns) over the headline
    # shape: append 5 steps, then one attention call answers steps 4091..4095
    sts = layers(8, 16, 4095)
    qb = synth.device_normal((16, 5, Hq, D), 77, torch.bfloat16, dev)
    kb = synth.device_normal((16, 5, Hkv, D), 78, torch.bfloat16, dev)
    vb = synth.device_normal((16, 5, Hkv, D), 79, torch.bfloat16, dev)
    ob = torch.empty_like(qb)

    def block_step(i):
        sts[i % 8].append_block(kb, vb, 4091, 5)
        sts[i % 8].attend_block(qb, ob, 4091, 5)

    dt = _timed(torch, block_step, 200, 20)
    plan = T.tempo_attn_block_plan(sts[0].kv, 16, Hq, 5, 4091, 0)
    out["block5_b16_t4091"] = {"us_per_call": round(dt * 1e6, 2), "us_per_query_step": round(dt * 1e6 / 5, 2),
                               "kv_gbs": round(16 * 4096 * kv_bytes_per_token / dt / 1e9, 1),
                               "splits": plan.num_splits, "tokens_per_split": plan.tokens_per_split,
                               "waves": plan.waves}
    # wider blocks through the LDS-staged kernel: 10, 21 and 42 steps (30, 63 and 126 columns)
    for C in (10, 21, 42):
        qc = synth.device_normal((16, C, Hq, D), 177, torch.bfloat16, dev)
        kc = synth.device_normal((16, C, Hkv, D), 178, torch.bfloat16, dev)
        vc = synth.device_normal((16, C, Hkv, D), 179, torch.bfloat16, dev)
        oc = torch.empty_like(qc)

        def wide_step(i):
            sts[i % 8].append_block(kc, vc, 4096 - C, C)
            sts[i % 8].attend_block(qc, oc, 4096 - C, C)

        dt = _timed(torch, wide_step, 200, 20)
        plan = T.tempo_attn_block_plan(sts[0].kv, 16, Hq, C, 4096 - C, 0)
        out[f"block{C}_b16_t{4096 - C}"] = {"us_per_call": round(dt * 1e6, 2),
                                            "us_per_query_step": round(dt * 1e6 / C, 2),
                                            "kv_gbs": round(16 * 4096 * kv_bytes_per_token / dt / 1e9, 1),
                                            "splits": plan.num_splits, "tokens_per_split": plan.tokens_per_split,
                                            "waves": plan.waves}
    # prompt processing: 4096 steps of 16 sequences in one tempo_prefill_causal call
    # (195 blocks of 21 steps + one of 1; per block: append, partial attention, combine)
    P = 4096
    qp = synth.device_normal((16, P, Hq, D), 277, torch.bfloat16, dev)
    kp = synth.device_normal((16, P, Hkv, D), 278, torch.bfloat16, dev)
    vp = synth.device_normal((16, P, Hkv, D), 279, torch.bfloat16, dev)
    op = torch.empty_like(qp)
    dt = _timed(torch, lambda i: sts[i % 8].prefill_attend(qp, kp, vp, op, 0, P), 5, 1)
    pairs = P * (P + 1) // 2                                             # (query, key) pairs per sequence
    tflops = 16 * pairs * 4 * D * Hq / dt / 1e12
    out["prompt_b16_t4096"] = {"ms": round(dt * 1e3, 3), "tokens_per_s": round(16 * P / dt, 1),
                               "tflops": round(tflops, 1),
                               "roofline": {"kernel": "attn_prefill_bf16<128, 8, false>", "bound": "mfma",
                                            "achieved": round(tflops, 1), "peak": 2500.0, "unit": "TFLOP/s",
                                            "frac": round(tflops / 2500.0, 4)},
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
    dt = _timed(torch, lambda i: sts[i % 8].rope_step(q16, k16, v16, o, 4095), 200, 20)

    def rope_separate(i):
        st = sts[i % 8]
        st.rope_rotate(q16, qr, 4095)
        st.rope_append(k16, v16, 4095)
        st.attend_causal(qr, o, 4095)

    dt3 = _timed(torch, rope_separate, 200, 20)
    out["rope_step_b16_t4095"] = {"us_per_step": round(dt * 1e6, 2),
                                  "kv_gbs": round(16 * 4096 * kv_bytes_per_token / dt / 1e9, 1),
                                  "separate_launches_us": round(dt3 * 1e6, 2),
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

    dt = _timed(torch, rope_block, 200, 20)
    out[f"rope_block{C}_b16_t{4096 - C}"] = {"us_per_call": round(dt * 1e6, 2),
                                             "us_per_query_step": round(dt * 1e6 / C, 2),
                                             "note": "rotating block write + block attention with unrotated queries"}
    del qc, kc, vc, oc
    del sts
    torch.cuda.empty_cache()

    # sliding window 512, batch 16, steady state (t >= 511), unaligned window position
    sts = layers(8, 16, 16383)
    o = sts[0].new_out()
    for t in (8191, 16383 - 100):
        dt = _timed(torch, lambda i: sts[i % 8].step_window(q16, k16, v16, o, t, 512), 200, 20)
        plan = T.tempo_attn_plan(sts[0].kv, 16, Hq, t, 512)
        out[f"window512_b16_t{t}"] = {"us_per_step": round(dt * 1e6, 2),
                                      "kv_gbs": round(16 * 512 * kv_bytes_per_token / dt / 1e9, 1),
                                      "splits": plan.num_splits, "tokens_per_split": plan.tokens_per_split}
    del sts
    torch.cuda.empty_cache()

    # the same window on a ring (window) store: 4 blocks per sequence whatever t is
    sts = []
    for layer in range(8):
        st = BlockStore(16, Hq, Hkv, D, Z, 2**30, T.TEMPO_BF16, device=dev, ring_blocks=4)
        st.k_pool.normal_()
        st.v_pool.normal_()
        sts.append(st)
    o = sts[0].new_out()
    t = 1000000
    dt = _timed(torch, lambda i: sts[i % 8].step_window(q16, k16, v16, o, t, 512), 200, 20)
    out[f"window512_ring4_b16_t{t}"] = {"us_per_step": round(dt * 1e6, 2),
                                        "kv_gbs": round(16 * 512 * kv_bytes_per_token / dt / 1e9, 1),
                                        "pool_mib_per_layer": round(2 * sts[0].k_pool.numel() * 2 / 2**20, 1),
                                        "linear_store_would_need_mib": round(16 * (t // Z + 1) * Hkv * Z * D * 2 * 2 / 2**20, 1)}
    del sts
    torch.cuda.empty_cache()

    # long single sequence
    sts = layers(8, 1, 65535)
    q1, k1, v1 = q16[:1].contiguous(), k16[:1].contiguous(), v16[:1].contiguous()
    o = sts[0].new_out()
    for t in (8191, 32767, 65535):
        dt = _timed(torch, lambda i: sts[i % 8].step_causal(q1, k1, v1, o, t), 200, 20)
        plan = T.tempo_attn_plan(sts[0].kv, 1, Hq, t, 0)
        out[f"long_b1_t{t}"] = {"us_per_step": round(dt * 1e6, 2),
                                "kv_gbs": round((t + 1) * kv_bytes_per_token / dt / 1e9, 1),
                                "splits": plan.num_splits, "work_items": plan.num_splits * Hkv}
    del sts
    torch.cuda.empty_cache()

    # ragged multi-layer: 28 layers, batch 64, lengths uniform in [1, 8192], one shared pool with
    # exactly the blocks the sequences need, a random block table per layer
    import numpy as np
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

    dt = _timed(torch, ragged_step, 10, 2)
    step_bytes = n_layers * int(lengths.astype(np.int64).sum()) * kv_bytes_per_token
    plan = T.tempo_attn_plan(sts[0].kv, B, Hq, 8191, 0, True)
    out["ragged_28layers_b64"] = {"ms_per_step": round(dt * 1e3, 3), "kv_gbs": round(step_bytes / dt / 1e9, 1),
                                  "kv_bytes_per_step": step_bytes, "pool_gib": round(2 * k_pool.numel() * 2 / 2**30, 1),
                                  "splits": plan.num_splits, "tokens_per_split": plan.tokens_per_split}
    return out


def prompt_only(torch, T, BlockStore, synth, dev, repeats):
    """The prompt-processing workload alone (for profiling its kernel): 4096 steps x 16
    sequences of the headline shape through one tempo_prefill_causal call, `repeats` times."""
    B, Hq, Hkv, D, Z, P = 16, 24, 8, 128, 256, 4096
    st = BlockStore(B, Hq, Hkv, D, Z, P - 1, T.TEMPO_BF16, device=dev)
    q = synth.device_normal((B, P, Hq, D), 277, torch.bfloat16, dev)
    k = synth.device_normal((B, P, Hkv, D), 278, torch.bfloat16, dev)
    v = synth.device_normal((B, P, Hkv, D), 279, torch.bfloat16, dev)
    o = torch.empty_like(q)
    dt = _timed(torch, lambda i: st.prefill_attend(q, k, v, o, 0, P), repeats, 2)
    flops = B * (P * (P + 1) // 2) * 4 * D * Hq
    return {"workload": "prompt of 4096 steps x 16 sequences, llama-3.2-3b attention shape, one tempo_prefill_causal call",
            "ms": round(dt * 1e3, 3), "tokens_per_s": round(B * P / dt, 1), "algorithmic_flops_per_call": flops,
            "roofline": {"kernel": "attn_prefill_bf16<128, 8, false>", "bound": "mfma", "achieved": round(flops / dt / 1e12, 1),
                         "peak": 2500.0, "unit": "TFLOP/s", "frac": round(flops / dt / 1e12 / 2500.0, 4)}}


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

    dt = _timed(torch, step, repeats, 10)
    plan = T.tempo_attn_block_plan(sts[0].kv, B, Hq, C, 4096 - C, 0)
    nbytes = B * 4096 * 2 * Hkv * D * 2
    return {"workload": f"block of {C} query steps x 16 sequences at t0={4096 - C}, llama-3.2-3b attention shape",
            "us_per_call": round(dt * 1e6, 2), "kv_gbs": round(nbytes / dt / 1e9, 1),
            "algorithmic_bytes_per_call": nbytes, "splits": plan.num_splits,
            "tokens_per_split": plan.tokens_per_split}


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
                dyn.append(_timed(torch, lambda i: sts[i % 4].step_causal(q, k, v, o, t), 40, 8))
                pad.append(_timed(torch, lambda i: sts[i % 4].attend_padded(q, o, t, T_len - 1), 40, 8))
            mean_dyn, mean_pad = sum(dyn) / len(dyn), sum(pad) / len(pad)
            mean_bytes = batch * (sum(steps) / len(steps) + 1) * kv_bytes_per_token
            rows[str(Z)] = {"dynamic_us": round(mean_dyn * 1e6, 2), "padded_us": round(mean_pad * 1e6, 2),
                            "padded_over_dynamic": round(mean_pad / mean_dyn, 2),
                            "dynamic_kv_gbs": round(mean_bytes / mean_dyn / 1e9, 1),
                            "last_step_dynamic_us": round(dyn[-1] * 1e6, 2)}
            del sts
            torch.cuda.empty_cache()
        out[f"batch{batch}"] = rows
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--layers", type=int, default=8, help="pools rotated over (cache defeat)")
    ap.add_argument("--no-extras", action="store_true", help="skip the per-t curve and whole-run legs")
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
    if args.tile_sweep:
        print(json.dumps({"tile_size_sweep": tile_sweep(torch, T, BlockStore, synth, dev)}))
        return 0

    B, Hq, Hkv, D, Z, t = 16, 24, 8, 128, 256, 4095
    R = args.layers
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
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    value = step_bytes / (elapsed / args.steps) / 1e9

    # --- the same step through the separate append / attend entry points -----------
    for i in range(args.warmup):
        step_separate(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step_separate(i)
    torch.cuda.synchronize()
    sep = (time.perf_counter() - t0) / args.steps

    # --- the dominant kernel alone: the step's partial-attention launch (fused append
    # included), K launches back to back on the launch stream between one pair of HIP
    # events, rotating over the same pools.  Its average period is what a kernel trace
    # of this command reports as that kernel's average duration.
    plan = T.tempo_attn_plan(stores[0].kv, B, Hq, t, 0)
    ws_bytes = stores[0].workspace_bytes

    def partial_only(i):
        st = stores[i % R]
        T.tempo_attn_decode_partial(st.kv, q, st.k_last, st.v_last, B, Hq, t, None, 0, scale, plan,
                                    st.workspace, ws_bytes)

    for i in range(args.warmup):
        partial_only(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.steps):
        partial_only(i)
    e1.record()
    torch.cuda.synchronize()
    kernel_avg_ms = e0.elapsed_time(e1) / args.steps
    achieved = step_bytes / (kernel_avg_ms * 1e-3) / 1e9

    # --- the streaming-read yardstick over the same bytes (one layer's two pools) -----
    sink = torch.zeros(16, dtype=torch.int32, device=dev)

    def stream_only(i):
        st = stores[i % R]
        T.tempo_stream_read(st.k_pool, 2 * st.k_pool.numel(), sink, 512)
        T.tempo_stream_read(st.v_pool, 2 * st.v_pool.numel(), sink, 512)

    for i in range(args.warmup):
        stream_only(i)
    e0.record()
    for i in range(args.steps):
        stream_only(i)
    e1.record()
    torch.cuda.synchronize()
    stream_ms = e0.elapsed_time(e1) / args.steps

    result = {
        "metric": "decode-attention KV GB/s (% of HBM peak) + steps/s, Llama-3.2-3B shape",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": "llama-3.2-3b attention-layer shape, causal decode at t=4095 "
                        "(append + partial attention + split combine per step, one launch)",
            "batch": B, "num_q_heads": Hq, "num_kv_heads": Hkv, "head_dim": D, "kv_block": Z,
            "t": t, "layers_rotated": R, "kv_bytes_per_step": step_bytes,
            "plan": {"tokens_per_split": plan.tokens_per_split, "num_splits": plan.num_splits,
                     "waves": plan.waves},
        },
        "pct_of_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "separate_calls": {"ms_per_step": round(sep * 1e3, 5), "kv_gbs": round(step_bytes / sep / 1e9, 1),
                           "launches": "tempo_kv_append + tempo_attn_decode_causal"},
        "steps_per_s": round(args.steps / elapsed, 1),
        "roofline": {
            "kernel": "attn_partial_bf16<128, false>",
            "bound": "hbm",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4),
            "traffic": MEASURED_TRAFFIC_BYTES,
            "kernel_avg_us": round(kernel_avg_ms * 1e3, 2),
            "algorithmic_bytes_per_launch": step_bytes,
            "stream_read_same_bytes": {"us": round(stream_ms * 1e3, 2),
                                       "gbs": round(step_bytes / (stream_ms * 1e-3) / 1e9, 1),
                                       "note": "two plain read launches (K pool, V pool) of one layer"},
        },
    }

    # --- CPU baseline: the oracle on this machine's host cores (the only leg that touches it);
    #     its output also serves as a parity spot check of the timed configuration --------
    K0, V0 = keep_flat
    if not args.no_cpu:
        from oracle import tempo_oracle as oracle

        Kc = K0.float().cpu().numpy().astype(np.float64)
        Vc = V0.float().cpu().numpy().astype(np.float64)
        qc = q.float().cpu().numpy().astype(np.float64)
        sample_b = [0, 7, 15]
        got = outs[0].float().cpu().numpy().astype(np.float64)
        ref = oracle.attend(qc, Kc, Vc, t, 0, scale)
        err = float(np.abs(got[sample_b] - ref[sample_b]).max())
        result["parity"] = {"max_abs_err": err,
                            "ok": bool(err <= 2e-2 and err <= 1e-2 * np.abs(ref[sample_b]).max()),
                            "sequences": sample_b}
        times = []
        budget_end = time.perf_counter() + 12.0
        while len(times) < 3 or (time.perf_counter() < budget_end and len(times) < 50):
            c0 = time.perf_counter()
            oracle.attend(qc, Kc, Vc, t, 0, scale)
            times.append(time.perf_counter() - c0)
        med = sorted(times)[len(times) // 2]
        result["cpu_baseline"] = {
            "value": round(step_bytes / med / 1e9, 3),
            "unit": "GB/s",
            "cores": oracle.threads(),
            "kind": "oracle",
            "sample": f"full batch of 16 sequences at t=4095 (one layer, attention only), "
                      f"median of {len(times)} runs, {med * 1e3:.1f} ms per step",
        }
        # the oracle at the steps of the per-t curve (two runs each, the faster one)
        per_t = {}
        for tt in (255, 511, 1023, 2047):
            best = None
            for _ in range(2):
                c0 = time.perf_counter()
                oracle.attend(qc, Kc, Vc, tt, 0, scale)   # reads keys 0..tt only
                d = time.perf_counter() - c0
                best = d if best is None or d < best else best
            per_t[str(tt)] = round(best * 1e3, 2)
        per_t[str(t)] = round(med * 1e3, 2)
        result["cpu_baseline"]["ms_per_step_at_t"] = per_t
        del Kc, Vc

    # --- extras: per-t curve and a whole decode run with real per-step appends ------
    if not args.no_extras:
        # the same step on ONE layer's pool (256 MiB of keys/values, the size of the last-level
        # cache): not the headline, reported so the effect of rotating pools is visible
        st0 = stores[0]
        dt1 = _timed(torch, lambda i: st0.step_causal(q, st0.k_last, st0.v_last, outs[0], t), args.steps, args.warmup)
        result["unrotated_single_pool"] = {"ms_per_step": round(dt1 * 1e3, 5),
                                           "kv_gbs": round(step_bytes / dt1 / 1e9, 1),
                                           "note": "one 256 MiB pool reused every step (partly cache resident)"}
        curve = {}
        for tt in (255, 511, 1023, 2047, 4095):
            n = 100
            for i in range(10):
                stores[i % R].attend_causal(q, outs[i % R], tt)
            torch.cuda.synchronize()
            c0 = time.perf_counter()
            for i in range(n):
                st = stores[i % R]
                st.step_causal(q, st.k_last, st.v_last, outs[i % R], tt)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - c0) / n
            curve[str(tt)] = {"us_per_step": round(dt * 1e6, 2),
                              "kv_gbs": round(B * (tt + 1) * kv_bytes_per_token / dt / 1e9, 1)}
        result["curve_t"] = curve
        # whole run t = 0..4095 on one layer: append step t, attend step t
        K0c, V0c = K0.transpose(0, 1).contiguous(), V0.transpose(0, 1).contiguous()  # [T][B][Hkv][D]
        st = stores[0]
        torch.cuda.synchronize()
        c0 = time.perf_counter()
        for tt in range(T_len):
            st.step_causal(q, K0c[tt], V0c[tt], outs[0], tt)
        torch.cuda.synchronize()
        run = time.perf_counter() - c0
        total_bytes = B * kv_bytes_per_token * T_len * (T_len + 1) // 2
        result["whole_run"] = {"steps": T_len, "seconds": round(run, 4),
                               "steps_per_s": round(T_len / run, 1),
                               "kv_gbs": round(total_bytes / run / 1e9, 1),
                               "note": "one layer, 256 MiB pool (partly cache resident at small t)"}

    # --- the other workloads of the metric's family (timing only; their parity is in tests/) -----
    if not args.no_extras:
        del stores, outs, keep_flat
        torch.cuda.empty_cache()
        result["other_workloads"] = other_workloads(torch, T, BlockStore, synth, dev, kv_bytes_per_token)

    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
