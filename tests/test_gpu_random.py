"""Seeded random configurations of every attention entry point against the fp64 CPU
oracle: shapes, tile sizes, steps, windows, block lengths, per-sequence steps, ring
stores and random block tables drawn together, so that combinations no hand-written
case lists are exercised.  Tolerances as in test_gpu_parity.py (bf16 2e-2 absolute and
1e-2 of the largest reference magnitude; fp32 1e-5 for both).
"""
import numpy as np
import pytest
import torch

from oracle import tempo_oracle as oracle
from paper_2501_05408_amd import synth
from paper_2501_05408_amd import tempo as T
from paper_2501_05408_amd.store import BlockStore

from test_gpu_parity import DEV, TDT, assert_close, dev, host_inputs, np64, random_table

pytestmark = pytest.mark.gpu


def draw(seed, n, lo, hi):
    return [int(x) for x in synth.integers(seed, 900, n, lo, hi)]


def config(case):
    """One random configuration, fully determined by the case number."""
    r = draw(1000 + case, 12, 0, 1 << 20)
    dtype = T.TEMPO_BF16 if r[0] % 4 else T.TEMPO_F32
    D = (64, 128)[r[1] % 2]
    G = (1, 2, 3, 4, 5, 8, 16, 20, 40)[r[2] % 9]
    Hkv = (1, 2, 3)[r[3] % 3]
    B = 1 + r[4] % 5
    Z = (32, 64, 128)[r[5] % 3] if dtype == T.TEMPO_BF16 else (4, 8, 32, 64)[r[5] % 4]
    steps = 40 + r[6] % 500
    window = (0, 0, 1, 2, 31, 32, 33, 100, 257)[r[7] % 9]
    C = 1 + r[8] % (128 // G)                      # block length, up to the column limit
    ragged = r[9] % 3 == 0
    ring = window > 0 and r[10] % 3 == 0
    return dict(dtype=dtype, D=D, G=G, Hkv=Hkv, B=B, Z=Z, steps=steps, window=window, C=C, ragged=ragged,
                ring=ring, seed=r[11])


@pytest.mark.parametrize("case", range(160))
def test_random_configuration(case):
    c = config(case)
    dtype, D, G, Hkv, B, Z, steps, window = (c[k] for k in ("dtype", "D", "G", "Hkv", "B", "Z", "steps", "window"))
    Hq = Hkv * G
    C = min(c["C"], steps - 1)
    q, K, V = host_inputs(c["seed"] % 10000, B, steps, Hq, Hkv, D, dtype)
    ring_blocks = 0
    if c["ring"]:                                   # the smallest ring that always holds window + C - 1 keys
        need = (window + C - 1 - 2 + Z) // Z + 1
        ring_blocks = 1
        while ring_blocks < max(need, 1):
            ring_blocks *= 2
    if ring_blocks:
        st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, ring_blocks=ring_blocks, fill="nan")
    else:
        table, nb = random_table(c["seed"], B, (steps - 1) // Z + 1)
        st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    scale = 1.0 / np.sqrt(D)
    what = f"case {case}: {c}"

    # per-sequence last steps (ragged) or one common step
    if c["ragged"]:
        last = [C + x % (steps - C) for x in draw(c["seed"] + 1, B, 0, 1 << 20)]
    else:
        last = [steps - 1] * B
    t_max = max(last)
    first = [l - C + 1 for l in last]               # first step of the final block of C steps

    # history up to (excluding) the final block: single appends with per-sequence steps
    # (every sequence has at least one step of history; one whose history is complete
    # rewrites its last step with the same values)
    assert min(first) >= 1
    ar = torch.arange(B, device=DEV)
    for t in range(max(first)):
        tps = torch.tensor([min(t, f - 1) for f in first], dtype=torch.int32, device=DEV)
        st.append(Kd[ar, tps.long()].contiguous(), Vd[ar, tps.long()].contiguous(), t, tps)

    fps = torch.tensor(first, dtype=torch.int32, device=DEV)
    rows_k = torch.stack([Kd[b, first[b]:first[b] + C] for b in range(B)]).contiguous()
    rows_v = torch.stack([Vd[b, first[b]:first[b] + C] for b in range(B)]).contiguous()
    qb = np.stack([np.stack([q[first[b] + cc][b] for cc in range(C)]) for b in range(B)])
    ref = np.stack([oracle.attend(qb[:, cc].astype(np.float64), K64, V64, np.array(first, dtype=np.int32) + cc,
                                  window, scale) for cc in range(C)], axis=1)

    # 1. the block entry points: append the C steps, answer them in one call
    st.append_block(rows_k, rows_v, max(first), C, fps if c["ragged"] else None)
    out = torch.empty((B, C, Hq, D), dtype=TDT[dtype], device=DEV)
    st.attend_block(dev(qb, dtype), out, max(first), C, window, fps if c["ragged"] else None)
    assert_close(out, ref, dtype, what + " [block]")

    # 2. the last step again through the single-step entry points (plain and fused append)
    lps = torch.tensor(last, dtype=torch.int32, device=DEV)
    o1 = st.new_out()
    q_last = dev(qb[:, C - 1], dtype)
    if window:
        st.attend_window(q_last, o1, t_max, window, lps if c["ragged"] else None)
    else:
        st.attend_causal(q_last, o1, t_max, lps if c["ragged"] else None)
    assert_close(o1, ref[:, C - 1], dtype, what + " [single step]")
    o2 = st.new_out()
    k_last = torch.stack([Kd[b, last[b]] for b in range(B)]).contiguous()
    v_last = torch.stack([Vd[b, last[b]] for b in range(B)]).contiguous()
    if window:
        st.step_window(q_last, k_last, v_last, o2, t_max, window, lps if c["ragged"] else None)
    else:
        st.step_causal(q_last, k_last, v_last, o2, t_max, lps if c["ragged"] else None)
    assert torch.equal(o1.view(torch.uint8), o2.view(torch.uint8)), what + " [fused step differs from append + attend]"

    # 2b. per-sequence steps, bf16, a group the single-step kernel serves: the same step with its
    #     launch driven by a work list gives the same bits
    if c["ragged"] and dtype == T.TEMPO_BF16 and G <= 16:
        worklist = st.build_worklist(t_max, lps, window)
        o4 = st.step_ragged(q_last, k_last, v_last, st.new_out(), t_max, lps, worklist, window)
        assert torch.equal(o4.view(torch.uint8), o1.view(torch.uint8)), what + " [work list differs from the dense grid]"
        o5 = st.step_ragged(q_last, None, None, st.new_out(), t_max, lps, worklist, window)
        assert torch.equal(o5.view(torch.uint8), o1.view(torch.uint8)), what + " [work list, attention only]"

    # 3. uniform steps only: the same block through the prompt entry point into a second store
    if not c["ragged"] and not ring_blocks:
        st2 = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=st.num_blocks, block_table=st.block_table.cpu(),
                         fill="nan")
        f0 = first[0]
        st2.append_block(Kd[:, :f0].contiguous(), Vd[:, :f0].contiguous(), 0, f0)
        o3 = torch.empty((B, C, Hq, D), dtype=TDT[dtype], device=DEV)
        st2.prefill_attend(dev(qb, dtype), rows_k, rows_v, o3, f0, C, window)
        assert_close(o3, ref, dtype, what + " [prompt entry point]")
        assert torch.equal(st2.k_pool.view(torch.uint8), st.k_pool.view(torch.uint8)), what + " [stores differ]"
        assert torch.equal(st2.v_pool.view(torch.uint8), st.v_pool.view(torch.uint8)), what + " [stores differ]"
