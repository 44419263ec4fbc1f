"""GPU parity of the block-of-queries entry points (C consecutive query steps per
call over the same tiled keys/values) against the fp64 CPU oracle, which answers
each step on its own, and of the multi-step in-place write against single-step
writes (bit for bit).

Tolerances are those of test_gpu_parity.py:
  bf16  |gpu - oracle| <= 2e-2 elementwise  and  max|gpu - oracle| <= 1e-2 * max|oracle|
  fp32  the same two measures with 1e-5
"""
import numpy as np
import pytest
import torch

from oracle import tempo_oracle as oracle
from paper_2501_05408_amd import synth
from paper_2501_05408_amd import tempo as T
from paper_2501_05408_amd.store import BlockStore

from test_gpu_parity import DEV, TDT, assert_close, dev, flat_kv, host_inputs, np64, random_table

pytestmark = pytest.mark.gpu


def block_of(q, t0, C):
    """q is [T][B][Hq][D]; the block's queries as [B][C][Hq][D]."""
    return np.ascontiguousarray(np.stack([q[t0 + c] for c in range(C)], axis=1))


def oracle_block(q, K64, V64, t0, C, window, D, t_per_seq=None):
    """One oracle call per query step: [B][C][Hq][D]."""
    outs = []
    for c in range(C):
        if t_per_seq is None:
            outs.append(oracle.attend(q[t0 + c].astype(np.float64), K64, V64, t0 + c, window, 1.0 / np.sqrt(D)))
        else:
            tq = np.asarray(t_per_seq) + c
            qc = np.stack([q[int(tq[b])][b] for b in range(len(tq))]).astype(np.float64)
            outs.append(oracle.attend(qc, K64, V64, tq, window, 1.0 / np.sqrt(D)))
    return np.stack(outs, axis=1)


# ----------------------------------------------------------------------------
# Multi-step in-place write == the same steps written one by one, bit for bit.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
def test_append_block_equals_single_appends(dtype):
    B, Hq, Hkv, D, Z, steps = 3, 4, 2, 128, 32, 150
    _, K, V = host_inputs(41, B, steps, Hq, Hkv, D, dtype)
    table, nb = random_table(41, B, steps // Z + 1)
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    one = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table)
    for t in range(steps):
        one.append(Kd[:, t].contiguous(), Vd[:, t].contiguous(), t)
    blk = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table)
    t = 0
    for count in (1, 5, 26, 1, 31, 32, 33, 21):     # crosses groups of 32 and blocks at every offset
        blk.append_block(Kd[:, t:t + count].contiguous(), Vd[:, t:t + count].contiguous(), t, count)
        t += count
    assert t == steps
    assert torch.equal(one.k_pool.view(torch.uint8), blk.k_pool.view(torch.uint8))
    assert torch.equal(one.v_pool.view(torch.uint8), blk.v_pool.view(torch.uint8))
    # per-sequence first steps: rows land at t_per_seq[b] + c and nowhere else
    rag = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table)
    first = [3, 140, 62]
    C = 7
    tps = torch.tensor(first, dtype=torch.int32, device=DEV)
    rows_k = torch.stack([Kd[b, first[b]:first[b] + C] for b in range(B)]).contiguous()
    rows_v = torch.stack([Vd[b, first[b]:first[b] + C] for b in range(B)]).contiguous()
    rag.append_block(rows_k, rows_v, max(first), C, tps)
    kg, vg = rag.gather(0, steps)
    for b in range(B):
        assert torch.equal(kg[b, first[b]:first[b] + C], Kd[b, first[b]:first[b] + C])
        assert torch.equal(vg[b, first[b]:first[b] + C], Vd[b, first[b]:first[b] + C])
        assert int((kg[b] != 0).any(dim=-1).any(dim=-1).sum()) == C
    with pytest.raises(T.TempoError):
        blk.append_block(Kd[:, :8].contiguous(), Vd[:, :8].contiguous(), one.max_t - 6, 8)   # runs past the table


# ----------------------------------------------------------------------------
# fp32: every start step, several block lengths, causal and windows.  The pool is
# NaN-poisoned and holds exactly the steps the block may see.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("window", [0, 1, 3, 20])
@pytest.mark.parametrize("C", [2, 5, 8])
def test_block_fp32_every_start(window, C):
    B, Hq, Hkv, D, Z, steps = 2, 4, 2, 64, 8, 90
    dtype = T.TEMPO_F32
    q, K, V = host_inputs(42, B, steps, Hq, Hkv, D, dtype)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, fill="nan")
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    starts = list(range(steps - C + 1))
    outs = torch.empty((len(starts), B, C, Hq, D), dtype=torch.float32, device=DEV)
    st.append_block(Kd[:, :C - 1].contiguous(), Vd[:, :C - 1].contiguous(), 0, C - 1)
    for t0 in starts:
        st.append(Kd[:, t0 + C - 1].contiguous(), Vd[:, t0 + C - 1].contiguous(), t0 + C - 1)
        st.attend_block(dev(block_of(q, t0, C), dtype), outs[t0], t0, C, window)
    torch.cuda.synchronize()
    got = np64(outs)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for t0 in starts:
        assert_close(got[t0], oracle_block(q, K64, V64, t0, C, window, D), dtype, f"fp32 block t0={t0}")


# ----------------------------------------------------------------------------
# bf16: group sizes x block lengths up to the 16-column limit, every start step,
# one sequence so the planner cuts the range into many short splits (queries whose
# range misses a split; both combine kernels), pool poisoned beyond the last step.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("G,C,D", [(3, 5, 128), (1, 16, 128), (4, 4, 64), (2, 3, 128), (16, 1, 64), (5, 3, 128),
                                   # more than 16 columns: the LDS-staged kernel, up to 128 columns
                                   (3, 10, 128), (3, 21, 128), (1, 64, 64), (4, 16, 128), (2, 9, 64), (16, 4, 128),
                                   (1, 17, 128), (5, 7, 64), (3, 42, 128), (1, 128, 64), (4, 32, 128), (16, 8, 64),
                                   (2, 33, 128)])
@pytest.mark.parametrize("window", [0, 1, 2, 33, 64, 65, 200])
def test_block_bf16_every_start(G, C, D, window):
    B, Hkv, Z, steps = 1, 2, 64, 700
    Hq = Hkv * G
    dtype = T.TEMPO_BF16
    q, K, V = host_inputs(43, B, steps, Hq, Hkv, D, dtype)
    table, nb = random_table(43, B, steps // Z + 1)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    starts = list(range(0, 140)) + list(range(140, steps - C + 1, 3))
    outs = torch.empty((len(starts), B, C, Hq, D), dtype=torch.bfloat16, device=DEV)
    filled = 0
    seen_splits = set()
    for i, t0 in enumerate(starts):
        need = t0 + C
        st.append_block(Kd[:, filled:need].contiguous(), Vd[:, filled:need].contiguous(), filled, need - filled)
        filled = need
        st.attend_block(dev(block_of(q, t0, C), dtype), outs[i], t0, C, window)
        seen_splits.add(T.tempo_attn_plan(st.kv, B, Hq, t0 + C - 1, window + C - 1 if window else 0).num_splits)
    torch.cuda.synchronize()
    got = np64(outs)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for i, t0 in enumerate(starts):
        assert_close(got[i], oracle_block(q, K64, V64, t0, C, window, D), dtype,
                     f"bf16 block G={G} C={C} w={window} t0={t0}")
    if window == 0:
        assert min(seen_splits) == 1 and max(seen_splits) > 8     # direct, few-split and many-split paths


# ----------------------------------------------------------------------------
# A block gives what C single-step calls give (same tolerance, against each other
# and the oracle), with per-sequence first steps and a shared random block table.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
@pytest.mark.parametrize("window", [0, 45])
def test_block_ragged_first_steps(dtype, window):
    B, Hq, Hkv, D, Z, steps, C = 5, 6, 2, 128, 32, 400, 4
    q, K, V = host_inputs(44, B, steps, Hq, Hkv, D, dtype)
    table, nb = random_table(44, B, steps // Z + 1)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    st.prefill(Kd, Vd, steps - 1)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for first in ([0, 396, 31, 200, 63], [395, 1, 32, 95, 300], [10, 10, 10, 10, 10]):
        tps = torch.tensor(first, dtype=torch.int32, device=DEV)
        qb = np.stack([np.stack([q[first[b] + c][b] for c in range(C)]) for b in range(B)])
        out = torch.empty((B, C, Hq, D), dtype=TDT[dtype], device=DEV)
        st.attend_block(dev(qb, dtype), out, max(first), C, window, tps)
        ref = oracle_block(q, K64, V64, 0, C, window, D, t_per_seq=first)
        assert_close(out, ref, dtype, f"ragged block first={first}")
        single = torch.empty_like(out)
        for c in range(C):
            tc = (tps + c).contiguous()
            o = st.new_out()
            if window:
                st.attend_window(dev(qb[:, c], dtype), o, max(first) + c, window, tc)
            else:
                st.attend_causal(dev(qb[:, c], dtype), o, max(first) + c, tc)
            single[:, c] = o
        assert_close(out, np64(single), dtype, f"block vs single steps first={first}")


# ----------------------------------------------------------------------------
# Ring (window) store: a block of queries over recycled blocks.
# ----------------------------------------------------------------------------
def test_block_on_ring_store_bf16():
    B, Hq, Hkv, D, Z, R, window, C, steps = 2, 6, 2, 128, 32, 4, 60, 5, 500
    dtype = T.TEMPO_BF16
    q, K, V = host_inputs(45, B, steps, Hq, Hkv, D, dtype)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, ring_blocks=R, fill="nan")
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    filled = 0
    for t0 in range(0, steps - C + 1, C):
        st.append_block(Kd[:, filled:t0 + C].contiguous(), Vd[:, filled:t0 + C].contiguous(), filled, t0 + C - filled)
        filled = t0 + C
        out = torch.empty((B, C, Hq, D), dtype=torch.bfloat16, device=DEV)
        st.attend_block(dev(block_of(q, t0, C), dtype), out, t0, C, window)
        assert_close(out, oracle_block(q, K64, V64, t0, C, window, D), dtype, f"ring block t0={t0}")
    with pytest.raises(T.TempoError):            # union of the ranges would touch a fifth tile
        st.attend_block(dev(block_of(q, 400, C), dtype), out, 400, C, 3 * Z - 2)


# ----------------------------------------------------------------------------
# Full-size Llama shape: blocks of 5 steps (5 x 3 heads = 15 of the 16 columns),
# of 21 and of 42 steps (63 and 126 columns, the LDS-staged kernel), including blocks
# that straddle the planner's split boundary at key 2048.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("C", [5, 21, 42])
def test_llama_shape_block_bf16_full_size(C):
    B, Hq, Hkv, D, Z, T_len = 16, 24, 8, 128, 256, 4096
    dtype = T.TEMPO_BF16
    K, V = flat_kv(46, B, T_len, Hkv, D)
    table, nb = random_table(46, B, T_len // Z, extra=0)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    st.prefill(K, V, T_len - 1)
    K64, V64 = np64(K), np64(V)
    for window in (0, 512):
        for t0 in (0, 29, 2043 - (C - 5), 2044, 2046, 2048, 4096 - C):
            q = synth.device_normal((B, C, Hq, D), 4600 + t0, torch.bfloat16, DEV)
            out = torch.empty((B, C, Hq, D), dtype=torch.bfloat16, device=DEV)
            st.attend_block(q, out, t0, C, window)
            q64 = np64(q)
            ref = np.stack([oracle.attend(q64[:, c], K64[:, :t0 + c + 1], V64[:, :t0 + c + 1], t0 + c, window,
                                          1.0 / np.sqrt(D)) for c in range(C)], axis=1)
            assert_close(out, ref, dtype, f"llama block w={window} t0={t0}")


# ----------------------------------------------------------------------------
# Prompt processing in one call: `count` steps written and answered, each step
# exactly the single-step result; the store ends up as single appends leave it.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,G,D", [(T.TEMPO_BF16, 3, 128), (T.TEMPO_BF16, 1, 64), (T.TEMPO_BF16, 16, 128),
                                       (T.TEMPO_F32, 2, 64)])
@pytest.mark.parametrize("window", [0, 50])
def test_prefill_every_step(dtype, G, D, window):
    B, Hkv, Z, steps, first = 2, 2, 32, 300, 37
    Hq = Hkv * G
    q, K, V = host_inputs(47, B, steps, Hq, Hkv, D, dtype)
    table, nb = random_table(47, B, steps // Z + 1)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    ref_store = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    qd = dev(np.ascontiguousarray(np.transpose(q, (1, 0, 2, 3))), dtype)       # [B][T][Hq][D]
    # a first call from step 0, a second one that continues the history
    o1 = torch.empty((B, first, Hq, D), dtype=TDT[dtype], device=DEV)
    st.prefill_attend(qd[:, :first].contiguous(), Kd[:, :first].contiguous(), Vd[:, :first].contiguous(), o1, 0,
                      first, window)
    o2 = torch.empty((B, steps - first, Hq, D), dtype=TDT[dtype], device=DEV)
    st.prefill_attend(qd[:, first:].contiguous(), Kd[:, first:].contiguous(), Vd[:, first:].contiguous(), o2, first,
                      steps - first, window)
    got = np.concatenate([np64(o1), np64(o2)], axis=1)
    for t in range(steps):
        ref_store.append(Kd[:, t].contiguous(), Vd[:, t].contiguous(), t)
    assert torch.equal(st.k_pool.view(torch.uint8), ref_store.k_pool.view(torch.uint8))
    assert torch.equal(st.v_pool.view(torch.uint8), ref_store.v_pool.view(torch.uint8))
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for t in range(steps):
        ref = oracle.attend(q[t].astype(np.float64), K64, V64, t, window, 1.0 / np.sqrt(D))
        assert_close(got[:, t], ref, dtype, f"prefill step {t} w={window}")


# ----------------------------------------------------------------------------
# The prompt kernel (enough query blocks to fill the part: one launch after the
# block-store write), every step against the oracle: group sizes, head dims,
# windows, a call that continues a history, NaN beyond the prompt.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("G,D,Hkv", [(3, 128, 4), (1, 64, 8), (16, 128, 2), (5, 64, 4)])
@pytest.mark.parametrize("window", [0, 1, 45, 200])
def test_prompt_kernel_every_step(G, D, Hkv, window):
    B, Z, steps, first = 16, 32, 330, 29
    Hq = Hkv * G
    dtype = T.TEMPO_BF16
    q, K, V = host_inputs(49, B, steps, Hq, Hkv, D, dtype)
    table, nb = random_table(49, B, steps // Z + 2)
    st = BlockStore(B, Hq, Hkv, D, Z, steps + Z - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    qd = dev(np.ascontiguousarray(np.transpose(q, (1, 0, 2, 3))), dtype)
    assert T.tempo_prefill_launches(st.kv, B, Hq, first) > 2          # a short first call goes block by block
    assert T.tempo_prefill_launches(st.kv, B, Hq, steps - first) == 2  # the rest is one launch of the prompt kernel
    o1 = torch.empty((B, first, Hq, D), dtype=torch.bfloat16, device=DEV)
    st.prefill_attend(qd[:, :first].contiguous(), Kd[:, :first].contiguous(), Vd[:, :first].contiguous(), o1, 0,
                      first, window)
    o2 = torch.empty((B, steps - first, Hq, D), dtype=torch.bfloat16, device=DEV)
    st.prefill_attend(qd[:, first:].contiguous(), Kd[:, first:].contiguous(), Vd[:, first:].contiguous(), o2, first,
                      steps - first, window)
    got = np.concatenate([np64(o1), np64(o2)], axis=1)
    kg, vg = st.gather(0, steps)
    assert torch.equal(kg, Kd) and torch.equal(vg, Vd)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for t in range(steps):
        ref = oracle.attend(q[t].astype(np.float64), K64, V64, t, window, 1.0 / np.sqrt(D))
        assert_close(got[:, t], ref, dtype, f"prompt kernel step {t} G={G} w={window}")


# ----------------------------------------------------------------------------
# Prompts of different lengths in one call: each sequence writes and answers its
# own steps only; everything beyond (store slots, rows of out) is left untouched.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("G,D,window,first", [(3, 128, 0, 0), (3, 128, 40, 0), (2, 64, 0, 45), (16, 128, 0, 7)])
def test_prompt_kernel_per_sequence_lengths(G, D, window, first):
    B, Hkv, Z, steps = 12, 2, 32, 200
    Hq = Hkv * G
    dtype = T.TEMPO_BF16
    q, K, V = host_inputs(50, B, first + steps, Hq, Hkv, D, dtype)
    counts = [0, 1, 200, 31, 32, 33, 64, 199, 100, 5, 96, 130]
    st = BlockStore(B, Hq, Hkv, D, Z, first + steps - 1, dtype, fill="nan")
    ref_store = BlockStore(B, Hq, Hkv, D, Z, first + steps - 1, dtype, fill="nan")
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    qd = dev(np.ascontiguousarray(np.transpose(q, (1, 0, 2, 3))), dtype)
    if first:                                   # a common history, written the plain way into both stores
        st.append_block(Kd[:, :first].contiguous(), Vd[:, :first].contiguous(), 0, first)
        ref_store.append_block(Kd[:, :first].contiguous(), Vd[:, :first].contiguous(), 0, first)
    cps = torch.tensor(counts, dtype=torch.int32, device=DEV)
    out = torch.full((B, steps, Hq, D), 7.0, dtype=torch.bfloat16, device=DEV)
    st.prefill_attend(qd[:, first:].contiguous(), Kd[:, first:].contiguous(), Vd[:, first:].contiguous(), out, first,
                      steps, window, count_per_seq=cps)
    # the store: as if every sequence had appended its own steps one by one
    for c in range(max(counts)):
        live = torch.tensor([first + min(c, n - 1) if n > 0 else -1 for n in counts], dtype=torch.int32, device=DEV)
        rows = [b for b in range(B) if counts[b] > c]
        if not rows:
            break
        # sequences whose prompt is over rewrite their last step (same bits); empty ones are handled below
        ar = torch.arange(B, device=DEV)
        tt = torch.clamp(live, min=0)
        ref_store.append(Kd[ar, tt.long()].contiguous(), Vd[ar, tt.long()].contiguous(), first + c, tt)
    got_k, got_v = st.gather(0, first + steps)
    ref_k, ref_v = ref_store.gather(0, first + steps)
    for b in range(B):
        n = counts[b]
        if n == 0 and first == 0:
            continue                            # the reference loop wrote step 0 of empty sequences; compare below
        assert torch.equal(got_k[b].view(torch.int16), ref_k[b].view(torch.int16)), f"keys of sequence {b}"
        assert torch.equal(got_v[b].view(torch.int16), ref_v[b].view(torch.int16)), f"values of sequence {b}"
    if first == 0:                              # an empty prompt leaves its (NaN-filled) blocks alone
        assert torch.isnan(got_k[0].float()).all() and torch.isnan(got_v[0].float()).all()
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    got = np64(out)
    for b in range(B):
        n = counts[b]
        assert (got[b, n:] == 7.0).all(), f"rows of out beyond the prompt of sequence {b} were written"
        for c in range(n):
            t = first + c
            ref = oracle.attend(q[t][b:b + 1].astype(np.float64), K64[b:b + 1], V64[b:b + 1], t, window, 1.0 / np.sqrt(D))
            assert_close(got[b:b + 1, c], ref, dtype, f"ragged prompt b={b} step {t}")


def test_llama_shape_prefill_bf16_full_size():
    B, Hq, Hkv, D, Z, T_len = 16, 24, 8, 128, 256, 4096
    dtype = T.TEMPO_BF16
    K, V = flat_kv(48, B, T_len, Hkv, D)
    table, nb = random_table(48, B, T_len // Z, extra=0)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    q = synth.device_normal((B, T_len, Hq, D), 4800, torch.bfloat16, DEV)
    out = torch.empty_like(q)
    assert T.tempo_prefill_launches(st.kv, B, Hq, T_len) == 2
    st.prefill_attend(q, K, V, out, 0, T_len)
    kg, vg = st.gather(0, T_len)
    assert torch.equal(kg, K) and torch.equal(vg, V)
    K64, V64 = np64(K), np64(V)
    sample = [0, 1, 20, 21, 22, 41, 42, 63, 1000, 2047, 2048, 2049, 2058, 3000, 4073, 4074, 4094, 4095]
    sample += [int(x) for x in synth.integers(48, 9, 24, 0, T_len - 1)]
    for t in sample:
        ref = oracle.attend(np64(q[:, t]), K64[:, :t + 1], V64[:, :t + 1], t, 0, 1.0 / np.sqrt(D))
        assert_close(out[:, t], ref, dtype, f"llama prefill step {t}")
