"""GPU parity: libtempo (through its C ABI) against the fp64 CPU oracle, element
by element, on the same seeded inputs.

Tolerances (written out here on purpose):
  bf16 workloads  |gpu - oracle| <= 2e-2 elementwise  and  max|gpu - oracle| <= 1e-2 * max|oracle|
  fp32 workloads  the same two measures with 1e-5
Integer results (visible range, tile, slot) and everything the block store holds
are compared bit for bit.
"""
import numpy as np
import pytest
import torch

from oracle import tempo_oracle as oracle
from paper_2501_05408_amd import synth
from paper_2501_05408_amd import tempo as T
from paper_2501_05408_amd.store import BlockStore

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
TOL = {T.TEMPO_BF16: (2e-2, 1e-2), T.TEMPO_F32: (1e-5, 1e-5)}
TDT = {T.TEMPO_BF16: torch.bfloat16, T.TEMPO_F32: torch.float32}
NAME = {T.TEMPO_BF16: "bf16", T.TEMPO_F32: "f32"}


def np64(x):
    return x.detach().float().cpu().numpy().astype(np.float64)


def assert_close(got, ref, dtype, what):
    atol, rtol = TOL[dtype]
    g = np64(got) if isinstance(got, torch.Tensor) else got
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    err = np.abs(g - ref).max()
    assert err <= atol, f"{what}: max-abs {err:.3e} > {atol}"
    assert err <= rtol * np.abs(ref).max(), f"{what}: max-abs {err:.3e} > {rtol} * {np.abs(ref).max():.3e}"


def host_inputs(seed, B, T_len, Hq, Hkv, D, dtype):
    """q for every step and K, V: fp32 arrays holding values rounded to dtype."""
    q = synth.normal_as(seed, 1, (T_len, B, Hq, D), NAME[dtype])
    K = synth.normal_as(seed, 2, (B, T_len, Hkv, D), NAME[dtype])
    V = synth.normal_as(seed, 3, (B, T_len, Hkv, D), NAME[dtype])
    return q, K, V


def dev(x, dtype):
    return torch.from_numpy(np.ascontiguousarray(x)).to(DEV).to(TDT[dtype])


def random_table(seed, batch, max_blocks, extra=3):
    n = batch * max_blocks + extra
    perm = synth.permutation(seed, 77, n)[: batch * max_blocks]
    return torch.from_numpy(perm.reshape(batch, max_blocks).copy()), n


# ----------------------------------------------------------------------------
# Block store: what append writes is what the header's layout says, bit for bit.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
@pytest.mark.parametrize("D,Z", [(128, 64), (64, 32)])
def test_append_then_gather_is_identity(dtype, D, Z):
    B, Hq, Hkv, steps = 3, 4, 2, 150
    _, K, V = host_inputs(31, B, steps, Hq, Hkv, D, dtype)
    table, nb = random_table(31, B, steps // Z + 1)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    for t in range(steps):
        st.append(Kd[:, t].contiguous(), Vd[:, t].contiguous(), t)
    kg, vg = st.gather(0, steps)
    assert torch.equal(kg, Kd) and torch.equal(vg, Vd)
    kg, vg = st.gather(37, 70)
    assert torch.equal(kg, Kd[:, 37:107]) and torch.equal(vg, Vd[:, 37:107])
    # the pool itself, element by element, at the offsets the ABI documents
    kp = st.k_pool.flatten().cpu()
    vp = st.v_pool.flatten().cpu()
    Kc, Vc = Kd.cpu(), Vd.cpu()
    rng = np.random.default_rng(5)
    for _ in range(400):
        b, t, h, d = rng.integers(B), rng.integers(steps), rng.integers(Hkv), rng.integers(D)
        tile, slot = T.tempo_append_slot(int(t), Z)
        assert (tile, slot) == oracle.append_slot(int(t), Z)
        blk = int(table[b, tile])
        assert kp[T.tempo_kv_element_offset(st.kv, 0, blk, int(h), slot, int(d))] == Kc[b, t, h, d]
        assert vp[T.tempo_kv_element_offset(st.kv, 1, blk, int(h), slot, int(d))] == Vc[b, t, h, d]
    # per-sequence steps: each sequence writes at its own position only
    st2 = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table)
    tps = torch.tensor([5, 149, 64], dtype=torch.int32, device=DEV)
    ar = torch.arange(B, device=DEV)
    st2.append(Kd[ar, tps.long()].contiguous(), Vd[ar, tps.long()].contiguous(), 149, tps)
    kg2, _ = st2.gather(0, steps)
    for b in range(B):
        assert torch.equal(kg2[b, int(tps[b])], Kd[b, int(tps[b])])
        assert int((kg2[b] != 0).any(dim=-1).any(dim=-1).sum()) == 1


# ----------------------------------------------------------------------------
# Tiny causal decode, fp32, every step (append then attend).
# ----------------------------------------------------------------------------
def test_tiny_causal_fp32_every_step():
    B, Hq, Hkv, D, Z, steps = 1, 8, 2, 64, 64, 512
    dtype = T.TEMPO_F32
    q, K, V = host_inputs(1, B, steps, Hq, Hkv, D, dtype)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, fill="nan")
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    outs = torch.empty((steps, B, Hq, D), dtype=torch.float32, device=DEV)
    for t in range(steps):
        st.append(Kd[:, t].contiguous(), Vd[:, t].contiguous(), t)
        st.attend_causal(qd[t], outs[t], t)
    torch.cuda.synchronize()
    got = np64(outs)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for t in range(steps):
        ref = oracle.attend(q[t].astype(np.float64), K64, V64, t, 0, 1.0 / np.sqrt(D))
        assert_close(got[t], ref, dtype, f"fp32 causal t={t}")
    # t = 0 is exactly V[0] (softmax over one key)
    assert np.array_equal(got[0][0, :4], np.broadcast_to(V64[0, 0, 0], (4, D)))


# ----------------------------------------------------------------------------
# bf16, small batch, every step: causal and several windows, tiles of 64 with a
# ragged tail, window fronts cutting through the middle of a 32-slot group.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("window", [0, 1, 2, 50, 51, 64, 65, 97])
def test_bf16_every_step_causal_and_window(window):
    B, Hq, Hkv, D, Z, steps = 2, 6, 2, 128, 64, 230
    dtype = T.TEMPO_BF16
    q, K, V = host_inputs(2, B, steps, Hq, Hkv, D, dtype)
    table, nb = random_table(2, B, steps // Z + 1)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    outs = torch.empty((steps, B, Hq, D), dtype=torch.bfloat16, device=DEV)
    for t in range(steps):
        st.append(Kd[:, t].contiguous(), Vd[:, t].contiguous(), t)
        if window:
            st.attend_window(qd[t], outs[t], t, window)
        else:
            st.attend_causal(qd[t], outs[t], t)
    torch.cuda.synchronize()
    got = np64(outs)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for t in range(steps):
        ref = oracle.attend(q[t].astype(np.float64), K64, V64, t, window, 1.0 / np.sqrt(D))
        assert_close(got[t], ref, dtype, f"bf16 window={window} t={t}")


@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("G", [1, 2, 3, 4, 5, 8, 16, 17, 24, 32, 71, 128])
def test_group_sizes_and_head_dims(dtype, D, G):
    B, Hkv, Z, steps = 2, 2, 32, 140
    Hq = Hkv * G
    q, K, V = host_inputs(3 + G, B, steps, Hq, Hkv, D, dtype)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, fill="nan")
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    st.prefill(Kd, Vd, steps - 1)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for t, w in ((0, 0), (31, 0), (32, 0), (77, 0), (139, 0), (139, 40), (100, 33)):
        out = st.new_out()
        if w:
            st.attend_window(qd[t], out, t, w, scale=0.2)
        else:
            st.attend_causal(qd[t], out, t, scale=0.2)
        ref = oracle.attend(q[t].astype(np.float64), K64, V64, t, w, 0.2)
        assert_close(out, ref, dtype, f"G={G} D={D} t={t} w={w}")


# ----------------------------------------------------------------------------
# The result does not depend on pool contents outside the visible range.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
def test_poisoned_pool_gives_identical_bits(dtype):
    B, Hq, Hkv, D, Z, steps = 2, 6, 2, 128, 64, 200
    q, K, V = host_inputs(4, B, steps, Hq, Hkv, D, dtype)
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    results = []
    for fill in ("zero", "nan"):
        st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, fill=fill)
        outs = []
        for t in range(steps):
            st.append(Kd[:, t].contiguous(), Vd[:, t].contiguous(), t)
            if t in (0, 1, 30, 31, 32, 33, 63, 64, 65, 100, 127, 128, 199):
                for w in (0, 1, 7, 33, 70):
                    out = st.new_out()
                    if w:
                        st.attend_window(qd[t], out, t, w)
                    else:
                        st.attend_causal(qd[t], out, t)
                    outs.append(out)
        results.append(torch.stack(outs))
    assert torch.isfinite(results[1].float()).all()
    assert torch.equal(results[0], results[1])


# ----------------------------------------------------------------------------
# Ragged batch (per-sequence steps), random block table in a shared pool.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
@pytest.mark.parametrize("window", [0, 45])
def test_ragged_steps_random_block_table(dtype, window):
    B, Hq, Hkv, D, Z, T_len = 7, 6, 2, 128, 32, 300
    q, K, V = host_inputs(5, B, T_len, Hq, Hkv, D, dtype)
    lengths = np.array([1, 300, 33, 32, 150, 257, 2], dtype=np.int32)
    table, nb = random_table(5, B, (T_len - 1) // Z + 1)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    len_d = torch.from_numpy(lengths).to(DEV)
    st.prefill(Kd, Vd, T_len - 1, lengths=len_d)
    tps = (len_d - 1).to(torch.int32)
    qd = dev(q[0], dtype)
    out = st.new_out()
    if window:
        st.attend_window(qd, out, T_len - 1, window, t_per_seq=tps)
    else:
        st.attend_causal(qd, out, T_len - 1, t_per_seq=tps)
    ref = oracle.attend(q[0].astype(np.float64), K.astype(np.float64), V.astype(np.float64),
                        lengths - 1, window, 1.0 / np.sqrt(D))
    assert_close(out, ref, dtype, f"ragged window={window}")
    # a ragged call with all steps equal is the uniform call, bit for bit
    st2 = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, num_blocks=nb, block_table=table)
    st2.prefill(Kd, Vd, 200)
    a, b = st2.new_out(), st2.new_out()
    same = torch.full((B,), 200, dtype=torch.int32, device=DEV)
    st2.attend_causal(qd, a, 200)
    st2.attend_causal(qd, b, 200, t_per_seq=same)
    assert torch.equal(a, b)


# ----------------------------------------------------------------------------
# Ragged steps driven by a work list: the list holds exactly the non-empty (sequence, split)
# items, full splits first and the newest splits by falling size; the step gives the bits of
# the entry points without a list, and the oracle's values.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("B,Hq,Hkv,D,Z,T_len,window", [(7, 6, 2, 128, 32, 300, 0), (7, 6, 2, 128, 32, 300, 45),
                                                        (300, 2, 1, 64, 32, 2100, 0), (33, 8, 8, 64, 64, 5000, 1500)])
def test_ragged_work_list(B, Hq, Hkv, D, Z, T_len, window):
    dtype = T.TEMPO_BF16
    lengths = synth.integers(60 + B, 1, B, 1, T_len)
    lengths[0], lengths[-1] = 1, T_len
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, fill="nan")
    plain = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, fill="nan")
    K = synth.device_normal((B, T_len, Hkv, D), 6001, torch.bfloat16, DEV)
    V = synth.device_normal((B, T_len, Hkv, D), 6002, torch.bfloat16, DEV)
    q = synth.device_normal((B, Hq, D), 6003, torch.bfloat16, DEV)
    # every sequence holds its steps 0..L-2 (rows beyond are NaN in the store); the step appends L-1
    for s_ in (st, plain):
        for b in range(B):
            L = int(lengths[b])
            if L > 1:
                one = T.make_kv(s_.k_pool, s_.v_pool, s_.block_table[b:b + 1], s_.num_blocks, s_.max_blocks_per_seq,
                                Z, Hkv, D, dtype)
                T.tempo_kv_append_block(one, K[b:b + 1, :L - 1].contiguous(), V[b:b + 1, :L - 1].contiguous(), 1, 0,
                                        None, L - 1)
    tps = torch.from_numpy(lengths - 1).to(DEV).to(torch.int32)
    ar = torch.arange(B, device=DEV)
    k_t, v_t = K[ar, tps.long()].contiguous(), V[ar, tps.long()].contiguous()
    plan = T.tempo_attn_plan(st.kv, B, Hq, T_len - 1, window, True)
    worklist = st.build_worklist(T_len - 1, tps, window)
    torch.cuda.synchronize()
    # the list, item by item
    wl = worklist.cpu().numpy()
    tps_ = plan.tokens_per_split
    want, newest = set(), {}
    for b in range(B):
        t_b = int(lengths[b]) - 1
        lo = max(0, t_b - window + 1) if window else 0
        n = t_b // tps_ - lo // tps_ + 1
        assert n <= plan.num_splits
        want |= {(b, s_) for s_ in range(n)}
        newest[b] = (n - 1, t_b - max(lo, (t_b // tps_) * tps_) + 1)
    count = int(wl[0])
    items = [(int(x) & 0xFFFF, int(x) >> 16) for x in wl[1:1 + count]]
    assert count == len(want) and set(items) == want and len(set(items)) == count
    n_full = count - B
    assert all(s_ < newest[b][0] for b, s_ in items[:n_full])            # full splits first
    tail_classes = [7 - ((newest[b][1] - 1) * 8) // tps_ for b, s_ in items[n_full:]]
    assert all(s_ == newest[b][0] for b, s_ in items[n_full:])
    assert tail_classes == sorted(tail_classes)                           # then the newest splits, longest class first
    # the step: same bits as without a list, the oracle's values, the same store
    out = st.step_ragged(q, k_t, v_t, st.new_out(), T_len - 1, tps, worklist, window)
    if window:
        ref_out = plain.step_window(q, k_t, v_t, plain.new_out(), T_len - 1, window, t_per_seq=tps)
    else:
        ref_out = plain.step_causal(q, k_t, v_t, plain.new_out(), T_len - 1, t_per_seq=tps)
    torch.cuda.synchronize()
    assert torch.equal(out, ref_out)
    assert torch.equal(st.k_pool.view(torch.int16), plain.k_pool.view(torch.int16))
    assert torch.equal(st.v_pool.view(torch.int16), plain.v_pool.view(torch.int16))
    ref = oracle.attend(np64(q), np64(K), np64(V), lengths - 1, window, 1.0 / np.sqrt(D))
    assert_close(out, ref, dtype, f"ragged step with a work list, window={window}")
    # attention only (the store already holds the steps): k_new = v_new = None
    again = st.step_ragged(q, None, None, st.new_out(), T_len - 1, tps, worklist, window)
    assert torch.equal(again, out)


# ----------------------------------------------------------------------------
# The padded + masked baseline gives the same result as the dynamic range at every
# step, while the pool beyond the step holds NaN (masking is by index).
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("B,t_pad", [(2, 229), (1, 699)])
def test_padded_baseline_matches_oracle_every_step(B, t_pad):
    Hq, Hkv, D, Z = 6, 2, 128, 64
    steps = t_pad + 1
    dtype = T.TEMPO_BF16
    q, K, V = host_inputs(6, B, steps, Hq, Hkv, D, dtype)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, fill="nan")
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    todo = list(range(steps)) if B == 2 else list(range(0, steps, 7)) + [steps - 1]
    outs = torch.empty((steps, B, Hq, D), dtype=torch.bfloat16, device=DEV)
    for t in range(steps):
        st.append(Kd[:, t].contiguous(), Vd[:, t].contiguous(), t)
        if t in todo:
            st.attend_padded(qd[t], outs[t], t, t_pad)
    torch.cuda.synchronize()
    got = np64(outs)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for t in todo:
        ref = oracle.attend(q[t].astype(np.float64), K64, V64, t, 0, 1.0 / np.sqrt(D))
        assert_close(got[t], ref, dtype, f"padded baseline t={t} of {t_pad}")
    # per-sequence steps under one padding bound
    tps = torch.tensor([t_pad // 3, 5][:B], dtype=torch.int32, device=DEV)
    out = st.attend_padded(qd[0], st.new_out(), t_pad, t_pad, t_per_seq=tps)
    ref = oracle.attend(q[0].astype(np.float64), K64, V64, tps.cpu().numpy(), 0, 1.0 / np.sqrt(D))
    assert_close(out, ref, dtype, "padded baseline, per-sequence steps")
    with pytest.raises(T.TempoError):
        st.attend_padded(qd[0], st.new_out(), 10, 9)             # padding bound below the step
    with pytest.raises(T.TempoError):
        st.attend_padded(qd[0], st.new_out(), 10, st.max_t + 1)  # beyond the store


# ----------------------------------------------------------------------------
# Any valid split plan gives the same result within tolerance; same plan, same bits.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
def test_explicit_plans_and_determinism(dtype):
    B, Hq, Hkv, D, Z, steps = 2, 6, 2, 128, 128, 700
    q, K, V = host_inputs(6, B, steps, Hq, Hkv, D, dtype)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, fill="nan")
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    st.prefill(Kd, Vd, steps - 1)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for t, w in ((699, 0), (699, 300), (415, 0), (31, 0)):
        ref = oracle.attend(q[t].astype(np.float64), K64, V64, t, w, 1.0 / np.sqrt(D))
        lo = 0 if w == 0 else max(0, t - w + 1)
        for tps in (32, 64, 128, 256, 512, 1024):
            for waves in (1, 2, 4, 8):
                plan = T.tempo_plan(tps, t // tps - lo // tps + 1, waves)
                out = st.new_out()
                st.attend_with_plan(qd[t], out, t, plan, window=w)
                assert_close(out, ref, dtype, f"plan tps={tps} waves={waves} t={t} w={w}")
                again = st.new_out()
                st.attend_with_plan(qd[t], again, t, plan, window=w)
                assert torch.equal(out, again)


# ----------------------------------------------------------------------------
# One-launch decode step (append fused into the attention kernel) against the
# oracle and, bit for bit, against the separate append + attend calls.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
@pytest.mark.parametrize("window", [0, 37])
def test_fused_step_equals_append_then_attend(dtype, window):
    B, Hq, Hkv, D, Z, steps = 3, 6, 2, 128, 64, 200
    q, K, V = host_inputs(8, B, steps, Hq, Hkv, D, dtype)
    table, nb = random_table(8, B, steps // Z + 1)
    fused = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    plain = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    of = torch.empty((steps, B, Hq, D), dtype=TDT[dtype], device=DEV)
    op = torch.empty_like(of)
    for t in range(steps):
        k_t, v_t = Kd[:, t].contiguous(), Vd[:, t].contiguous()
        plain.append(k_t, v_t, t)
        if window:
            plain.attend_window(qd[t], op[t], t, window)
            fused.step_window(qd[t], k_t, v_t, of[t], t, window)
        else:
            plain.attend_causal(qd[t], op[t], t)
            fused.step_causal(qd[t], k_t, v_t, of[t], t)
    torch.cuda.synchronize()
    assert torch.equal(of, op)
    kf, vf = fused.gather(0, steps)
    assert torch.equal(kf, Kd) and torch.equal(vf, Vd)
    got = np64(of)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for t in range(0, steps, 7):
        ref = oracle.attend(q[t].astype(np.float64), K64, V64, t, window, 1.0 / np.sqrt(D))
        assert_close(got[t], ref, dtype, f"fused step window={window} t={t}")


@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
def test_fused_step_ragged(dtype):
    B, Hq, Hkv, D, Z, T_len = 5, 8, 2, 64, 32, 260
    q, K, V = host_inputs(9, B, T_len, Hq, Hkv, D, dtype)
    lengths = np.array([1, 260, 33, 97, 160], dtype=np.int32)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, fill="nan")
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    len_d = torch.from_numpy(lengths).to(DEV)
    # every sequence holds steps 0..len-2; the fused step appends step len-1 and attends
    st.prefill(Kd, Vd, T_len - 2, lengths=torch.clamp(len_d - 1, min=1))
    tps = (len_d - 1).to(torch.int32)
    ar = torch.arange(B, device=DEV)
    k_t, v_t = Kd[ar, tps.long()].contiguous(), Vd[ar, tps.long()].contiguous()
    qd = dev(q[0], dtype)
    out = st.step_causal(qd, k_t, v_t, st.new_out(), T_len - 1, t_per_seq=tps)
    ref = oracle.attend(q[0].astype(np.float64), K.astype(np.float64), V.astype(np.float64),
                        lengths - 1, 0, 1.0 / np.sqrt(D))
    assert_close(out, ref, dtype, "fused ragged step")
    kg, vg = st.gather(0, T_len)
    for b in range(B):
        L = int(lengths[b])
        assert torch.equal(kg[b, :L], Kd[b, :L]) and torch.equal(vg[b, :L], Vd[b, :L])


# ----------------------------------------------------------------------------
# Window store: a ring of R blocks per sequence, reused in turn, answers windowed
# decode for any number of steps in constant memory -- same bits as the linear
# store, and the oracle's values.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,Z,R,window", [(T.TEMPO_BF16, 64, 4, 150), (T.TEMPO_BF16, 32, 2, 33),
                                              (T.TEMPO_F32, 16, 4, 40), (T.TEMPO_BF16, 64, 4, 193)])
@pytest.mark.parametrize("fused", [False, True])
def test_ring_store_windowed_decode(dtype, Z, R, window, fused):
    B, Hq, Hkv, D, steps = 2, 6, 2, 128, 700
    # the ring is the size the library's own helper gives for this window; one more key needs twice as much
    assert T.tempo_ring_blocks(window, Z) == R
    assert T.tempo_ring_blocks((R - 1) * Z + 1, Z) == R and T.tempo_ring_blocks((R - 1) * Z + 2, Z) == 2 * R
    q, K, V = host_inputs(12, B, steps, Hq, Hkv, D, dtype)
    ring_table = torch.from_numpy(synth.permutation(12, 3, B * R).reshape(B, R).copy())
    ring = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=B * R, block_table=ring_table,
                      fill="nan", ring_blocks=R)
    flat = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, fill="nan")
    assert ring.k_pool.numel() == B * R * Hkv * Z * D          # constant memory
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    o_ring = torch.empty((steps, B, Hq, D), dtype=TDT[dtype], device=DEV)
    o_flat = torch.empty_like(o_ring)
    for t in range(steps):
        k_t, v_t = Kd[:, t].contiguous(), Vd[:, t].contiguous()
        if fused:
            ring.step_window(qd[t], k_t, v_t, o_ring[t], t, window)
            flat.step_window(qd[t], k_t, v_t, o_flat[t], t, window)
        else:
            ring.append(k_t, v_t, t)
            flat.append(k_t, v_t, t)
            ring.attend_window(qd[t], o_ring[t], t, window)
            flat.attend_window(qd[t], o_flat[t], t, window)
    torch.cuda.synchronize()
    assert torch.equal(o_ring, o_flat)
    got = np64(o_ring)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    for t in list(range(0, steps, 13)) + [R * Z - 1, R * Z, R * Z + 1, steps - 1]:
        ref = oracle.attend(q[t].astype(np.float64), K64, V64, t, window, 1.0 / np.sqrt(D))
        assert_close(got[t], ref, dtype, f"ring store t={t}")
    # the ring holds the last R*Z steps at most; the newest ones read back exactly
    kg, vg = ring.gather(steps - Z, Z)
    assert torch.equal(kg, Kd[:, steps - Z:]) and torch.equal(vg, Vd[:, steps - Z:])
    # a window the ring cannot hold any more is refused, not answered wrongly
    with pytest.raises(T.TempoError):
        ring.attend_window(qd[0], ring.new_out(), steps - 1, (R - 1) * Z + 2)
    with pytest.raises(T.TempoError):
        ring.attend_causal(qd[0], ring.new_out(), steps - 1)


# ----------------------------------------------------------------------------
# Inferred deallocation on a linear store: the host frees the blocks that
# tempo_kv_release reports dead, poisons them, and hands them to the tiles opened
# later (other sequences' included).  Windowed decode of any length then lives in
# a pool of a few blocks per sequence, and never reads a released block.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype,Z,window", [(T.TEMPO_BF16, 32, 70), (T.TEMPO_F32, 8, 9), (T.TEMPO_BF16, 64, 64)])
def test_linear_store_recycles_released_blocks(dtype, Z, window):
    B, Hq, Hkv, D, steps = 3, 4, 2, 64, 400
    q, K, V = host_inputs(14, B, steps, Hq, Hkv, D, dtype)
    live_tiles = (window - 2 + Z) // Z + 1 if window > 1 else 1   # most tiles a range touches
    nb = B * (live_tiles + 1)                                      # one spare per sequence for the tile being opened
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb,
                    block_table=torch.zeros((B, (steps - 1) // Z + 1), dtype=torch.int32), fill="nan")
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    free = list(range(nb))
    owner = {}                                                     # (b, tile) -> physical block
    released = 0
    out = torch.empty((steps, B, Hq, D), dtype=TDT[dtype], device=DEV)
    for t in range(steps):
        if t % Z == 0:                                             # a new tile opens: take blocks off the free list
            for b in range(B):
                owner[(b, t // Z)] = free.pop(0)
                st.block_table[b, t // Z] = owner[(b, t // Z)]
        st.step_window(qd[t], Kd[:, t].contiguous(), Vd[:, t].contiguous(), out[t], t, window)
        dead_keys, dead_tiles = T.tempo_kv_release(t, window, Z)
        for n in range(released, dead_tiles):                      # newly dead tiles: poison, then free
            for b in range(B):
                blk = owner.pop((b, n))
                st.k_pool[blk] = float("nan")
                st.v_pool[blk] = float("nan")
                st.block_table[b, n] = nb - 1 - b                  # a stale entry must not matter either
                free.append(blk)
        released = max(released, dead_tiles)
        assert len(owner) <= B * (live_tiles + 1)
    torch.cuda.synchronize()
    assert released == (steps - 1 - window + 2) // Z > 0
    got = np64(out)
    for t in list(range(0, steps, 7)) + [steps - 1]:
        ref = oracle.attend(q[t].astype(np.float64), K64, V64, t, window, 1.0 / np.sqrt(D))
        assert_close(got[t], ref, dtype, f"recycled linear store t={t} window={window}")


# ----------------------------------------------------------------------------
# Full-size workloads, in the launch configuration the benchmark times.
# Keys/values are drawn on the GPU (seeded), appended through the ABI, and the
# oracle reads the same values back from the flat tensors.
# ----------------------------------------------------------------------------
def flat_kv(seed, B, T_len, Hkv, D):
    K = synth.device_normal((B, T_len, Hkv, D), seed * 10 + 1, torch.bfloat16, DEV)
    V = synth.device_normal((B, T_len, Hkv, D), seed * 10 + 2, torch.bfloat16, DEV)
    return K, V


def test_llama_shape_causal_bf16_full_size():
    B, Hq, Hkv, D, Z, T_len = 16, 24, 8, 128, 256, 4096
    dtype = T.TEMPO_BF16
    K, V = flat_kv(21, B, T_len, Hkv, D)
    table, nb = random_table(21, B, T_len // Z, extra=0)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    st.prefill(K, V, T_len - 2)
    K64, V64 = np64(K), np64(V)
    # the benchmark's own launch: the fused step at t = 4095 (append + partial + combine)
    t = T_len - 1
    q = synth.device_normal((B, Hq, D), 2100 + t, torch.bfloat16, DEV)
    out = st.step_causal(q, K[:, t].contiguous(), V[:, t].contiguous(), st.new_out(), t)
    ref = oracle.attend(np64(q), K64, V64, t, 0, 1.0 / np.sqrt(D))
    assert_close(out, ref, dtype, "llama causal fused step t=4095")
    plan = T.tempo_attn_plan(st.kv, B, Hq, t, 0)
    assert (plan.tokens_per_split, plan.num_splits, plan.waves) == (2048, 2, 8)
    kg, vg = st.gather(t, 1)
    assert torch.equal(kg[:, 0], K[:, t]) and torch.equal(vg[:, 0], V[:, t])
    # every step with t mod 256 in {0, 1, 254, 255}, every 16th step, and a few more
    steps = sorted({t for t in range(T_len) if t % 256 in (0, 1, 254, 255)} | set(range(0, T_len, 16)) |
                   {31, 32, 257, 1000, 2047, 2048, 3000, 4094, 4095})
    for t in steps:
        q = synth.device_normal((B, Hq, D), 2100 + t, torch.bfloat16, DEV)
        out = st.attend_causal(q, st.new_out(), t)
        ref = oracle.attend(np64(q), K64, V64, t, 0, 1.0 / np.sqrt(D))    # reads keys 0..t only
        assert_close(out, ref, dtype, f"llama causal t={t}")


def test_llama_shape_causal_bf16_full_size_every_step_appended():
    # The whole causal workload the way a decoder runs it: t = 0 .. 4095, each step through the fused
    # entry point (block-store write of step t + attention over 0..t in one call), no prefill.
    B, Hq, Hkv, D, Z, T_len = 16, 24, 8, 128, 256, 4096
    dtype = T.TEMPO_BF16
    K, V = flat_kv(25, B, T_len, Hkv, D)
    table, nb = random_table(25, B, T_len // Z, extra=0)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    Q = synth.device_normal((T_len, B, Hq, D), 2500, torch.bfloat16, DEV)
    Kt, Vt = K.transpose(0, 1).contiguous(), V.transpose(0, 1).contiguous()      # [T][B][Hkv][D]
    outs = torch.empty_like(Q)
    for t in range(T_len):
        st.step_causal(Q[t], Kt[t], Vt[t], outs[t], t)
    torch.cuda.synchronize()
    # the store now holds exactly the flat keys/values, bit for bit
    kg, vg = st.gather(0, T_len)
    assert torch.equal(kg, K) and torch.equal(vg, V)
    del kg, vg, Kt, Vt
    assert torch.isfinite(outs.float()).all()
    # every step with t mod 256 in {0, 1, 254, 255}, every 16th step, and a few more
    steps = sorted({t for t in range(T_len) if t % 256 in (0, 1, 254, 255)} | set(range(0, T_len, 16)) |
                   {31, 32, 257, 1000, 2047, 2048, 3000, 4094, 4095})
    K64, V64 = np64(K), np64(V)
    Q64, got = np64(Q[steps]), np64(outs[steps])
    for i, t in enumerate(steps):
        ref = oracle.attend(Q64[i], K64, V64, t, 0, 1.0 / np.sqrt(D))             # reads keys 0..t only
        assert_close(got[i], ref, dtype, f"llama causal, appended step by step, t={t}")


def test_head_dim_64_shape_causal_bf16_full_size():
    # The other head size the library serves, at a real shape (32 query heads in groups of 4, head_dim 64,
    # the attention layer of the 1B model of the same family): fused steps at sampled t, append checked.
    B, Hq, Hkv, D, Z, T_len = 16, 32, 8, 64, 256, 4096
    dtype = T.TEMPO_BF16
    K, V = flat_kv(27, B, T_len, Hkv, D)
    table, nb = random_table(27, B, T_len // Z, extra=0)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    K64, V64 = np64(K), np64(V)
    steps = [0, 1, 31, 32, 255, 256, 257, 1000, 2047, 2048, 3000, 4094, 4095]
    done = -1
    for t in steps:
        if t - 1 > done:
            st.append_block(K[:, done + 1:t].contiguous(), V[:, done + 1:t].contiguous(), done + 1, t - 1 - done)
        q = synth.device_normal((B, Hq, D), 2700 + t, torch.bfloat16, DEV)
        out = st.step_causal(q, K[:, t].contiguous(), V[:, t].contiguous(), st.new_out(), t)
        done = t
        ref = oracle.attend(np64(q), K64, V64, t, 0, 1.0 / np.sqrt(D))
        assert_close(out, ref, dtype, f"head_dim 64 causal fused step t={t}")
    kg, vg = st.gather(0, T_len)
    assert torch.equal(kg, K) and torch.equal(vg, V)
    # the same store through the window pattern and a block of 4 steps (16 columns)
    for t, w in ((4095, 512), (3000, 77)):
        q = synth.device_normal((B, Hq, D), 2750 + t, torch.bfloat16, DEV)
        out = st.attend_window(q, st.new_out(), t, w)
        assert_close(out, oracle.attend(np64(q), K64, V64, t, w, 1.0 / np.sqrt(D)), dtype, f"head_dim 64 window t={t}")
    qb = synth.device_normal((B, 4, Hq, D), 2790, torch.bfloat16, DEV)
    ob = st.attend_block(qb, torch.empty_like(qb), 4092, 4)
    for c in range(4):
        ref = oracle.attend(np64(qb[:, c]), K64, V64, 4092 + c, 0, 1.0 / np.sqrt(D))
        assert_close(ob[:, c], ref, dtype, f"head_dim 64 block step {c}")


def test_llama_shape_window_bf16_full_size():
    B, Hq, Hkv, D, Z, T_len, w = 16, 24, 8, 128, 256, 16384, 512
    dtype = T.TEMPO_BF16
    K, V = flat_kv(22, B, T_len, Hkv, D)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, fill="nan")
    st.prefill(K, V, T_len - 1)
    K64, V64 = np64(K), np64(V)
    # every step below 1100, every block boundary and its neighbours, a seeded sample of 256 steps
    steps = set(range(1100)) | {t for k in range(1, T_len // Z) for t in (k * Z - 1, k * Z, k * Z + 1)}
    steps |= {int(x) for x in synth.integers(22, 5, 256, 0, T_len - 1)} | {5000, 8191, 8192, T_len - 1}
    for t in sorted(steps):
        if t % 97 == 0:
            r = T.tempo_visible_range(t, w, Z)
            assert r == {k: v for k, v in oracle.visible_range(t, w, Z).items() if k in r}
        q = synth.device_normal((B, Hq, D), 2200 + t, torch.bfloat16, DEV)
        out = st.attend_window(q, st.new_out(), t, w)
        ref = oracle.attend(np64(q), K64, V64, t, w, 1.0 / np.sqrt(D))    # reads its window only
        assert_close(out, ref, dtype, f"llama window t={t}")


def test_llama_shape_window_bf16_full_size_ring_store_every_step_appended():
    # The window workload on the window store: a ring of tempo_ring_blocks(512, 256) blocks per
    # sequence (constant memory), t = 0 .. 16383, each step through the fused entry point.
    B, Hq, Hkv, D, Z, T_len, w = 16, 24, 8, 128, 256, 16384, 512
    dtype = T.TEMPO_BF16
    R = T.tempo_ring_blocks(w, Z)
    need = oracle.ring_blocks(w, Z)
    assert R >= need and R & (R - 1) == 0 and R // 2 < need        # the oracle's count, rounded up by the library
    K, V = flat_kv(26, B, T_len, Hkv, D)
    ring_table = torch.from_numpy(synth.permutation(26, 3, B * R).reshape(B, R).copy())
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, num_blocks=B * R, block_table=ring_table,
                    fill="nan", ring_blocks=R)
    assert st.k_pool.numel() == B * R * Hkv * Z * D                 # R blocks per sequence, whatever T is
    Q = synth.device_normal((T_len, B, Hq, D), 2600, torch.bfloat16, DEV)
    Kt, Vt = K.transpose(0, 1).contiguous(), V.transpose(0, 1).contiguous()
    outs = torch.empty_like(Q)
    for t in range(T_len):
        st.step_window(Q[t], Kt[t], Vt[t], outs[t], t, w)
    torch.cuda.synchronize()
    kg, vg = st.gather(T_len - w, w)                                 # the last window reads back exactly
    assert torch.equal(kg, K[:, T_len - w:]) and torch.equal(vg, V[:, T_len - w:])
    del kg, vg, Kt, Vt
    assert torch.isfinite(outs.float()).all()
    # every step below 1100, every block boundary and its neighbours, a seeded sample of 256 steps
    steps = set(range(1100)) | {t for k in range(1, T_len // Z) for t in (k * Z - 1, k * Z, k * Z + 1)}
    steps |= {int(x) for x in synth.integers(26, 5, 256, 0, T_len - 1)} | {5000, 8191, 8192, T_len - 1}
    steps = sorted(steps)
    K64, V64 = np64(K), np64(V)
    Q64, got = np64(Q[steps]), np64(outs[steps])
    for i, t in enumerate(steps):
        ref = oracle.attend(Q64[i], K64, V64, t, w, 1.0 / np.sqrt(D))             # reads its window only
        assert_close(got[i], ref, dtype, f"llama window on a ring, appended step by step, t={t}")


def test_long_single_sequence_bf16_full_size():
    B, Hq, Hkv, D, Z, T_len = 1, 24, 8, 128, 256, 65536
    dtype = T.TEMPO_BF16
    K, V = flat_kv(23, B, T_len, Hkv, D)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, fill="nan")
    st.prefill(K, V, T_len - 1)
    K64, V64 = np64(K), np64(V)
    for t, strict_tps in ((8191, 32), (32767, 128), (65535, 256)):
        q = synth.device_normal((B, Hq, D), 2300 + t, torch.bfloat16, DEV)
        ref = oracle.attend(np64(q), K64[:, :t + 1], V64[:, :t + 1], t, 0, 1.0 / np.sqrt(D))
        plan = T.tempo_attn_plan(st.kv, B, Hq, t, 0)
        assert plan.num_splits * Hkv >= 256          # at least 256 partial-attention work items
        out = st.attend_causal(q, st.new_out(), t)
        assert_close(out, ref, dtype, f"long t={t} default plan")
        strict = T.tempo_plan(strict_tps, (t + 1) // strict_tps, 1 if strict_tps == 32 else 4)
        assert strict.num_splits >= 256               # at least 256 partitions along the sequence
        out = st.attend_with_plan(q, st.new_out(), t, strict)
        assert_close(out, ref, dtype, f"long t={t} 256-way plan")


@pytest.mark.timeout(900)
def test_ragged_multi_layer_shared_pool_bf16():
    # The ragged multi-layer workload at its real shape: 28 layers, batch 64, lengths uniform in
    # [1, 8192], ONE shared pool that holds exactly the blocks the sequences need (about 30 GiB), a
    # random block table per layer.  One decode step = per layer, the fused ragged step (append
    # step L-1, attend over 0..L-1).  Every layer and every sequence is compared with the oracle.
    layers, B, Hq, Hkv, D, Z, T_max = 28, 64, 24, 8, 128, 256, 8192
    dtype = T.TEMPO_BF16
    lengths = synth.integers(24, 1, B, 1, T_max)
    lengths[0], lengths[1] = 1, T_max                    # both extremes are present
    need = (lengths.astype(np.int64) + Z - 1) // Z       # blocks per sequence
    per_layer = int(need.sum())
    nb = layers * per_layer
    perm = synth.permutation(24, 2, nb)
    shape = (nb, Hkv, Z * D)
    k_pool = torch.full(shape, float("nan"), dtype=torch.bfloat16, device=DEV)
    v_pool = torch.full(shape, float("nan"), dtype=torch.bfloat16, device=DEV)
    len_d = torch.from_numpy(lengths).to(DEV)
    tps = (len_d - 1).to(torch.int32)
    ar = torch.arange(B, device=DEV)
    # the oracle's fp64 inputs travel through two reused pinned host buffers
    pin_k = torch.empty((B, T_max, Hkv, D), dtype=torch.float64, pin_memory=True)
    pin_v = torch.empty_like(pin_k, pin_memory=True)
    stores, flats, outs = [], [], []
    for layer in range(layers):
        table = np.full((B, T_max // Z), -1, dtype=np.int32)        # entries beyond a sequence's blocks are never read
        ids = perm[layer * per_layer:(layer + 1) * per_layer]
        pos = 0
        for b in range(B):
            table[b, :need[b]] = ids[pos:pos + need[b]]
            pos += int(need[b])
        st = BlockStore(B, Hq, Hkv, D, Z, T_max - 1, dtype, num_blocks=nb, block_table=torch.from_numpy(table),
                        pools=(k_pool, v_pool))
        K, V = flat_kv(240 + layer, B, T_max, Hkv, D)
        # every sequence holds its steps 0..L-2 (one block-store write per sequence through a
        # one-sequence view of the same store); the step itself appends step L-1
        for b in range(B):
            L = int(lengths[b])
            if L > 1:
                one = T.make_kv(k_pool, v_pool, st.block_table[b:b + 1], nb, st.max_blocks_per_seq, Z, Hkv, D, dtype)
                T.tempo_kv_append_block(one, K[b:b + 1, :L - 1].contiguous(), V[b:b + 1, :L - 1].contiguous(), 1, 0,
                                        None, L - 1)
        stores.append(st)
        flats.append((K, V))
    # the step: all 28 layers, one fused call each
    qs = [synth.device_normal((B, Hq, D), 2400 + layer, torch.bfloat16, DEV) for layer in range(layers)]
    worklist = stores[0].build_worklist(T_max - 1, tps)            # one list serves every layer of the step
    for layer, st in enumerate(stores):
        K, V = flats[layer]
        k_t, v_t = K[ar, tps.long()].contiguous(), V[ar, tps.long()].contiguous()
        if layer % 2:                                              # odd layers: the launch driven by the work list
            outs.append(st.step_ragged(qs[layer], k_t, v_t, st.new_out(), T_max - 1, tps, worklist))
        else:
            outs.append(st.step_causal(qs[layer], k_t, v_t, st.new_out(), T_max - 1, t_per_seq=tps))
    torch.cuda.synchronize()
    for layer, st in enumerate(stores):
        K, V = flats[layer]
        pin_k.copy_(K.double())
        pin_v.copy_(V.double())
        torch.cuda.synchronize()
        ref = oracle.attend(np64(qs[layer]), pin_k.numpy(), pin_v.numpy(), lengths - 1, 0, 1.0 / np.sqrt(D))
        assert_close(outs[layer], ref, dtype, f"ragged step, layer {layer}, all {B} sequences")
        # the appended step is in the store (a short, a median and the longest sequence)
        for b in (0, 1, int(np.argsort(lengths)[B // 2])):
            L = int(lengths[b])
            one = T.make_kv(k_pool, v_pool, st.block_table[b:b + 1], nb, st.max_blocks_per_seq, Z, Hkv, D, dtype)
            kg = torch.empty((1, 1, Hkv, D), dtype=torch.bfloat16, device=DEV)
            vg = torch.empty_like(kg)
            T.tempo_kv_gather(one, kg, vg, 1, L - 1, 1)
            assert torch.equal(kg[0, 0], K[b, L - 1]) and torch.equal(vg[0, 0], V[b, L - 1])
        flats[layer] = None
        del K, V
        print(f"ragged multi-layer: layer {layer} matches the oracle", flush=True)


# ----------------------------------------------------------------------------
# The entry points allocate nothing and never synchronise, so a step can be
# captured in a HIP graph; every replay must give the eager result.
# ----------------------------------------------------------------------------
def test_step_replayed_from_a_hip_graph():
    B, Hq, Hkv, D, Z, T_len = 4, 12, 4, 128, 64, 600
    dtype = T.TEMPO_BF16
    q, K, V = host_inputs(10, B, T_len, Hq, Hkv, D, dtype)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, fill="nan")
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    t = T_len - 1
    st.prefill(Kd, Vd, t - 1)
    k_t, v_t = Kd[:, t].contiguous(), Vd[:, t].contiguous()
    q_buf = qd[0].clone()
    eager = st.step_causal(q_buf, k_t, v_t, st.new_out(), t).clone()
    assert T.tempo_attn_plan(st.kv, B, Hq, t, 0).num_splits > 1      # partial + combine are both captured
    out = st.new_out()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        st.step_causal(q_buf, k_t, v_t, out, t)                       # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    with torch.cuda.graph(graph):
        st.step_causal(q_buf, k_t, v_t, out, t)
    for rep in range(4):
        out.zero_()
        q_buf.copy_(qd[rep % 2])                                       # new query, same graph
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = st.step_causal(qd[rep % 2], k_t, v_t, st.new_out(), t)
        assert torch.equal(out, want)
    ref = oracle.attend(q[0].astype(np.float64), K.astype(np.float64), V.astype(np.float64), t, 0,
                        1.0 / np.sqrt(D))
    assert_close(eager, ref, dtype, "graph test eager")


def test_ragged_step_with_work_list_replayed_from_a_hip_graph():
    # The list is built once (outside the graph); the captured ragged step is replayed with new queries
    # and new key/value rows and must give the eager bits every time.
    B, Hq, Hkv, D, Z, T_len = 6, 12, 4, 128, 64, 900
    dtype = T.TEMPO_BF16
    q, K, V = host_inputs(15, B, T_len, Hq, Hkv, D, dtype)
    lengths = np.array([900, 1, 333, 640, 65, 512], dtype=np.int32)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, fill="nan")
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    len_d = torch.from_numpy(lengths).to(DEV)
    st.prefill(Kd, Vd, T_len - 2, lengths=torch.clamp(len_d - 1, min=1))
    tps = (len_d - 1).to(torch.int32)
    ar = torch.arange(B, device=DEV)
    k_t, v_t = Kd[ar, tps.long()].contiguous(), Vd[ar, tps.long()].contiguous()
    worklist = st.build_worklist(T_len - 1, tps)
    q_buf, out = qd[0].clone(), st.new_out()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        st.step_ragged(q_buf, k_t, v_t, out, T_len - 1, tps, worklist)     # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        st.step_ragged(q_buf, k_t, v_t, out, T_len - 1, tps, worklist)
    for rep in range(4):
        out.zero_()
        q_buf.copy_(qd[rep])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = st.step_causal(qd[rep], k_t, v_t, st.new_out(), T_len - 1, t_per_seq=tps)
        assert torch.equal(out, want)
    ref = oracle.attend(q[3].astype(np.float64), K.astype(np.float64), V.astype(np.float64), lengths - 1, 0,
                        1.0 / np.sqrt(D))
    assert_close(out, ref, dtype, "ragged step with a work list, replayed from a graph")
