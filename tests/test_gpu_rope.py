"""GPU parity of the rotary producer step (rotate, rotate-and-append, and the fully
fused rotate + append + attend launch) against the fp64 CPU oracle.

The cos / sin tables are an INPUT of the path: the tests take the oracle's fp64
table, round it to fp32 and hand it to the library.

Tolerances:
  rotation, fp32      |gpu - oracle| <= 1e-5 * max(1, max|oracle|)
  rotation, bf16      the stored bf16 value equals the oracle's fp64 value rounded to
                      bf16, or its neighbour (fp32 arithmetic rounds once more): at most
                      one bf16 step (2^-7 relative), and at least 99% of elements identical
  attention outputs   as test_gpu_parity.py (bf16 2e-2 / 1e-2 relative to the max, fp32 1e-5)
What the fused launch stores is compared bit for bit with the separate launches.
"""
import numpy as np
import pytest
import torch

from oracle import tempo_oracle as oracle
from paper_2501_05408_amd import synth
from paper_2501_05408_amd import tempo as T
from paper_2501_05408_amd.store import BlockStore

from test_gpu_parity import DEV, TDT, NAME, assert_close, dev, flat_kv, host_inputs, np64, random_table

pytestmark = pytest.mark.gpu

THETA = 500000.0


def tables(positions, D, theta=THETA):
    c, s = oracle.rope_table(positions, D, theta)
    return (torch.from_numpy(c.astype(np.float32)).to(DEV), torch.from_numpy(s.astype(np.float32)).to(DEV))


def assert_rotated(got, ref64, dtype, what):
    g = np64(got)
    assert np.isfinite(g).all(), what
    if dtype == T.TEMPO_F32:
        assert np.abs(g - ref64).max() <= 1e-5 * max(1.0, np.abs(ref64).max()), what
        return
    want = synth.round_to_bf16(ref64.astype(np.float32)).astype(np.float64)
    same = g == want
    assert same.mean() >= 0.99, f"{what}: only {same.mean():.4f} of the elements are the oracle's bf16 value"
    step = np.maximum(np.abs(want), 2.0 ** -126) * 2.0 ** -7
    assert (np.abs(g - want) <= step).all(), f"{what}: more than one bf16 step away"


def oracle_rotated_kv(q, K, dtype, t_of_row=None):
    """q [T][B][Hq][D] and K [B][T][Hkv][D] rotated to their own steps (fp64), then rounded to
    the storage dtype the way the producer rounds."""
    steps = K.shape[1]
    Kr = np.stack([oracle.rope(K[:, t].astype(np.float64), t, THETA) for t in range(steps)], axis=1)
    qr = np.stack([oracle.rope(q[t].astype(np.float64), t, THETA) for t in range(steps)], axis=0)
    if dtype == T.TEMPO_BF16:
        Kr = synth.round_to_bf16(Kr.astype(np.float32)).astype(np.float64)
        qr = synth.round_to_bf16(qr.astype(np.float32)).astype(np.float64)
    else:
        Kr = Kr.astype(np.float32).astype(np.float64)
        qr = qr.astype(np.float32).astype(np.float64)
    return qr, Kr


# ----------------------------------------------------------------------------
# Rotation alone, and rotation written straight into the block store.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
@pytest.mark.parametrize("D", [64, 128])
def test_rotate_and_rotate_append_match_oracle(dtype, D):
    B, Hq, Hkv, Z, steps = 3, 4, 2, 32, 140
    q, K, V = host_inputs(51, B, steps, Hq, Hkv, D, dtype)
    cos_t, sin_t = tables(steps, D)
    table, nb = random_table(51, B, steps // Z + 1)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    st.set_rope(cos_t, sin_t)
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    rot = torch.empty_like(Kd)
    for t in range(steps):
        st.rope_append(Kd[:, t].contiguous(), Vd[:, t].contiguous(), t)
        tmp = torch.empty((B, Hkv, D), dtype=TDT[dtype], device=DEV)
        st.rope_rotate(Kd[:, t].contiguous(), tmp, t)
        rot[:, t] = tmp
    kg, vg = st.gather(0, steps)
    assert torch.equal(kg.view(torch.uint8), rot.view(torch.uint8))        # store holds the rotation's bits
    assert torch.equal(vg, Vd)
    ref = np.stack([oracle.rope(K[:, t].astype(np.float64), t, THETA) for t in range(steps)], axis=1)
    assert_rotated(kg, ref, dtype, f"rotated keys D={D}")
    assert torch.equal(kg[:, 0], Kd[:, 0])                                  # position 0 is the identity
    # per-sequence positions, in place
    pos = [7, 139, 64]
    tps = torch.tensor(pos, dtype=torch.int32, device=DEV)
    x = dev(q[0], dtype).clone()
    st.rope_rotate(x, x, max(pos), tps)
    assert_rotated(x, oracle.rope(q[0].astype(np.float64), pos, THETA), dtype, "per-sequence positions, in place")
    with pytest.raises(T.TempoError):
        st.rope_rotate(x, x, steps)                                         # beyond the tables


# ----------------------------------------------------------------------------
# The fused launch (rotate q and k, append, attend) at every step: bit-identical
# to the three separate launches, and within tolerance of the oracle.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
@pytest.mark.parametrize("window", [0, 50])
@pytest.mark.parametrize("D", [64, 128])
def test_fused_rope_step_every_step(dtype, window, D):
    B, Hq, Hkv, Z, steps = 2, 6, 2, 32, 200
    q, K, V = host_inputs(52, B, steps, Hq, Hkv, D, dtype)
    cos_t, sin_t = tables(steps, D)
    table, nb = random_table(52, B, steps // Z + 1)
    fused = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    plain = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    fused.set_rope(cos_t, sin_t)
    plain.set_rope(cos_t, sin_t)
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    out_f = torch.empty((steps, B, Hq, D), dtype=TDT[dtype], device=DEV)
    out_p = torch.empty_like(out_f)
    for t in range(steps):
        k, v = Kd[:, t].contiguous(), Vd[:, t].contiguous()
        fused.rope_step(qd[t], k, v, out_f[t], t, window)
        plain.rope_append(k, v, t)
        qr = plain.rope_rotate(qd[t], torch.empty_like(qd[t]), t)
        if window:
            plain.attend_window(qr, out_p[t], t, window)
        else:
            plain.attend_causal(qr, out_p[t], t)
    torch.cuda.synchronize()
    assert torch.equal(fused.k_pool.view(torch.uint8), plain.k_pool.view(torch.uint8))
    assert torch.equal(fused.v_pool.view(torch.uint8), plain.v_pool.view(torch.uint8))
    assert torch.equal(out_f.view(torch.uint8), out_p.view(torch.uint8))
    qr64, Kr64 = oracle_rotated_kv(q, K, dtype)
    V64 = V.astype(np.float64)
    got = np64(out_f)
    for t in range(steps):
        ref = oracle.attend(qr64[t], Kr64, V64, t, window, 1.0 / np.sqrt(D))
        assert_close(got[t], ref, dtype, f"fused rope step t={t} w={window} D={D}")


# ----------------------------------------------------------------------------
# Groups of more than 16 query heads per key/value head (multi-query layouts): the
# step entry points write the store with a launch of their own and answer through
# the LDS-staged kernel.  Same checks as above, plus the plain fused step.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
@pytest.mark.parametrize("G,window", [(24, 0), (32, 45), (71, 0), (128, 70)])
def test_large_group_steps_every_step(dtype, G, window):
    B, Hkv, D, Z, steps = 2, 2, 128, 32, 150
    Hq = Hkv * G
    q, K, V = host_inputs(57 + G, B, steps, Hq, Hkv, D, dtype)
    cos_t, sin_t = tables(steps, D)
    table, nb = random_table(57, B, steps // Z + 1)
    fused = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    plain = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    unrot = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    fused.set_rope(cos_t, sin_t)
    plain.set_rope(cos_t, sin_t)
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    out_f = torch.empty((steps, B, Hq, D), dtype=TDT[dtype], device=DEV)
    out_p = torch.empty_like(out_f)
    out_u = torch.empty_like(out_f)
    for t in range(steps):
        k, v = Kd[:, t].contiguous(), Vd[:, t].contiguous()
        fused.rope_step(qd[t], k, v, out_f[t], t, window)
        plain.rope_append(k, v, t)
        qr = plain.rope_rotate(qd[t], torch.empty_like(qd[t]), t)
        if window:
            plain.attend_window(qr, out_p[t], t, window)
            unrot.step_window(qd[t], k, v, out_u[t], t, window)
        else:
            plain.attend_causal(qr, out_p[t], t)
            unrot.step_causal(qd[t], k, v, out_u[t], t)
    torch.cuda.synchronize()
    assert torch.equal(fused.k_pool.view(torch.uint8), plain.k_pool.view(torch.uint8))
    assert torch.equal(fused.v_pool.view(torch.uint8), plain.v_pool.view(torch.uint8))
    assert torch.equal(out_f.view(torch.uint8), out_p.view(torch.uint8))
    qr64, Kr64 = oracle_rotated_kv(q, K, dtype)
    K64, V64 = K.astype(np.float64), V.astype(np.float64)
    got, got_u = np64(out_f), np64(out_u)
    for t in range(steps):
        ref = oracle.attend(qr64[t], Kr64, V64, t, window, 1.0 / np.sqrt(D))
        assert_close(got[t], ref, dtype, f"large group rope step G={G} t={t} w={window}")
        ref = oracle.attend(q[t].astype(np.float64), K64, V64, t, window, 1.0 / np.sqrt(D))
        assert_close(got_u[t], ref, dtype, f"large group step G={G} t={t} w={window}")


# ----------------------------------------------------------------------------
# Per-sequence steps: each sequence is rotated to, written at and answered for
# its own position.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("dtype", [T.TEMPO_BF16, T.TEMPO_F32])
def test_fused_rope_step_ragged(dtype):
    B, Hq, Hkv, D, Z, steps = 5, 8, 2, 128, 64, 300
    q, K, V = host_inputs(53, B, steps, Hq, Hkv, D, dtype)
    cos_t, sin_t = tables(steps, D)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, fill="nan")
    st.set_rope(cos_t, sin_t)
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    last = [0, 299, 63, 64, 131]
    for t in range(steps):                      # history: every sequence up to (excluding) its last step
        tps = torch.tensor([min(t, l) for l in last], dtype=torch.int32, device=DEV)
        live = [b for b in range(B) if t < last[b]]
        if not live:
            break
        ar = torch.arange(B, device=DEV)
        st.rope_append(Kd[ar, tps.long()].contiguous(), Vd[ar, tps.long()].contiguous(), t, tps)
    tps = torch.tensor(last, dtype=torch.int32, device=DEV)
    ar = torch.arange(B, device=DEV)
    qb = torch.stack([qd[last[b], b] for b in range(B)]).contiguous()
    out = st.new_out()
    st.rope_step(qb, Kd[ar, tps.long()].contiguous(), Vd[ar, tps.long()].contiguous(), out, max(last), 0, tps)
    qr64, Kr64 = oracle_rotated_kv(q, K, dtype)
    qref = np.stack([qr64[last[b], b] for b in range(B)])
    ref = oracle.attend(qref, Kr64, V.astype(np.float64), np.array(last, dtype=np.int32), 0, 1.0 / np.sqrt(D))
    assert_close(out, ref, dtype, "ragged fused rope step")


# ----------------------------------------------------------------------------
# Large positions on a ring store (angles of ~1e5 radians), and the headline shape.
# ----------------------------------------------------------------------------
def test_fused_rope_step_large_positions_ring_bf16():
    # A ring store at positions around 1e5: the window's worth of history before the first answered
    # step is written with rotating appends, then every step goes through the fused rotary step.
    B, Hq, Hkv, D, Z, R, window, t0, n = 2, 6, 2, 128, 32, 4, 70, 100000, 120
    dtype = T.TEMPO_BF16
    hist = window - 1                                   # steps t0-hist .. t0-1 are history
    q, K, V = host_inputs(54, B, hist + n, Hq, Hkv, D, dtype)
    c, s = oracle.rope_table(t0 + n, D, THETA)
    cos_t = torch.from_numpy(c.astype(np.float32)).to(DEV)
    sin_t = torch.from_numpy(s.astype(np.float32)).to(DEV)
    st = BlockStore(B, Hq, Hkv, D, Z, 2 ** 30, dtype, ring_blocks=R, fill="nan")
    st.set_rope(cos_t, sin_t)
    qd, Kd, Vd = dev(q, dtype), dev(K, dtype), dev(V, dtype)
    first = t0 - hist                                   # position of row 0 of K, V
    Kr = np.stack([oracle.rope(K[:, i].astype(np.float64), first + i, THETA) for i in range(hist + n)], axis=1)
    Kr = synth.round_to_bf16(Kr.astype(np.float32)).astype(np.float64)
    V64 = V.astype(np.float64)
    for i in range(hist):
        st.rope_append(Kd[:, i].contiguous(), Vd[:, i].contiguous(), first + i)
    for i in range(hist, hist + n):
        out = st.rope_step(qd[i], Kd[:, i].contiguous(), Vd[:, i].contiguous(), st.new_out(), first + i, window)
        qr = synth.round_to_bf16(oracle.rope(q[i].astype(np.float64), first + i, THETA).astype(np.float32)).astype(np.float64)
        ref = oracle.attend(qr, Kr[:, :i + 1], V64[:, :i + 1], i, window, 1.0 / np.sqrt(D))
        assert_close(out, ref, dtype, f"ring rope step t={first + i}")


# ----------------------------------------------------------------------------
# Blocks with the rotary producer fused in: the rotating block write stores the bits of
# step-by-step rotating appends, and the block call with unrotated queries gives the bits
# of rotating first; every step of the block against the oracle.  Column counts on both
# kernels (up to 16: single-step kernel; more: LDS-staged kernel), per-sequence steps.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("C", [1, 4, 5, 9, 42])
@pytest.mark.parametrize("window,ragged", [(0, False), (37, False), (0, True), (60, True)])
def test_rope_block_write_and_block_attention(C, window, ragged):
    B, Hq, Hkv, D, Z, T_len = 4, 6, 2, 128, 32, 200
    dtype = T.TEMPO_BF16
    q, K, V = host_inputs(59 + C, B, T_len, Hq, Hkv, D, dtype)
    cos_t, sin_t = tables(T_len, D)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, fill="nan")
    one = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, fill="nan")
    st.set_rope(cos_t, sin_t)
    one.set_rope(cos_t, sin_t)
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    qd = dev(np.ascontiguousarray(np.transpose(q, (1, 0, 2, 3))), dtype)   # [B][T][Hq][D]
    first = [101, 64, 33, 150 - C] if ragged else [120] * B       # first step of each sequence's block
    hist = max(first)
    # history: steps 0 .. first[b]-1 of every sequence, one rotating append per step
    ar = torch.arange(B, device=DEV)
    for t in range(hist):
        tps = torch.tensor([min(t, f - 1) for f in first], dtype=torch.int32, device=DEV)
        for store in (st, one):
            store.rope_append(Kd[ar, tps.long()].contiguous(), Vd[ar, tps.long()].contiguous(), t, tps)
    fps = torch.tensor(first, dtype=torch.int32, device=DEV)
    kblk = torch.stack([Kd[b, first[b]:first[b] + C] for b in range(B)]).contiguous()
    vblk = torch.stack([Vd[b, first[b]:first[b] + C] for b in range(B)]).contiguous()
    qblk = torch.stack([qd[b, first[b]:first[b] + C] for b in range(B)]).contiguous()
    tp = fps if ragged else None
    st.rope_append_block(kblk, vblk, hist, C, tp)
    qrot = torch.empty_like(qblk)
    for c in range(C):                                            # the same, one step at a time
        tc = (fps + c).to(torch.int32)
        one.rope_append(kblk[:, c].contiguous(), vblk[:, c].contiguous(), hist + c, tc)
        qrot[:, c] = one.rope_rotate(qblk[:, c].contiguous(), torch.empty_like(qblk[:, c]), hist + c, tc)
    torch.cuda.synchronize()
    assert torch.equal(st.k_pool.view(torch.uint8), one.k_pool.view(torch.uint8))
    assert torch.equal(st.v_pool.view(torch.uint8), one.v_pool.view(torch.uint8))
    o_fused = torch.empty_like(qblk)
    o_plain = torch.empty_like(qblk)
    st.attend_block(qblk, o_fused, hist, C, window, tp, rope=True)
    one.attend_block(qrot, o_plain, hist, C, window, tp)
    assert torch.equal(o_fused.view(torch.uint8), o_plain.view(torch.uint8))
    qr64, Kr64 = oracle_rotated_kv(q, K, dtype)
    V64 = V.astype(np.float64)
    got = np64(o_fused)
    for c in range(C):
        tt = np.array([f + c for f in first], dtype=np.int32)
        qref = np.stack([qr64[first[b] + c, b] for b in range(B)])
        ref = oracle.attend(qref, Kr64, V64, tt, window, 1.0 / np.sqrt(D))
        assert_close(got[:, c], ref, dtype, f"rope block C={C} step {c} window={window} ragged={ragged}")
    with pytest.raises(T.TempoError):                             # tables too short for the block's last step
        short = T.make_rope(cos_t[:hist + C - 1].contiguous(), sin_t[:hist + C - 1].contiguous(), D)
        T.tempo_rope_kv_append_block(st.kv, short, kblk, vblk, B, hist, tp, C)


# ----------------------------------------------------------------------------
# A serving loop end to end: prompts of different lengths in one call (rotary producer
# fused in), then decode steps in which every sequence stands at its own position
# (fused rotate + append + attend), some through a block of steps; every decode output
# against the oracle on the rotated history.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("window", [0, 45])
def test_prompt_then_ragged_decode_end_to_end(window):
    B, Hq, Hkv, D, Z, T_len = 5, 6, 2, 128, 32, 260
    dtype = T.TEMPO_BF16
    q, K, V = host_inputs(58, B, T_len, Hq, Hkv, D, dtype)       # q [T][B][Hq][D]
    cos_t, sin_t = tables(T_len, D)
    table, nb = random_table(58, B, (T_len - 1) // Z + 1)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    st.set_rope(cos_t, sin_t)
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    qd = dev(np.ascontiguousarray(np.transpose(q, (1, 0, 2, 3))), dtype)   # [B][T][Hq][D]
    prompt = [130, 1, 64, 97, 33]                                 # prompt lengths
    P = max(prompt)
    cps = torch.tensor(prompt, dtype=torch.int32, device=DEV)
    op = torch.zeros((B, P, Hq, D), dtype=torch.bfloat16, device=DEV)
    st.prefill_attend(qd[:, :P].contiguous(), Kd[:, :P].contiguous(), Vd[:, :P].contiguous(), op, 0, P, window,
                      count_per_seq=cps, rope=True)
    qr64, Kr64 = oracle_rotated_kv(q, K, dtype)
    V64 = V.astype(np.float64)
    scale = 1.0 / np.sqrt(D)
    got = np64(op)
    for b in range(B):                                            # the last prompt step of every sequence
        t = prompt[b] - 1
        ref = oracle.attend(qr64[t][b:b + 1], Kr64[b:b + 1], V64[b:b + 1], t, window, scale)
        assert_close(got[b:b + 1, t], ref, dtype, f"prompt seq {b} step {t}")
    # decode: 60 single steps, each sequence at its own position
    pos = list(prompt)
    ar = torch.arange(B, device=DEV)
    for step in range(60):
        tps = torch.tensor(pos, dtype=torch.int32, device=DEV)
        qb = torch.stack([qd[b, pos[b]] for b in range(B)]).contiguous()
        out = st.rope_step(qb, Kd[ar, tps.long()].contiguous(), Vd[ar, tps.long()].contiguous(), st.new_out(),
                           max(pos), window, tps)
        if step % 7 == 0 or step == 59:
            qref = np.stack([qr64[pos[b], b] for b in range(B)])
            ref = oracle.attend(qref, Kr64, V64, np.array(pos, dtype=np.int32), window, scale)
            assert_close(out, ref, dtype, f"decode step {step} positions {pos}")
        pos = [x + 1 for x in pos]
    # then a block of 9 steps per sequence: one rotating block write, one call with unrotated queries
    C = 9
    tps = torch.tensor(pos, dtype=torch.int32, device=DEV)
    kblk = torch.stack([Kd[b, pos[b]:pos[b] + C] for b in range(B)]).contiguous()
    vblk = torch.stack([Vd[b, pos[b]:pos[b] + C] for b in range(B)]).contiguous()
    qblk = torch.stack([qd[b, pos[b]:pos[b] + C] for b in range(B)]).contiguous()
    st.rope_append_block(kblk, vblk, max(pos), C, tps)
    oblk = torch.empty_like(qblk)
    st.attend_block(qblk, oblk, max(pos), C, window, tps, rope=True)
    gotb = np64(oblk)
    for c in range(C):
        tt = np.array([x + c for x in pos], dtype=np.int32)
        qref = np.stack([qr64[pos[b] + c, b] for b in range(B)])
        ref = oracle.attend(qref, Kr64, V64, tt, window, scale)
        assert_close(gotb[:, c], ref, dtype, f"block step {c}")


# ----------------------------------------------------------------------------
# A prompt with the rotary producer fused in: keys rotated on their way into the
# store (the bits tempo_rope_kv_append stores), queries when the prompt kernel
# loads them; every step against the oracle, per-sequence lengths included.
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("D,G,window", [(128, 3, 0), (64, 2, 60), (128, 1, 0)])
def test_rope_prompt_every_step(D, G, window):
    B, Hkv, Z, steps, first = 6, 2, 32, 150, 21
    Hq = Hkv * G
    dtype = T.TEMPO_BF16
    q, K, V = host_inputs(56, B, steps, Hq, Hkv, D, dtype)
    cos_t, sin_t = tables(steps, D)
    st = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, fill="nan")
    one = BlockStore(B, Hq, Hkv, D, Z, steps - 1, dtype, fill="nan")
    st.set_rope(cos_t, sin_t)
    one.set_rope(cos_t, sin_t)
    Kd, Vd = dev(K, dtype), dev(V, dtype)
    qd = dev(np.ascontiguousarray(np.transpose(q, (1, 0, 2, 3))), dtype)
    counts = [steps - first, 1, 40, 0, 100, 129]
    cps = torch.tensor(counts, dtype=torch.int32, device=DEV)
    o1 = torch.empty((B, first, Hq, D), dtype=torch.bfloat16, device=DEV)
    st.prefill_attend(qd[:, :first].contiguous(), Kd[:, :first].contiguous(), Vd[:, :first].contiguous(), o1, 0,
                      first, window, rope=True)
    o2 = torch.full((B, steps - first, Hq, D), 7.0, dtype=torch.bfloat16, device=DEV)
    st.prefill_attend(qd[:, first:].contiguous(), Kd[:, first:].contiguous(), Vd[:, first:].contiguous(), o2, first,
                      steps - first, window, count_per_seq=cps, rope=True)
    last = [first + n for n in counts]                     # steps each sequence holds
    for t in range(steps):                                  # the same keys through single rotate-and-append calls
        tps = torch.tensor([min(t, l - 1) for l in last], dtype=torch.int32, device=DEV)
        ar = torch.arange(B, device=DEV)
        one.rope_append(Kd[ar, tps.long()].contiguous(), Vd[ar, tps.long()].contiguous(), t, tps)
    assert torch.equal(st.k_pool.view(torch.int16), one.k_pool.view(torch.int16))
    assert torch.equal(st.v_pool.view(torch.int16), one.v_pool.view(torch.int16))
    qr64, Kr64 = oracle_rotated_kv(q, K, dtype)
    V64 = V.astype(np.float64)
    got = np.concatenate([np64(o1), np64(o2)], axis=1)
    for b in range(B):
        assert (got[b, last[b]:] == 7.0).all()
        for t in range(last[b]):
            ref = oracle.attend(qr64[t][b:b + 1], Kr64[b:b + 1], V64[b:b + 1], t, window, 1.0 / np.sqrt(D))
            assert_close(got[b:b + 1, t], ref, dtype, f"rope prompt b={b} step {t}")


def test_llama_shape_fused_rope_step_full_size():
    B, Hq, Hkv, D, Z, T_len = 16, 24, 8, 128, 256, 4096
    dtype = T.TEMPO_BF16
    K, V = flat_kv(55, B, T_len, Hkv, D)          # treated as already rotated history
    table, nb = random_table(55, B, T_len // Z, extra=0)
    st = BlockStore(B, Hq, Hkv, D, Z, T_len - 1, dtype, num_blocks=nb, block_table=table, fill="nan")
    st.set_rope(*tables(T_len, D))
    st.prefill(K, V, T_len - 2)
    t = T_len - 1
    q = synth.device_normal((B, Hq, D), 5500, torch.bfloat16, DEV)
    k_raw = synth.device_normal((B, Hkv, D), 5501, torch.bfloat16, DEV)
    out = st.rope_step(q, k_raw, V[:, t].contiguous(), st.new_out(), t)
    K64, V64 = np64(K), np64(V)
    K64[:, t] = synth.round_to_bf16(oracle.rope(np64(k_raw), t, THETA).astype(np.float32)).astype(np.float64)
    qr = synth.round_to_bf16(oracle.rope(np64(q), t, THETA).astype(np.float32)).astype(np.float64)
    ref = oracle.attend(qr, K64, V64, t, 0, 1.0 / np.sqrt(D))
    assert_close(out, ref, dtype, "llama fused rope step t=4095")
    kg, _ = st.gather(t, 1)
    assert_rotated(kg[:, 0], oracle.rope(np64(k_raw), t, THETA), dtype, "stored rotated key t=4095")
