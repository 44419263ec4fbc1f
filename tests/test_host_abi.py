"""Host-side tests of libtempo: the library loads and exports every symbol the
header declares, the integer functions agree bit for bit with the oracle's
counting loops, the block-store layout is the one the header describes, the
split planner's promises hold, and bad arguments are refused before any launch.
No test here computes anything on a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import tempo_oracle as oracle
from paper_2501_05408_amd import tempo as T

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    text = open(os.path.join(ROOT, "include", "tempo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tempo_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = T.load()
    names = header_functions()
    assert len(names) >= 14
    for name in names:
        assert hasattr(lib, name), f"libtempo.so lacks {name}"
    assert sorted(T.SIGNATURES) == names, "binding and header disagree on the entry points"
    for name in names:
        assert callable(getattr(T, name)), f"binding lacks {name}"


def test_visible_range_and_slot_match_oracle_bit_exact():
    for Z in (1, 2, 3, 4, 8, 64, 256):
        for t in list(range(0, 70)) + [255, 256, 257, 511, 4095, 16383]:
            for w in (0, 1, 2, 3, 4, 9, 64, 512, 100000):
                got = T.tempo_visible_range(t, w, Z)
                ref = oracle.visible_range(t, w, Z)
                for k in got:
                    assert got[k] == ref[k], (t, w, Z, k)
            assert T.tempo_append_slot(t, Z) == oracle.append_slot(t, Z)
    with pytest.raises(T.TempoError):
        T.tempo_visible_range(-1, 0, 4)
    with pytest.raises(T.TempoError):
        T.tempo_append_slot(3, 0)


def test_release_and_ring_size_match_oracle_bit_exact():
    for Z in (1, 2, 3, 8, 64, 256):
        for w in (0, 1, 2, 3, 9, 64, 65, 512, 513, 514):
            for t in list(range(0, 40)) + [255, 256, 511, 512, 513, 4095]:
                assert T.tempo_kv_release(t, w, Z) == oracle.release(t, w, Z), (t, w, Z)
            for queries in (1, 2, 5, 42):
                if w >= 1:
                    # The oracle gives the fewest resident tiles of a circular store (Section 6).  The
                    # library's ring indexes its table with a bit mask, so ITS answer is that count
                    # rounded up to a power of two: a constraint of the library, not of the method.
                    need = oracle.ring_blocks(w, Z, queries)
                    got = T.tempo_ring_blocks(w, Z, queries)
                    assert got >= need and got & (got - 1) == 0 and (got == 1 or got // 2 < need), (w, Z, queries)
    assert T.tempo_kv_release(2 ** 31 - 2, 1, 1) == (2 ** 31 - 1, 2 ** 31 - 1)   # no overflow at the top
    for bad in ((-1, 3, 4), (3, -1, 4), (3, 3, 0), (2 ** 31 - 1, 1, 1)):
        with pytest.raises(T.TempoError):
            T.tempo_kv_release(*bad)
    for bad in ((0, 8, 1), (8, 0, 1), (8, 8, 0), (2 ** 31 - 1, 1, 2 ** 31 - 1)):
        with pytest.raises(T.TempoError):
            T.tempo_ring_blocks(*bad)


def kv_desc(dtype, D=128, Z=64, Hkv=2, num_blocks=3, max_blocks=4, pools=(1 << 20, 1 << 21, 1 << 22), ring=0):
    return T.tempo_kv(pools[0], pools[1], pools[2], num_blocks, max_blocks, Z, Hkv, D, dtype, ring)


@pytest.mark.parametrize("D", [64, 128])
def test_layout_is_a_bijection_and_matches_the_documented_order(D):
    Z, Hkv, NB = 64, 2, 3
    kv = kv_desc(T.TEMPO_BF16, D=D, Z=Z, Hkv=Hkv, num_blocks=NB)
    n = NB * Hkv * Z * D
    assert T.tempo_kv_pool_bytes(kv) == n * 2
    for which in (0, 1):
        seen = np.zeros(n, dtype=bool)
        for blk in range(NB):
            for head in range(Hkv):
                for slot in range(Z):
                    for d in range(D):
                        off = T.tempo_kv_element_offset(kv, which, blk, head, slot, d)
                        base = (blk * Hkv + head) * Z * D
                        grp, u = divmod(slot, 32)
                        if which == 0:
                            # K: lane (row + 16c) of unit (tile, s) holds dims 32s+8c..+7 of slot row
                            tile, row = divmod(u, 16)
                            s, rem = divmod(d, 32)
                            c, e = divmod(rem, 8)
                            unit, lane = tile * (D // 32) + s, c * 16 + row
                        else:
                            # V: lane (n + 16c) of unit dt holds dim 16dt+n of slots {4c..4c+3, 16+4c..}
                            half, uu = divmod(u, 16)
                            c, e = uu // 4, uu % 4 + 4 * half
                            unit, nn = divmod(d, 16)
                            lane = c * 16 + nn
                        assert off == base + grp * 32 * D + (unit * 64 + lane) * 8 + e
                        seen[off] = True
        assert seen.all()
    kvf = kv_desc(T.TEMPO_F32, D=D, Z=Z, Hkv=Hkv, num_blocks=NB)
    assert T.tempo_kv_pool_bytes(kvf) == n * 4
    assert T.tempo_kv_element_offset(kvf, 0, 2, 1, 5, 7) == ((2 * Hkv + 1) * Z + 5) * D + 7
    assert T.tempo_kv_element_offset(kvf, 1, 2, 1, 5, 7) == ((2 * Hkv + 1) * Z + 5) * D + 7
    assert T.tempo_kv_element_offset(kv, 0, NB, 0, 0, 0) == -1
    assert T.tempo_kv_element_offset(kv, 0, 0, 0, Z, 0) == -1
    assert T.tempo_kv_element_offset(kv, 2, 0, 0, 0, 0) == -1


def test_plan_covers_every_step_and_workspace_bound_holds():
    for dtype, hq_hkv in ((T.TEMPO_BF16, (24, 8)), (T.TEMPO_F32, (8, 2)), (T.TEMPO_BF16, (4, 4))):
        Hq, Hkv = hq_hkv
        for batch in (1, 3, 16, 64):
            for max_t in (0, 31, 32, 511, 4095, 70000):
                kv = kv_desc(dtype, Hkv=Hkv, Z=64, max_blocks=max_t // 64 + 1)
                bound = T.tempo_attn_workspace_bytes(kv, batch, Hq, max_t)
                assert bound > 0 and bound % 256 == 0
                ts = sorted(set(list(range(0, min(max_t, 700) + 1, 7)) + [max_t, max_t // 2, max_t // 3]))
                for t in ts:
                    for w in (0, 1, 5, 512, 513):
                      for ragged in (False, True):
                        plan = T.tempo_attn_plan(kv, batch, Hq, t, w, ragged)
                        tps = plan.tokens_per_split
                        assert not ragged or tps <= 1024
                        assert tps >= 32 and tps & (tps - 1) == 0
                        assert plan.waves in (1, 2, 4, 8) and plan.waves * 32 <= max(tps, 32)
                        lo = 0 if w == 0 else max(0, t - w + 1)
                        assert plan.num_splits >= t // tps - lo // tps + 1
                        # any earlier step of a ragged batch is covered too
                        for t2 in (t, t // 2, max(0, t - 17)):
                            lo2 = 0 if w == 0 else max(0, t2 - w + 1)
                            assert plan.num_splits >= t2 // tps - lo2 // tps + 1
                        assert plan.num_splits <= 1024
                        assert T.tempo_attn_plan_workspace_bytes(kv, batch, Hq, plan) <= bound


def test_block_plan_fits_its_workspace_bound_and_lds():
    D = 128
    for dtype, Hq, Hkv in ((T.TEMPO_BF16, 24, 8), (T.TEMPO_BF16, 16, 1), (T.TEMPO_BF16, 2, 2), (T.TEMPO_F32, 8, 2)):
        G = Hq // Hkv
        for queries in sorted({1, min(2, 128 // G), 16 // G, 32 // G, 128 // G}):
            for batch in (1, 16, 64):
                for max_t in (0, 40, 4095, 70000):
                    kv = kv_desc(dtype, D=D, Hkv=Hkv, Z=64, max_blocks=(max_t + queries) // 64 + 1)
                    bound = T.tempo_attn_block_workspace_bytes(kv, batch, Hq, queries, max_t)
                    assert bound > 0 and bound % 256 == 0
                    for t in sorted({0, max_t // 3, max(0, max_t - 1), max_t}):
                        for w in (0, 1, 33, 512):
                            for ragged in (False, True):
                                plan = T.tempo_attn_block_plan(kv, batch, Hq, queries, t, w, ragged)
                                tps = plan.tokens_per_split
                                lo = 0 if w == 0 else max(0, t - w + 1)
                                assert plan.num_splits >= (t + queries - 1) // tps - lo // tps + 1
                                rows = batch * queries * Hq
                                need = -(-rows * plan.num_splits * 8 // 256) * 256 + \
                                    -(-rows * plan.num_splits * D * 4 // 256) * 256
                                assert need <= bound
                                if dtype == T.TEMPO_BF16 and queries * G <= 16:   # wave-merge area + staged rows within 64 KiB
                                    assert plan.waves * (32 + queries * G * D) * 4 + 4 * D <= 65536
                                elif dtype == T.TEMPO_BF16:                       # the LDS-staged kernel's fixed shape
                                    assert plan.waves == 8
    with pytest.raises(T.TempoError):
        T.tempo_attn_block_plan(kv_desc(T.TEMPO_BF16, Hkv=2), 1, 8, 33, 10)     # 33 x 4 columns > 128
    assert T.tempo_attn_block_workspace_bytes(kv_desc(T.TEMPO_BF16, Hkv=2), 1, 8, 33, 10) == 0
    assert T.tempo_attn_block_workspace_bytes(kv_desc(T.TEMPO_BF16, Hkv=2), 1, 8, 0, 10) == 0


def test_bad_arguments_are_refused_before_any_launch():
    lib = T.load()
    good = kv_desc(T.TEMPO_BF16)
    fake = 1 << 20   # a non-NULL address that is never dereferenced: validation fails first

    def append(kv, k=fake, v=fake, batch=2, t=5):
        return lib.tempo_kv_append(ctypes.byref(kv), k, v, batch, t, None, None)

    assert append(kv_desc(T.TEMPO_BF16, pools=(None, 1, 1))) == T.TEMPO_ERR_NULL
    assert append(good, k=None) == T.TEMPO_ERR_NULL
    assert append(kv_desc(7)) == T.TEMPO_ERR_DTYPE
    assert append(kv_desc(T.TEMPO_BF16, D=96)) == T.TEMPO_ERR_SHAPE
    assert append(kv_desc(T.TEMPO_BF16, Z=48)) == T.TEMPO_ERR_SHAPE
    assert append(kv_desc(T.TEMPO_BF16, Z=16)) == T.TEMPO_ERR_SHAPE
    assert append(good, batch=0) == T.TEMPO_ERR_SHAPE
    assert append(good, t=-1) == T.TEMPO_ERR_RANGE
    assert append(good, t=4 * 64) == T.TEMPO_ERR_RANGE          # needs a fifth block of four

    def causal(kv, Hq=6, t=5, ws=fake << 4, ws_bytes=1 << 30, q=fake, out=fake):
        return lib.tempo_attn_decode_causal(ctypes.byref(kv), q, out, 2, Hq, t, None, 0.1, ws, ws_bytes, None)

    assert causal(good, Hq=5) == T.TEMPO_ERR_SHAPE              # not a multiple of Hkv
    assert causal(good, Hq=2 * 129) == T.TEMPO_ERR_SHAPE        # group larger than 128
    assert causal(good, q=None) == T.TEMPO_ERR_NULL
    for bad_scale in (0.0, -0.1, float("inf"), float("nan")):   # Eq. 1's constant s is finite and positive
        assert lib.tempo_attn_decode_causal(ctypes.byref(good), fake, fake, 2, 6, 5, None, bad_scale, fake << 4,
                                            1 << 30, None) == T.TEMPO_ERR_RANGE
    assert causal(good, t=1000) == T.TEMPO_ERR_RANGE
    assert causal(good, ws=None) == T.TEMPO_ERR_WORKSPACE
    assert causal(good, ws=(fake << 4) + 8) == T.TEMPO_ERR_WORKSPACE     # misaligned
    assert causal(good, ws_bytes=16) == T.TEMPO_ERR_WORKSPACE

    def window(kv, w):
        return lib.tempo_attn_decode_window(ctypes.byref(kv), fake, fake, 2, 6, 5, None, w, 0.1, fake << 4,
                                            1 << 30, None)

    assert window(good, 0) == T.TEMPO_ERR_RANGE
    assert window(good, -3) == T.TEMPO_ERR_RANGE

    # ring (window) stores: size must be a power of two within the table row; a step is
    # answered only while every tile of its visible range is still resident
    assert append(kv_desc(T.TEMPO_BF16, ring=3)) == T.TEMPO_ERR_SHAPE
    assert append(kv_desc(T.TEMPO_BF16, ring=8)) == T.TEMPO_ERR_SHAPE          # row has 4 columns

    def ring_window(t, w, ring=4):
        kv = kv_desc(T.TEMPO_BF16, ring=ring)
        return lib.tempo_attn_decode_window(ctypes.byref(kv), fake, fake, 2, 6, t, None, w, 0.1, None, 0, None)

    def ring_causal(t, ring=4):
        kv = kv_desc(T.TEMPO_BF16, ring=ring)
        return lib.tempo_attn_decode_causal(ctypes.byref(kv), fake, fake, 2, 6, t, None, 0.1, None, 0, None)

    # Z = 64, ring of 4: a window of up to 3*64+1 keys always fits, 3*64+2 may touch 5 tiles
    assert ring_window(100000, 193) == T.TEMPO_ERR_WORKSPACE                  # passes the ring check
    assert ring_window(100000, 194) == T.TEMPO_ERR_RANGE
    assert ring_window(100, 5000) == T.TEMPO_ERR_WORKSPACE                    # window longer than history: 2 tiles
    assert ring_causal(255) == T.TEMPO_ERR_WORKSPACE
    assert ring_causal(256) == T.TEMPO_ERR_RANGE

    # the padded + masked baseline lives in the single-step kernel: bf16, groups of at most 16 heads
    def padded(kv, Hq=6, t=5, t_pad=100):
        return lib.tempo_attn_decode_padded_causal(ctypes.byref(kv), fake, fake, 2, Hq, t, None, t_pad, 0.1, None, 0,
                                                   None)

    assert padded(good) == T.TEMPO_ERR_WORKSPACE                 # everything else is fine
    assert padded(good, Hq=2 * 16) == T.TEMPO_ERR_WORKSPACE
    assert padded(good, Hq=2 * 17) == T.TEMPO_ERR_SHAPE          # served by a kernel with no padded form
    assert padded(good, t=101) == T.TEMPO_ERR_RANGE
    assert padded(kv_desc(T.TEMPO_F32)) == T.TEMPO_ERR_DTYPE

    # ragged work list: bf16, groups of at most 16 heads, batch * splits within one grid dimension
    wl_kv = kv_desc(T.TEMPO_BF16, Z=256, Hkv=8, num_blocks=64 * 32, max_blocks=32)
    assert T.tempo_attn_worklist_bytes(wl_kv, 64, 24, 8191) >= 4 * (1 + 64 * 8)
    assert T.tempo_attn_worklist_bytes(kv_desc(T.TEMPO_F32, Z=256, Hkv=8, max_blocks=32), 64, 24, 8191) == 0
    assert T.tempo_attn_worklist_bytes(wl_kv, 64, 8 * 17, 8191) == 0
    assert lib.tempo_attn_worklist_build(ctypes.byref(wl_kv), 64, 24, 8191, fake, 0, fake, 16, None) == T.TEMPO_ERR_WORKSPACE
    assert lib.tempo_attn_worklist_build(ctypes.byref(wl_kv), 64, 24, 8191, None, 0, fake, 1 << 20, None) == T.TEMPO_ERR_NULL
    assert lib.tempo_attn_worklist_build(ctypes.byref(wl_kv), 64, 24, 8191, fake, 0, fake + 2, 1 << 20, None) == T.TEMPO_ERR_WORKSPACE
    assert lib.tempo_decode_step_ragged(ctypes.byref(wl_kv), fake, fake, fake, fake, 64, 24, 8191, fake, 0, 0.1, None,
                                        fake << 4, 1 << 30, None) == T.TEMPO_ERR_NULL
    assert lib.tempo_decode_step_ragged(ctypes.byref(wl_kv), fake, fake, None, fake, 64, 24, 8191, fake, 0, 0.1, fake,
                                        fake << 4, 1 << 30, None) == T.TEMPO_ERR_NULL
    assert lib.tempo_decode_step_ragged(ctypes.byref(wl_kv), fake, fake, fake, fake, 64, 24, 8191, fake, 0, 0.1, fake,
                                        fake << 4, 16, None) == T.TEMPO_ERR_WORKSPACE

    # the anti-causal window reduction: a short window or the whole future, a finite discount, no aliasing
    def dsum(r=fake, g=fake + 4096, batch=2, T_len=5000, n=5, gamma=0.9):
        return lib.tempo_discounted_sum(r, g, batch, T_len, n, gamma, None)

    assert dsum(r=None) == T.TEMPO_ERR_NULL and dsum(g=None) == T.TEMPO_ERR_NULL
    assert dsum(g=fake) == T.TEMPO_ERR_SHAPE
    assert dsum(batch=0) == T.TEMPO_ERR_SHAPE and dsum(T_len=0) == T.TEMPO_ERR_SHAPE
    assert dsum(n=-1) == T.TEMPO_ERR_RANGE and dsum(n=1025) == T.TEMPO_ERR_RANGE and dsum(n=4999) == T.TEMPO_ERR_RANGE
    assert dsum(gamma=float("inf")) == T.TEMPO_ERR_RANGE and dsum(gamma=float("nan")) == T.TEMPO_ERR_RANGE

    def block(kv, queries, t=5, Hq=6, w=None):
        if w is None:
            return lib.tempo_attn_block_causal(ctypes.byref(kv), fake, fake, 2, Hq, queries, t, None, 0.1, None, 0, None)
        return lib.tempo_attn_block_window(ctypes.byref(kv), fake, fake, 2, Hq, queries, t, None, w, 0.1, None, 0, None)

    assert block(good, 0) == T.TEMPO_ERR_SHAPE
    assert block(good, 43) == T.TEMPO_ERR_SHAPE                  # 43 steps x 3 heads > 128 columns
    assert block(good, 42) == T.TEMPO_ERR_WORKSPACE              # 126 columns: the LDS-staged kernel
    assert block(good, 5) == T.TEMPO_ERR_WORKSPACE               # everything else is fine
    assert block(good, 5, t=4 * 64 - 5) == T.TEMPO_ERR_WORKSPACE  # last step is the store's last slot
    assert block(good, 5, t=4 * 64 - 4) == T.TEMPO_ERR_RANGE     # last step needs a fifth block
    assert block(good, 2, w=0) == T.TEMPO_ERR_RANGE
    ringed = kv_desc(T.TEMPO_BF16, ring=4)
    assert block(ringed, 1, t=100000, w=193) == T.TEMPO_ERR_WORKSPACE
    assert block(ringed, 2, t=100000, w=193) == T.TEMPO_ERR_RANGE   # the union of two ranges may touch 5 tiles

    def append_block(kv, count, t=0):
        return lib.tempo_kv_append_block(ctypes.byref(kv), fake, fake, 2, t, None, count, None)

    assert append_block(good, 0) == T.TEMPO_ERR_SHAPE
    assert append_block(good, 4 * 64 + 1) == T.TEMPO_ERR_RANGE
    assert append_block(good, 10, t=4 * 64 - 9) == T.TEMPO_ERR_RANGE
    assert append_block(ringed, 4 * 64 + 1, t=7) == T.TEMPO_ERR_RANGE   # would wrap onto its own rows
    assert lib.tempo_kv_append_block(ctypes.byref(good), None, fake, 2, 0, None, 3, None) == T.TEMPO_ERR_NULL

    # rotary tables: both present, 16-byte aligned, made for the store's head_dim, long enough
    def rope_desc(cos=fake, sin=fake, positions=100, head_dim=128):
        return T.tempo_rope(cos, sin, positions, head_dim)

    def rope_append(rope, t=5):
        return lib.tempo_rope_kv_append(ctypes.byref(good), ctypes.byref(rope), fake, fake, 2, t, None, None)

    assert rope_append(rope_desc(cos=None)) == T.TEMPO_ERR_NULL
    assert rope_append(rope_desc(sin=None)) == T.TEMPO_ERR_NULL
    assert rope_append(rope_desc(head_dim=64)) == T.TEMPO_ERR_SHAPE
    assert rope_append(rope_desc(cos=fake + 4)) == T.TEMPO_ERR_SHAPE
    assert rope_append(rope_desc(positions=5)) == T.TEMPO_ERR_RANGE        # step 5 needs 6 rows
    assert lib.tempo_rope_kv_append(ctypes.byref(good), None, fake, fake, 2, 5, None, None) == T.TEMPO_ERR_NULL

    def rope_step(rope, t=5, w=None):
        r = ctypes.byref(rope) if rope is not None else None
        if w is None:
            return lib.tempo_rope_decode_step_causal(ctypes.byref(good), r, fake, fake, fake, fake, 2, 6, t, None,
                                                     0.1, None, 0, None)
        return lib.tempo_rope_decode_step_window(ctypes.byref(good), r, fake, fake, fake, fake, 2, 6, t, None, w,
                                                 0.1, None, 0, None)

    assert rope_step(None) == T.TEMPO_ERR_NULL
    assert rope_step(rope_desc(positions=5)) == T.TEMPO_ERR_RANGE
    assert rope_step(rope_desc(head_dim=64)) == T.TEMPO_ERR_SHAPE
    assert rope_step(rope_desc()) == T.TEMPO_ERR_WORKSPACE                  # everything else is fine
    assert rope_step(rope_desc(), w=0) == T.TEMPO_ERR_RANGE
    assert rope_step(rope_desc(), w=7) == T.TEMPO_ERR_WORKSPACE
    assert lib.tempo_rope_rotate(ctypes.byref(rope_desc()), fake, fake, 9, 2, 6, 5, None, None) == T.TEMPO_ERR_DTYPE
    assert lib.tempo_rope_rotate(ctypes.byref(rope_desc()), None, fake, T.TEMPO_F32, 2, 6, 5, None, None) == T.TEMPO_ERR_NULL
    assert lib.tempo_rope_rotate(ctypes.byref(rope_desc(head_dim=7)), fake, fake, T.TEMPO_F32, 2, 6, 5, None, None) == T.TEMPO_ERR_SHAPE
    assert lib.tempo_rope_rotate(ctypes.byref(rope_desc()), fake, fake, T.TEMPO_F32, 2, 6, 100, None, None) == T.TEMPO_ERR_RANGE

    # blocks with the rotary producer: the rotating block write and the block call with raw queries
    def rope_append_block(kv, rope, count=3, t=5):
        r = ctypes.byref(rope) if rope is not None else None
        return lib.tempo_rope_kv_append_block(ctypes.byref(kv), r, fake, fake, 2, t, None, count, None)

    assert rope_append_block(good, None) == T.TEMPO_ERR_NULL
    assert rope_append_block(kv_desc(T.TEMPO_F32), rope_desc()) == T.TEMPO_ERR_DTYPE
    assert rope_append_block(good, rope_desc(), count=0) == T.TEMPO_ERR_SHAPE
    assert rope_append_block(good, rope_desc(positions=7)) == T.TEMPO_ERR_RANGE      # steps 5..7 need 8 rows
    assert rope_append_block(good, rope_desc(), t=4 * 64 - 2) == T.TEMPO_ERR_RANGE  # runs past the last block

    def rope_block(rope, queries=3, t=5, w=None):
        r = ctypes.byref(rope) if rope is not None else None
        if w is None:
            return lib.tempo_rope_attn_block_causal(ctypes.byref(good), r, fake, fake, 2, 6, queries, t, None, 0.1,
                                                    None, 0, None)
        return lib.tempo_rope_attn_block_window(ctypes.byref(good), r, fake, fake, 2, 6, queries, t, None, w, 0.1,
                                                None, 0, None)

    assert rope_block(None) == T.TEMPO_ERR_NULL
    assert rope_block(rope_desc(positions=7)) == T.TEMPO_ERR_RANGE          # the last query stands at step 7
    assert rope_block(rope_desc(), queries=0) == T.TEMPO_ERR_SHAPE
    assert rope_block(rope_desc()) == T.TEMPO_ERR_WORKSPACE                  # everything else is fine
    assert rope_block(rope_desc(), w=0) == T.TEMPO_ERR_RANGE
    assert rope_block(rope_desc(), w=9) == T.TEMPO_ERR_WORKSPACE

    def prefill(kv, t=0, count=10, w=None, k=fake):
        if w is None:
            return lib.tempo_prefill_causal(ctypes.byref(kv), fake, k, fake, fake, 2, 6, t, count, None, 0.1, None, 0,
                                            None)
        return lib.tempo_prefill_window(ctypes.byref(kv), fake, k, fake, fake, 2, 6, t, count, None, w, 0.1, None, 0,
                                        None)

    assert prefill(good) == T.TEMPO_ERR_WORKSPACE                 # everything else is fine
    assert prefill(good, count=0) == T.TEMPO_ERR_SHAPE
    assert prefill(good, k=None) == T.TEMPO_ERR_NULL
    assert prefill(good, t=250, count=7) == T.TEMPO_ERR_RANGE     # last step 256 needs a fifth block
    assert prefill(good, t=250, count=6) == T.TEMPO_ERR_WORKSPACE
    assert prefill(good, w=0) == T.TEMPO_ERR_RANGE
    f32_store = kv_desc(T.TEMPO_F32)   # per-sequence prompt lengths: bf16 linear stores only
    assert lib.tempo_prefill_causal(ctypes.byref(f32_store), fake, fake, fake, fake, 2, 6, 0, 10, fake, 0.1,
                                    fake << 4, 1 << 30, None) == T.TEMPO_ERR_SHAPE
    assert T.tempo_prefill_workspace_bytes(good, 2, 6, 255) >= T.tempo_attn_block_workspace_bytes(good, 2, 6, 42, 255)

    bad_plan = T.tempo_plan(48, 1, 1)
    assert lib.tempo_attn_decode_partial(ctypes.byref(good), fake, None, None, 2, 6, 5, None, 0, 0.1,
                                         ctypes.byref(bad_plan), fake << 4, 1 << 30, None) == T.TEMPO_ERR_SHAPE
    assert lib.tempo_attn_decode_partial(ctypes.byref(good), fake, fake, None, 2, 6, 5, None, 0, 0.1,
                                         ctypes.byref(bad_plan), fake << 4, 1 << 30, None) == T.TEMPO_ERR_NULL
    short_plan = T.tempo_plan(32, 1, 1)                          # step 100 needs 4 splits of 32
    assert lib.tempo_attn_decode_partial(ctypes.byref(good), fake, None, None, 2, 6, 100, None, 0, 0.1,
                                         ctypes.byref(short_plan), fake << 4, 1 << 30, None) == T.TEMPO_ERR_RANGE
    assert lib.tempo_kv_gather(ctypes.byref(good), fake, fake, 2, 0, 4 * 64 + 1, None) == T.TEMPO_ERR_RANGE
    assert T.tempo_attn_workspace_bytes(kv_desc(T.TEMPO_BF16, D=96), 2, 6, 100) == 0
    assert "workspace" in T.tempo_strerror(T.TEMPO_ERR_WORKSPACE)


# ----------------------------------------------------------------------------
# The product path never reaches for the CPU oracle, and without the built library
# it fails loudly instead of falling back to anything.
# ----------------------------------------------------------------------------
def test_product_path_does_not_touch_the_oracle_and_has_no_fallback(monkeypatch):
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2501_05408_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "tempo_oracle" not in text, f
    bench = open(os.path.join(root, "bench.py")).read()
    assert bench.count("from oracle import") == 1
    assert bench.index("if not args.no_cpu:") < bench.index("from oracle import")   # inside the CPU-baseline leg
    # no library, and no way to build one: load() raises
    from paper_2501_05408_amd import build as B
    monkeypatch.setattr(T, "_lib", None)
    monkeypatch.setattr(B, "LIB", os.path.join(root, "no_such_dir", "libtempo.so"))

    def cannot_build(force=True):
        raise RuntimeError("no compiler here")

    monkeypatch.setattr(B, "build", cannot_build)
    with pytest.raises((RuntimeError, OSError)):
        T.load()


def test_planner_choice_is_near_the_best_measured_plan():
    """The split planner against a sweep of explicit plans measured on an MI355X and kept in
    profiles/ (batch 4, 16 and 64; the planner's time model was fitted at batch 16): the plan the
    library picks must have been measured within 5% of the fastest plan of its case."""
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles",
                        "attn_partial_bf16_plan_sweep.txt")
    cases = {}
    for line in open(path):
        parts = line.split()
        if len(parts) == 3 and parts[0].startswith("b") and "_t" in parts[0] and "x" in parts[1]:
            cases.setdefault(parts[0], {})[parts[1]] = float(parts[2])
    assert len(cases) >= 15
    for case, plans in cases.items():
        batch, t = int(case[1:case.index("_t")]), int(case[case.index("_t") + 2:])
        kv = kv_desc(T.TEMPO_BF16, D=128, Z=256, Hkv=8, num_blocks=batch * 32, max_blocks=32)
        plan = T.tempo_attn_plan(kv, batch, 24, t, 0)
        tps = plan.tokens_per_split
        if plan.num_splits == 1:                       # every single split that covers the range is the same plan
            tps = 1 << (t + 1 - 1).bit_length() if t > 0 else 32
            tps = max(tps, 32)
        key = f"{tps}x{plan.waves}"
        assert key in plans, f"{case}: the library's plan {key} was not part of the sweep"
        assert plans[key] <= 1.05 * min(plans.values()), (case, key, plans[key], min(plans.values()))
