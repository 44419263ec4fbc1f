"""The entry point that allocates nothing (split partials in the library's static device
array) against the entry point it is a variant of, through the C ABI.

Bar: identical bits (same kernels, same plan), and the oracle's values within the bf16
tolerance |gpu - oracle| <= 2e-2 elementwise and max|gpu - oracle| <= 1e-2 * max|oracle|.
Two calls in a row on the same GPU, the second with a smaller input, so that whatever the
first call left in the array must not matter.
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


def np64(x):
    return x.detach().float().cpu().numpy().astype(np.float64)


def one_call(seed, B, Hq, Hkv, D, Z, t, ragged=None):
    """Step t through both entry points on two stores with the same contents; returns the outputs."""
    T_len = t + 1
    K = synth.device_normal((B, T_len, Hkv, D), seed * 10 + 1, torch.bfloat16, DEV)
    V = synth.device_normal((B, T_len, Hkv, D), seed * 10 + 2, torch.bfloat16, DEV)
    q = synth.device_normal((B, Hq, D), seed * 10 + 3, torch.bfloat16, DEV)
    stores = []
    for _ in range(2):
        st = BlockStore(B, Hq, Hkv, D, Z, t, T.TEMPO_BF16, device=DEV, fill="nan")
        st.prefill(K, V, t - 1)
        stores.append(st)
    tps = None
    if ragged is not None:
        tps = torch.tensor(ragged, dtype=torch.int32, device=DEV)
        ar = torch.arange(B, device=DEV)
        k_t, v_t = K[ar, tps.long()].contiguous(), V[ar, tps.long()].contiguous()
    else:
        k_t, v_t = K[:, t].contiguous(), V[:, t].contiguous()
    plan = T.tempo_attn_plan(stores[0].kv, B, Hq, t, 0, ragged is not None)
    assert plan.num_splits > 1, "the call must use split partials, or the static array is not exercised"
    want = stores[0].step_causal(q, k_t, v_t, stores[0].new_out(), t, t_per_seq=tps)
    got = stores[1].step_causal_noalloc(q, k_t, v_t, stores[1].new_out(), t, t_per_seq=tps)
    torch.cuda.synchronize()
    assert torch.equal(got, want), "static-array step differs from the workspace step"
    assert torch.equal(stores[0].k_pool.view(torch.int16), stores[1].k_pool.view(torch.int16))
    assert torch.equal(stores[0].v_pool.view(torch.int16), stores[1].v_pool.view(torch.int16))
    steps = np.array(ragged, dtype=np.int32) if ragged is not None else t
    ref = oracle.attend(np64(q), np64(K), np64(V), steps, 0, 1.0 / np.sqrt(D))
    err = np.abs(np64(got) - ref).max()
    assert err <= 2e-2 and err <= 1e-2 * np.abs(ref).max(), f"max-abs {err:.3e}"
    return got


def test_no_alloc_step_twice_second_call_smaller():
    # first call: the headline shape (2 splits of 2048 keys, 0.4 MiB of partials)
    one_call(31, 16, 24, 8, 128, 256, 4095)
    # second call, smaller in every dimension, ragged steps, many short splits
    one_call(32, 3, 8, 2, 64, 64, 700, ragged=[700, 5, 333])
    # and a third, uniform again, to see that the order of sizes does not matter
    one_call(33, 2, 6, 2, 128, 32, 1500)


def test_no_alloc_refuses_what_does_not_fit():
    # batch 64 x 64 query heads, ragged steps up to 8191: 8 splits x 4096 rows x 520 B = 17 MB > 8 MiB
    B, Hq, Hkv, D, Z, t = 64, 64, 8, 128, 256, 8191
    st = BlockStore(B, Hq, Hkv, D, Z, t, T.TEMPO_BF16, device=DEV)
    q = torch.zeros((B, Hq, D), dtype=torch.bfloat16, device=DEV)
    kv_new = torch.zeros((B, Hkv, D), dtype=torch.bfloat16, device=DEV)
    tps = torch.full((B,), 100, dtype=torch.int32, device=DEV)
    out = st.new_out().fill_(7.0)
    with pytest.raises(T.TempoError) as e:
        st.step_causal_noalloc(q, kv_new, kv_new, out, t, t_per_seq=tps)
    assert e.value.status == T.TEMPO_ERR_WORKSPACE
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())                              # nothing was launched
    st.step_causal(q, kv_new, kv_new, out, t, t_per_seq=tps)       # the workspace entry point takes it
    torch.cuda.synchronize()
