"""Device-memory plumbing around the C ABI: allocate a block pool, a block table
and a workspace with torch, keep the tempo_kv descriptor next to the tensors it
points into, and forward to the entry points.  No arithmetic of the method lives
here; every step runs in libtempo's kernels.
"""
from __future__ import annotations

import math

import torch

from . import tempo as T

_TORCH_DTYPE = {T.TEMPO_BF16: torch.bfloat16, T.TEMPO_F32: torch.float32}


class BlockStore:
    """A paged key/value pool (the paper's block store, Section 6) for `batch`
    sequences, plus the workspace the attention entry points need.

    block_table: int32 tensor [batch][max_blocks_per_seq] (tile n -> physical
    block); by default sequence b owns blocks b*max_blocks_per_seq + n.
    fill: "nan" poisons the pool so that any read outside the visible range shows.
    """

    def __init__(self, batch, num_q_heads, num_kv_heads, head_dim, block_size, max_t, dtype,
                 device="cuda:0", num_blocks=None, block_table=None, fill="zero", pools=None,
                 ring_blocks=0):
        self.batch, self.Hq, self.Hkv, self.D, self.Z = batch, num_q_heads, num_kv_heads, head_dim, block_size
        self.dtype = dtype
        self.device = torch.device(device)
        self.ring_blocks = ring_blocks
        # a ring (window) store keeps ring_blocks blocks per sequence whatever max_t is
        self.max_blocks_per_seq = ring_blocks if ring_blocks else max_t // block_size + 1
        self.max_t = max_t if ring_blocks else self.max_blocks_per_seq * block_size - 1
        self.num_blocks = num_blocks if num_blocks is not None else batch * self.max_blocks_per_seq
        tdt = _TORCH_DTYPE[dtype]
        shape = (self.num_blocks, num_kv_heads, block_size * head_dim)
        if pools is not None:
            self.k_pool, self.v_pool = pools
            assert tuple(self.k_pool.shape) == shape and tuple(self.v_pool.shape) == shape
        elif fill == "nan":
            self.k_pool = torch.full(shape, float("nan"), dtype=tdt, device=self.device)
            self.v_pool = torch.full(shape, float("nan"), dtype=tdt, device=self.device)
        else:
            self.k_pool = torch.zeros(shape, dtype=tdt, device=self.device)
            self.v_pool = torch.zeros(shape, dtype=tdt, device=self.device)
        if block_table is None:
            block_table = torch.arange(batch * self.max_blocks_per_seq, dtype=torch.int32).reshape(
                batch, self.max_blocks_per_seq)
        self.block_table = block_table.to(device=self.device, dtype=torch.int32).contiguous()
        assert tuple(self.block_table.shape) == (batch, self.max_blocks_per_seq)
        self.kv = T.make_kv(self.k_pool, self.v_pool, self.block_table, self.num_blocks,
                            self.max_blocks_per_seq, block_size, num_kv_heads, head_dim, dtype, ring_blocks)
        # a ring store only ever answers ranges of at most ring_blocks * block_size keys,
        # which may straddle one more 32-key split than a range that starts at 0
        ws_t = ring_blocks * block_size + 32 if ring_blocks else self.max_t
        self.workspace_bytes = T.tempo_attn_workspace_bytes(self.kv, batch, num_q_heads, ws_t)
        self.workspace = torch.zeros(self.workspace_bytes, dtype=torch.uint8, device=self.device)
        self.scale = 1.0 / math.sqrt(head_dim)

    # -- forwarding ----------------------------------------------------------------
    def append(self, k_new, v_new, t, t_per_seq=None):
        T.tempo_kv_append(self.kv, k_new, v_new, self.batch, t, t_per_seq)

    def append_block(self, k_new, v_new, t, count, t_per_seq=None):
        """Write steps t .. t+count-1 (rows [batch][count][Hkv][D]) in one launch."""
        T.tempo_kv_append_block(self.kv, k_new, v_new, self.batch, t, t_per_seq, count)

    def gather(self, j0, count):
        tdt = _TORCH_DTYPE[self.dtype]
        k = torch.empty((self.batch, count, self.Hkv, self.D), dtype=tdt, device=self.device)
        v = torch.empty_like(k)
        T.tempo_kv_gather(self.kv, k, v, self.batch, j0, count)
        return k, v

    def new_out(self):
        return torch.empty((self.batch, self.Hq, self.D), dtype=_TORCH_DTYPE[self.dtype], device=self.device)

    def attend_causal(self, q, out, t, t_per_seq=None, scale=None):
        T.tempo_attn_decode_causal(self.kv, q, out, self.batch, self.Hq, t, t_per_seq,
                                   self.scale if scale is None else scale, self.workspace,
                                   self.workspace_bytes)
        return out

    def attend_window(self, q, out, t, window, t_per_seq=None, scale=None):
        T.tempo_attn_decode_window(self.kv, q, out, self.batch, self.Hq, t, t_per_seq, window,
                                   self.scale if scale is None else scale, self.workspace,
                                   self.workspace_bytes)
        return out

    def attend_padded(self, q, out, t, t_pad, t_per_seq=None, scale=None):
        """The padded + masked baseline: reads keys 0..t_pad, masks those beyond t."""
        T.tempo_attn_decode_padded_causal(self.kv, q, out, self.batch, self.Hq, t, t_per_seq, t_pad,
                                          self.scale if scale is None else scale, self.workspace,
                                          self.workspace_bytes)
        return out

    def step_causal(self, q, k_new, v_new, out, t, t_per_seq=None, scale=None):
        """Append step t and attend over 0..t in one launch."""
        T.tempo_decode_step_causal(self.kv, q, k_new, v_new, out, self.batch, self.Hq, t, t_per_seq,
                                   self.scale if scale is None else scale, self.workspace,
                                   self.workspace_bytes)
        return out

    def build_worklist(self, t_max, t_per_seq, window=0):
        """The work list of a ragged step at per-sequence steps t_per_seq (int32 device tensor): the
        non-empty (sequence, split) items, longest first.  Valid for every store of the same shape."""
        nbytes = T.tempo_attn_worklist_bytes(self.kv, self.batch, self.Hq, t_max, window)
        if nbytes == 0:
            raise T.TempoError(T.TEMPO_ERR_SHAPE, "tempo_attn_worklist_bytes")
        worklist = torch.empty(nbytes // 4, dtype=torch.int32, device=self.device)
        T.tempo_attn_worklist_build(self.kv, self.batch, self.Hq, t_max, t_per_seq, window, worklist, nbytes)
        return worklist

    def step_ragged(self, q, k_new, v_new, out, t_max, t_per_seq, worklist, window=0, scale=None):
        """The ragged step (append fused unless k_new is None) with its launch driven by a work list."""
        T.tempo_decode_step_ragged(self.kv, q, k_new, v_new, out, self.batch, self.Hq, t_max, t_per_seq, window,
                                   self.scale if scale is None else scale, worklist, self.workspace,
                                   self.workspace_bytes)
        return out

    def step_causal_noalloc(self, q, k_new, v_new, out, t, t_per_seq=None, scale=None):
        """step_causal with the split partials in the library's static device array (no workspace)."""
        T.tempo_decode_step_causal_noalloc(self.kv, q, k_new, v_new, out, self.batch, self.Hq, t, t_per_seq,
                                           self.scale if scale is None else scale)
        return out

    def step_window(self, q, k_new, v_new, out, t, window, t_per_seq=None, scale=None):
        T.tempo_decode_step_window(self.kv, q, k_new, v_new, out, self.batch, self.Hq, t, t_per_seq, window,
                                   self.scale if scale is None else scale, self.workspace,
                                   self.workspace_bytes)
        return out

    # -- rotary producer ------------------------------------------------------------
    def set_rope(self, cos_table, sin_table):
        """Tables [positions][D/2], fp32, on the store's device (kept alive here)."""
        self._rope_tables = (cos_table.contiguous(), sin_table.contiguous())
        self.rope = T.make_rope(self._rope_tables[0], self._rope_tables[1], self.D)

    def rope_rotate(self, x, y, t, t_per_seq=None):
        T.tempo_rope_rotate(self.rope, x, y, self.dtype, x.shape[0], x.shape[1], t, t_per_seq)
        return y

    def rope_append(self, k_raw, v_new, t, t_per_seq=None):
        T.tempo_rope_kv_append(self.kv, self.rope, k_raw, v_new, self.batch, t, t_per_seq)

    def rope_step(self, q_raw, k_raw, v_new, out, t, window=0, t_per_seq=None, scale=None):
        """Rotate q and k, append step t, attend: the launches of step_causal / step_window."""
        s = self.scale if scale is None else scale
        if window:
            T.tempo_rope_decode_step_window(self.kv, self.rope, q_raw, k_raw, v_new, out, self.batch, self.Hq, t,
                                            t_per_seq, window, s, self.workspace, self.workspace_bytes)
        else:
            T.tempo_rope_decode_step_causal(self.kv, self.rope, q_raw, k_raw, v_new, out, self.batch, self.Hq, t,
                                            t_per_seq, s, self.workspace, self.workspace_bytes)
        return out

    def rope_append_block(self, k_raw, v_new, t, count, t_per_seq=None):
        """Write steps t .. t+count-1 with the keys rotated to their own positions on the way in."""
        T.tempo_rope_kv_append_block(self.kv, self.rope, k_raw, v_new, self.batch, t, t_per_seq, count)

    def attend_block(self, q, out, t, queries, window=0, t_per_seq=None, scale=None, rope=False):
        """Steps t .. t+queries-1 in one call; q, out are [batch][queries][Hq][D].  With rope=True the
        queries arrive unrotated (set_rope tables)."""
        ws_t = self.ring_blocks * self.Z + 32 if self.ring_blocks else self.max_t
        nbytes = T.tempo_attn_block_workspace_bytes(self.kv, self.batch, self.Hq, queries, ws_t)
        if getattr(self, "_block_ws", None) is None or self._block_ws.numel() < nbytes:
            self._block_ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        s = self.scale if scale is None else scale
        if rope and window:
            T.tempo_rope_attn_block_window(self.kv, self.rope, q, out, self.batch, self.Hq, queries, t, t_per_seq,
                                           window, s, self._block_ws, nbytes)
        elif rope:
            T.tempo_rope_attn_block_causal(self.kv, self.rope, q, out, self.batch, self.Hq, queries, t, t_per_seq, s,
                                           self._block_ws, nbytes)
        elif window:
            T.tempo_attn_block_window(self.kv, q, out, self.batch, self.Hq, queries, t, t_per_seq, window, s,
                                      self._block_ws, nbytes)
        else:
            T.tempo_attn_block_causal(self.kv, q, out, self.batch, self.Hq, queries, t, t_per_seq, s,
                                      self._block_ws, nbytes)
        return out

    def prefill_attend(self, q, k_new, v_new, out, t, count, window=0, scale=None, count_per_seq=None,
                       rope=False):
        """Write steps t .. t+count-1 and answer all of them in one call
        (q, out [batch][count][Hq][D]; k_new, v_new [batch][count][Hkv][D]).  With
        count_per_seq (int32 device tensor) sequence b has only that many steps; with
        rope=True q and k_new arrive unrotated (set_rope tables)."""
        ws_t = self.ring_blocks * self.Z + 128 if self.ring_blocks else self.max_t
        nbytes = T.tempo_prefill_workspace_bytes(self.kv, self.batch, self.Hq, ws_t)
        if getattr(self, "_prefill_ws", None) is None or self._prefill_ws.numel() < nbytes:
            self._prefill_ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        s = self.scale if scale is None else scale
        if rope and window:
            T.tempo_rope_prefill_window(self.kv, self.rope, q, k_new, v_new, out, self.batch, self.Hq, t, count,
                                        count_per_seq, window, s, self._prefill_ws, nbytes)
        elif rope:
            T.tempo_rope_prefill_causal(self.kv, self.rope, q, k_new, v_new, out, self.batch, self.Hq, t, count,
                                        count_per_seq, s, self._prefill_ws, nbytes)
        elif window:
            T.tempo_prefill_window(self.kv, q, k_new, v_new, out, self.batch, self.Hq, t, count, count_per_seq,
                                   window, s, self._prefill_ws, nbytes)
        else:
            T.tempo_prefill_causal(self.kv, q, k_new, v_new, out, self.batch, self.Hq, t, count, count_per_seq, s,
                                   self._prefill_ws, nbytes)
        return out

    def attend_with_plan(self, q, out, t, plan, window=0, t_per_seq=None, scale=None):
        """Partial + combine with an explicit plan (its own workspace)."""
        nbytes = T.tempo_attn_plan_workspace_bytes(self.kv, self.batch, self.Hq, plan)
        if getattr(self, "_plan_ws", None) is None or self._plan_ws.numel() < nbytes:
            self._plan_ws = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        s = self.scale if scale is None else scale
        T.tempo_attn_decode_partial(self.kv, q, None, None, self.batch, self.Hq, t, t_per_seq, window, s, plan,
                                    self._plan_ws, nbytes)
        T.tempo_attn_decode_combine(self.kv, out, self.batch, self.Hq, t, t_per_seq, window, plan,
                                    self._plan_ws, nbytes)
        return out

    def prefill(self, K, V, upto, lengths=None):
        """Write steps 0..upto of flat K, V ([batch][T][Hkv][D] device tensors)
        into the pool: one tempo_kv_append_block for a linear store, one
        tempo_kv_append per step otherwise.  With `lengths` (int32 device tensor of
        per-sequence lengths) sequence b stops at its own last step."""
        if lengths is None and not self.ring_blocks:
            self.append_block(K[:, :upto + 1].contiguous(), V[:, :upto + 1].contiguous(), 0, upto + 1)
            return
        if lengths is None:
            for j in range(upto + 1):
                self.append(K[:, j].contiguous(), V[:, j].contiguous(), j)
            return
        last = (lengths.to(torch.int64) - 1).clamp_(min=0)
        ar = torch.arange(self.batch, device=self.device)
        for j in range(upto + 1):
            tj = torch.clamp(last, max=j)
            self.append(K[ar, tj].contiguous(), V[ar, tj].contiguous(), j, tj.to(torch.int32))
