// Partial attention of one split, bf16 keys/values, MFMA on gfx950.
//
// What is computed (Section 2, Eq. 1, restricted to one split of the visible
// range; Section 4.3: per-tile reductions with a -inf mask under the max and a
// 0 mask under the sums): for the G query heads that share one key/value head,
//     m   = max_j  s * <q_g, k_j>
//     l   = sum_j  exp(s * <q_g, k_j> - m)
//     acc = sum_j  exp(s * <q_g, k_j> - m) * v_j
// over the split's key positions j, kept as running values (online softmax) in
// fp32 and in base-2 units (s * log2(e) is folded into one multiply).
//
// Mapping.  One workgroup = one (sequence, kv head, split); its wavefronts take
// the split's 32-slot groups round-robin.  A group is 8 KiB of keys and 8 KiB of
// values (D = 128) that the block store already holds in MFMA operand order, so
// each wavefront streams them with 16-byte-per-lane, 1-KiB-per-instruction loads
// straight into operand registers: no LDS staging, no transposition.
//   S^T tile  = K(16 slots x 32 dims) * Q^T(32 dims x 16 heads)   2 row tiles x D/32 steps
//   acc tile  = P(16 heads x 32 slots) * V(32 slots x 16 dims)    D/16 column tiles
// The accumulator image of the two S tiles (lane = head + 16c, registers =
// slots 4c..4c+3 of each tile) is, after exp and bf16 rounding, exactly the
// A-operand image of the P.V product, because the value layout orders its 8
// contraction slots per lane as {4c..4c+3, 16+4c..16+4c+3}.
// Only G of the 16 head columns carry data (G = 3 for the Llama shape): the MFMA
// is mostly padding, which is free here -- the kernel is bound by HBM reads.
//
// Padded baseline.  With pad_t set the kernel reads keys and values up to pad_t
// whatever the step is and masks what lies beyond the step: the static-shape
// formulation (Section 2.1, workaround (c)) that the dynamic range is measured
// against.
//
// Block of queries.  The 16 columns can also hold C consecutive query steps of
// the G heads (column = c*G + g, C*G <= 16): step t+c sees keys up to t+c (and
// from its own window start), which is one more per-lane bound in the index mask.
// The keys and values are still read once, now for C steps.  Blocks of more than
// 16 columns are served by the LDS-staged kernel of attn_prefill_bf16.hip.
//
// Rotary embedding (kRope instantiations).  q, and the k_new of a fused append,
// arrive unrotated; the kernel turns them to their step's position with fp32
// arithmetic and rounds to bf16 once, so the producer's output never exists as a
// tensor of its own (Section 6, "in-place writes", applied to the whole step).
// Dimension i pairs with i + D/2: for q both live in the same lane (operand
// registers s and s + D/64), for the fetched key row in lanes l and l ^ (D/16).
//
// Pipeline.  A wavefront owns ONE register image of a group (keys: 2*D/32 units,
// values: D/16 units) and refills each half as soon as the MFMAs that read it
// have been issued: the next group's keys are requested right after Q.K^T, its
// values right after P.V.  About one group (16 KiB) per wavefront is therefore in
// flight all the time, without a second register image; how many bytes a compute
// unit keeps in flight is then set by the number of resident wavefronts.
#include "attn_bf16_common.h"

namespace tempo {
namespace {

// ---- fused block-store write (Section 6, "in-place writes") --------------------
// Step t's own key and value arrive in k_new / v_new.  The wavefront that owns the
// group holding slot t fetches those two rows when it starts, and when it reaches
// that group it puts them into the group's register image, so that this step
// attends over them, and into the pool, so that later steps do.

// Lanes 0..D/8-1 fetch the new key row, the next D/8 lanes the new value row, 16
// bytes each.  Nothing waits for this load until the group is reached.
template <int D>
__device__ inline u32x4 fetch_new_row(const AttnParams& p, int b, int hkv, int lane) {
  constexpr int UNITS = D / 8;
  u32x4 v = {0u, 0u, 0u, 0u};
  if (lane < 2 * UNITS) {
    const uint16_t* src = static_cast<const uint16_t*>(lane < UNITS ? p.k_new : p.v_new) +
                          ((int64_t)b * p.Hkv + hkv) * D + (lane % UNITS) * 8;
    v = *reinterpret_cast<const u32x4*>(src);
  }
  return v;
}

// Keys: lanes (row + 16c) hold the units of slot `row`; patch them, then the whole
// wavefront writes the group's key image back as full 1 KiB units (the other slots
// are rewritten with the values just read -- nobody else writes this sequence's
// group -- so the pool sees whole cache lines, not 16-byte fragments).
template <int D>
__device__ __forceinline__ void append_keys(const AttnParams& p, int64_t base, int t_b, int lane,
                                            u32x4 fetched, uint16_t* stage, Group<D>& g) {
  constexpr int KS = D / 32;
  const int u = t_b & 31, row = u & 15, tile = u >> 4;
  const int n = lane & 15, c = lane >> 4;
  // the two fetched rows go through LDS to reach the lanes that need them
  if (lane < 2 * (D / 8)) *reinterpret_cast<u32x4*>(stage + lane * 8) = fetched;
  if (n == row) {
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const u32x4 val = *reinterpret_cast<const u32x4*>(stage + 32 * s + 8 * c);
      g.k[s] = tile == 0 ? val : g.k[s];
      g.k[KS + s] = tile == 1 ? val : g.k[KS + s];
    }
  }
  u32x4* kp = reinterpret_cast<u32x4*>(static_cast<uint16_t*>(p.k_pool) + base) + lane;
#pragma unroll
  for (int i = 0; i < 2 * KS; ++i) kp[i * 64] = g.k[i];  // both row-tiles: static register indices
}

// Values: lanes (n + 16c) with c = row>>2 hold dim 16dt+n of the 8 slots that
// include slot t; patch that 16-bit element and write the 16-byte unit back
// (16 lanes x 16 bytes = 256 contiguous bytes per column tile).  Called after
// append_keys of the same group, which staged the value row at stage[D..2D).
template <int D>
__device__ __forceinline__ void append_values(const AttnParams& p, int64_t base, int t_b, int lane,
                                              const uint16_t* stage, Group<D>& g) {
  constexpr int DT = D / 16;
  const int u = t_b & 31, row = u & 15, tile = u >> 4;
  const int n = lane & 15, c = lane >> 4;
  if (c == (row >> 2)) {
    const int e = (row & 3) + 4 * tile;  // position of slot t among the lane's 8 slots
    u32x4* vp = reinterpret_cast<u32x4*>(static_cast<uint16_t*>(p.v_pool) + base) + lane;
    const uint32_t shift = (e & 1) ? 16u : 0u;
    const uint32_t keep = (e & 1) ? 0x0000FFFFu : 0xFFFF0000u;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const uint32_t val = stage[D + 16 * dt + n];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t patched = (g.v[dt][w] & keep) | (val << shift);
        g.v[dt][w] = (w == (e >> 1)) ? patched : g.v[dt][w];
      }
      vp[dt * 64] = g.v[dt];
    }
  }
}

// ---- rotary embedding of the fetched key row ---------------------------------------
// The row pair fetch_new_row returned: lanes 0..D/8-1 hold the key row (lane l:
// dims 8l .. 8l+7), whose partner dims sit in lane l ^ (D/16).  All lanes call this.
template <int D>
__device__ inline u32x4 rotate_fetched_key(const AttnParams& p, int pos, int lane, u32x4 fetched) {
  constexpr int UNITS = D / 8;
  u32x4 other;
#pragma unroll
  for (int w = 0; w < 4; ++w) other[w] = __shfl_xor(fetched[w], UNITS / 2);
  if (lane < UNITS) {
    float cs[8], sn[8], x[8], o[8], y[8];
    load_angles(p.rope_cos, pos, D / 2, 8 * (lane % (UNITS / 2)), cs);
    load_angles(p.rope_sin, pos, D / 2, 8 * (lane % (UNITS / 2)), sn);
    unpack8(fetched, x);
    unpack8(other, o);
    const bool first = lane < UNITS / 2;  // dims below D/2: y = x cos - partner sin
#pragma unroll
    for (int e = 0; e < 8; ++e)
      y[e] = first ? rope_lo(x[e], o[e], cs[e], sn[e]) : rope_hi(o[e], x[e], cs[e], sn[e]);
    fetched = pack8(y);
  }
  return fetched;
}

// ---- merge of the workgroup's wavefronts -----------------------------------------------
// Every wavefront has left its (m, l) per column at smem[w][16] / smem[NW][w][16] and its
// accumulators at smem[2*NW*16 ...][w][ncols][D].  Thread idx owns element (column j, dim d):
// all NW wavefronts' values of that element are requested at once, so the merge costs one trip
// to LDS, not one per wavefront.  NW is a template parameter so that no wave-count predicate
// sits between the barrier and the stores.
template <int D, int NW>
__device__ __forceinline__ void merge_waves(const AttnParams& p, const float* smem, int ncols, int b, int hkv, int split) {
  const float* sm_m = smem;
  const float* sm_l = smem + NW * 16;
  const float* sm_acc = smem + NW * 32;
  for (int idx = threadIdx.x; idx < ncols * D; idx += 64 * NW) {
    const int j = idx / D, d = idx - j * D;
    float mw[NW], lw[NW], aw[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      mw[w] = sm_m[w * 16 + j];
      lw[w] = sm_l[w * 16 + j];
      aw[w] = sm_acc[(w * ncols + j) * D + d];
    }
    float M = mw[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) M = fmaxf(M, mw[w]);
    float num = 0.f, den = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      // a wavefront that saw no key of this column contributes nothing, whatever it holds
      const bool seen = mw[w] != -INFINITY;
      const float wgt = fast_exp2(mw[w] - M);
      num += seen ? wgt * aw[w] : 0.f;
      den += seen ? wgt * lw[w] : 0.f;
    }
    const int jc = p.queries == 1 ? 0 : j / p.G, jg = j - jc * p.G;
    if (p.direct) {
      const int64_t orow = ((int64_t)b * p.io_steps + jc) * p.Hq + (int64_t)hkv * p.G + jg;
      static_cast<__bf16*>(p.out)[orow * D + d] = (__bf16)(num / den);
    } else {
      const int64_t row = ((int64_t)b * p.queries + jc) * p.Hq + (int64_t)hkv * p.G + jg;
      const int64_t part = row * p.num_splits + split;
      p.ws_acc[part * D + d] = num;
      if (d == 0) {
        p.ws_ml[part * 2] = M;
        p.ws_ml[part * 2 + 1] = den;
      }
    }
  }
}

template <int D, bool kRope, bool kList>
__global__ __launch_bounds__(512) void attn_partial_bf16(AttnParams p) {
  constexpr int KS = D / 32;
  constexpr int DT = D / 16;
  extern __shared__ float smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nwaves = blockDim.x >> 6;
  const int hkv = blockIdx.x;
  // Which (sequence, split) this workgroup takes: its grid position, or, for a ragged batch
  // with a work list, the list's item (non-empty items only, longest first).
  // (A template parameter, not a test of the pointer: a branch here sits in front of the
  // argument -> table -> data chain of EVERY launch and cost 0.3 us when it was one.)
  int b = blockIdx.y, zsplit = blockIdx.z;
  if (kList) {
    const_i32_ptr list = (const_i32_ptr)p.worklist;
    if ((int)blockIdx.y >= list[0]) return;  // uniform over the workgroup
    const int item = list[1 + blockIdx.y];
    b = item & 0xFFFF;
    zsplit = (int)((unsigned)item >> 16);
  }
  int t_b = p.t_per_seq ? ((const_i32_ptr)p.t_per_seq)[b] : p.t;
  t_b = t_b > p.t ? p.t : (t_b < 0 ? 0 : t_b);
  const SeqRange rg = seq_range(t_b, p.window, p.tps_log2, p.queries, p.pad_t);
  if (zsplit >= rg.nchunks) return;  // uniform over the workgroup
  // Dispatch order: the split index is the slowest grid dimension and runs from
  // the newest split to the oldest.  The newest split of every (sequence, head)
  // is the one a fused append lands in and the one t may cut short; launching
  // all of those first keeps their longer path out of the launch's last round.
  // (A work list names the split itself.)
  const int split = kList ? zsplit : rg.nchunks - 1 - zsplit;
  const int chunk = rg.chunk0 + split;
  const int cs = chunk << p.tps_log2, ce = ((chunk + 1) << p.tps_log2) - 1;
  const int start = rg.lo > cs ? rg.lo : cs;
  const int end = rg.hi < ce ? rg.hi : ce;
  const int g_last = end >> 5;

  // The first group's keys and values are requested before anything else.
  int grp = (start >> 5) + wave;
  Group<D> g;
  int64_t base = 0;
  if (grp <= g_last) {
    base = group_base<D>(p, b, hkv, grp);
    load_keys<D>(p, base, lane, g);
    load_values<D>(p, base, lane, g);
  }

  // Columns: j = cq*G + gq for query step cq and head gq of the group; ncols = C*G <= 16.
  const int ncols = p.queries * p.G;

  // A fused append lands in group t_b>>5, which only the newest split holds; the
  // wavefront that will reach that group fetches the new rows right away.  Its LDS
  // staging area is a region of its own behind the wave-merge area.
  int grp_new = -1;
  uint16_t* stage = reinterpret_cast<uint16_t*>(smem + nwaves * (32 + ncols * D));
  u32x4 fetched = {0u, 0u, 0u, 0u};
  if (p.k_new && split == rg.nchunks - 1 && ((t_b >> 5) - grp) % nwaves == 0 && (t_b >> 5) >= grp) {
    grp_new = t_b >> 5;
    fetched = fetch_new_row<D>(p, b, hkv, lane);
    if (kRope) fetched = rotate_fetched_key<D>(p, t_b, lane, fetched);
  }

  // The bounds that decide whether a group is cut by any column (a group inside
  // [all_lo, all_hi] needs no mask): the last query's window start, the first query's step.
  int lo_last = (p.window > 0 && (t_b + p.queries - 1) - p.window + 1 > 0) ? (t_b + p.queries - 1) - p.window + 1 : 0;
  const int all_lo = lo_last > start ? lo_last : start;
  const int all_hi = t_b < end ? t_b : end;
  // last key any column sees (below `end` only for the padded baseline, whose extra
  // keys are read, masked out of the logits and zeroed in the value operand)
  const int seen_hi = (t_b + p.queries - 1) < end ? (t_b + p.queries - 1) : end;

  // This lane's column, its own range cut to the split, and its query operand: lane
  // (j + 16c) holds dims 32s + 8c .. +7 of column j (0 for unused columns, which
  // behave like the last query step).
  const int col = lane & 15;
  const int cq = col < ncols ? col / p.G : p.queries - 1;
  const int gq = col < ncols ? col - cq * p.G : 0;
  const int hi_col = (t_b + cq) < end ? (t_b + cq) : end;
  const int lo_q = (p.window > 0 && t_b + cq - p.window + 1 > 0) ? t_b + cq - p.window + 1 : 0;
  const int lo_col = lo_q > start ? lo_q : start;
  u32x4 qreg[KS];
  {
    const int c = lane >> 4;
    const uint16_t* qp = static_cast<const uint16_t*>(p.q) +
                         (((int64_t)b * p.io_steps + cq) * p.Hq + (int64_t)hkv * p.G + gq) * D + 8 * c;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const u32x4 zero = {0u, 0u, 0u, 0u};
      const u32x4 v = *reinterpret_cast<const u32x4*>(qp + 32 * s);
      qreg[s] = col < ncols ? v : zero;
    }
  }
  if (kRope) rotate_query<D>(p, t_b + cq, lane, qreg);

  WaveState<D> st;
  st.m = -INFINITY;
  st.l = 0.f;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) st.acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  while (grp <= g_last) {
    const int nxt = grp + nwaves;
    const bool more = nxt <= g_last;
    const int64_t base_nxt = more ? group_base<D>(p, b, hkv, nxt) : 0;  // scalar loads, off the vector path
    if (grp == grp_new) append_keys<D>(p, base, t_b, lane, fetched, stage, g);

    float x[8];
    logits_of_group<D>(p, qreg, g, x);
    if (more) load_keys<D>(p, base_nxt, lane, g);  // the key registers are free again

    uint32_t keep[4] = {~0u, ~0u, ~0u, ~0u};
    const bool cut = (grp << 5) < all_lo || (grp << 5) + 31 > all_hi;  // wave-uniform
    if (cut) {
      mask_logits(grp, lo_col, hi_col, lane, x);
      value_masks(grp, start, seen_hi, lane, keep);
    }
    const bf16x8 pa = softmax_update<D>(x, lane, st);

    if (grp == grp_new) append_values<D>(p, base, t_b, lane, stage, g);
    // 0 mask under the sums: unwritten slots may hold NaN, and 0 * NaN is NaN.  The mask (all
    // ones for a group no range cuts) is applied to a copy that feeds the product, never to
    // the group's registers themselves.
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      u32x4 vv = g.v[dt];
      vv.x &= keep[0]; vv.y &= keep[1]; vv.z &= keep[2]; vv.w &= keep[3];
      st.acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, as_bf16x8(vv), st.acc[dt], 0, 0, 0);
    }
    if (more) load_values<D>(p, base_nxt, lane, g);  // the value registers are free again

    grp = nxt;
    base = base_nxt;
  }

  // Wave result -> LDS.  Columns live in lane&15 for (m, l) and in (4c + r) for acc.
  const float l_tot = column_sum(st.l);
  float* sm_m = smem;                       // [nwaves][16]
  float* sm_l = smem + nwaves * 16;         // [nwaves][16]
  float* sm_acc = smem + nwaves * 32;       // [nwaves][ncols][D]
  if (lane < 16) {
    sm_m[wave * 16 + lane] = st.m;
    sm_l[wave * 16 + lane] = l_tot;
  }
  {
    const int n = lane & 15, c = lane >> 4;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int j = 4 * c + r;
      if (j < ncols) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) sm_acc[(wave * ncols + j) * D + 16 * dt + n] = st.acc[dt][r];
      }
    }
  }
  __syncthreads();

  // Merge the wavefronts of the workgroup (same rule the split combine uses).  A
  // column that saw no key in this split leaves (m, l, acc) = (-inf, 0, 0).
  if (nwaves == 8) merge_waves<D, 8>(p, smem, ncols, b, hkv, split);
  else if (nwaves == 4) merge_waves<D, 4>(p, smem, ncols, b, hkv, split);
  else if (nwaves == 2) merge_waves<D, 2>(p, smem, ncols, b, hkv, split);
  else merge_waves<D, 1>(p, smem, ncols, b, hkv, split);
}

}  // namespace

size_t partial_bf16_lds_bytes(int waves, int columns, int D) {
  // wave-merge area, then room for one staged key row and one value row (bf16)
  return (size_t)waves * (32 + (size_t)columns * D) * sizeof(float) + 2 * (size_t)D * sizeof(uint16_t);
}

// Up to 16 (step, head) columns; wider blocks use the LDS-staged kernel.
hipError_t launch_partial_bf16(const AttnParams& p, int batch, int D, int grid_splits, int waves,
                               hipStream_t stream) {
  if (p.queries * p.G > 16) return hipErrorInvalidConfiguration;
  // with a work list: one grid row per possible item, the rows beyond the list's count exit at once
  const dim3 grid = p.worklist ? dim3(p.Hkv, (unsigned)((int64_t)batch * grid_splits), 1) : dim3(p.Hkv, batch, grid_splits);
  if (grid.y > 65535u) return hipErrorInvalidConfiguration;
  const dim3 block(64 * waves);
  const size_t lds = partial_bf16_lds_bytes(waves, p.queries * p.G, D);
  if (p.worklist) {
    if (p.rope_cos) return hipErrorInvalidConfiguration;  // no caller combines the two
    if (D == 128) return launch((attn_partial_bf16<128, false, true>), grid, block, lds, stream, p);
    return launch((attn_partial_bf16<64, false, true>), grid, block, lds, stream, p);
  }
  if (p.rope_cos) {
    if (D == 128) return launch((attn_partial_bf16<128, true, false>), grid, block, lds, stream, p);
    return launch((attn_partial_bf16<64, true, false>), grid, block, lds, stream, p);
  }
  if (D == 128) return launch((attn_partial_bf16<128, false, false>), grid, block, lds, stream, p);
  return launch((attn_partial_bf16<64, false, false>), grid, block, lds, stream, p);
}

}  // namespace tempo
