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
#include "tempo_internal.h"

namespace tempo {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D>
struct Group {
  u32x4 k[2 * (D / 32)];
  u32x4 v[D / 16];
};

template <int D>
__device__ inline void load_group(const AttnParams& p, int b, int hkv, int grp, int lane, Group<D>& g) {
  const int j0 = grp << 5;
  const int tile = j0 >> p.z_log2;
  const int Z = 1 << p.z_log2;
  int phys = p.block_table[(int64_t)b * p.max_blocks_per_seq + tile];
  phys = __builtin_amdgcn_readfirstlane(clamp_block(phys, p.num_blocks));
  const int64_t base = (((int64_t)phys * p.Hkv + hkv) << p.z_log2) * D + (int64_t)(j0 & (Z - 1)) * D;
  const u32x4* kp = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.k_pool) + base) + lane;
  const u32x4* vp = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.v_pool) + base) + lane;
#pragma unroll
  for (int i = 0; i < 2 * (D / 32); ++i) g.k[i] = kp[i * 64];
#pragma unroll
  for (int i = 0; i < D / 16; ++i) g.v[i] = vp[i * 64];
}

template <int D>
struct WaveState {
  float m;              // running max (log2 units) of head lane&15
  float l;              // running sum over this lane's slots
  f32x4 acc[D / 16];    // lane (n + 16c): dims 16*dt + n of heads 4c..4c+3
};

template <int D>
__device__ inline void consume_group(const AttnParams& p, int grp, int start, int end, int lane,
                                     const u32x4* qreg, Group<D>& g, WaveState<D>& st) {
  constexpr int KS = D / 32;
  constexpr int DT = D / 16;
  const int c = lane >> 4;
  f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(g.k[s]), as_bf16x8(qreg[s]), sa, 0, 0, 0);
    sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(g.k[KS + s]), as_bf16x8(qreg[s]), sb, 0, 0, 0);
  }
  float x[8];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    x[r] = sa[r] * p.scale_log2e;
    x[4 + r] = sb[r] * p.scale_log2e;
  }
  const int j0 = grp << 5;
  if (j0 < start || j0 + 31 > end) {  // wave-uniform: a group cut by lo, by t, or by the split
    uint32_t keep[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int ja = j0 + 4 * c + r, jb = ja + 16;
      const bool va = ja >= start && ja <= end, vb = jb >= start && jb <= end;
      x[r] = va ? x[r] : -INFINITY;          // -inf mask under the max
      x[4 + r] = vb ? x[4 + r] : -INFINITY;
      // value slot e of this lane: e<4 -> slot 4c+e, e>=4 -> slot 16+4c+e-4
      const uint32_t ma = va ? 0xFFFFu : 0u, mb = vb ? 0xFFFFu : 0u;
      if ((r & 1) == 0) { keep[r >> 1] = ma; keep[2 + (r >> 1)] = mb; }
      else { keep[r >> 1] |= ma << 16; keep[2 + (r >> 1)] |= mb << 16; }
    }
    // 0 mask under the sums: unwritten slots may hold NaN, and 0 * NaN is NaN
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      g.v[dt].x &= keep[0]; g.v[dt].y &= keep[1]; g.v[dt].z &= keep[2]; g.v[dt].w &= keep[3];
    }
  }
  float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(st.m, mx);
  const float alpha = fast_exp2(st.m - m_new);  // first group: exp2(-inf) = 0
  bf16x8 pa;
  float psum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const __bf16 pb = (__bf16)fast_exp2(x[i] - m_new);
    pa[i] = pb;
    psum += (float)pb;  // the sum uses the rounded weights, so out stays a convex combination
  }
  st.l = st.l * alpha + psum;
  st.m = m_new;
  if (__any(alpha != 1.0f)) {
    float a[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) a[r] = __shfl(alpha, 4 * c + r);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int r = 0; r < 4; ++r) st.acc[dt][r] *= a[r];
    }
  }
#pragma unroll
  for (int dt = 0; dt < DT; ++dt)
    st.acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, as_bf16x8(g.v[dt]), st.acc[dt], 0, 0, 0);
}

template <int D>
__global__ __launch_bounds__(512) void attn_partial_bf16(AttnParams p) {
  constexpr int KS = D / 32;
  constexpr int DT = D / 16;
  extern __shared__ float smem[];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nwaves = blockDim.x >> 6;
  const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
  int t_b = p.t_per_seq ? p.t_per_seq[b] : p.t;
  t_b = t_b > p.t ? p.t : (t_b < 0 ? 0 : t_b);
  const SeqRange rg = seq_range(t_b, p.window, p.tps_log2);
  if (split >= rg.nchunks) return;  // uniform over the workgroup
  const int chunk = rg.chunk0 + split;
  const int cs = chunk << p.tps_log2, ce = ((chunk + 1) << p.tps_log2) - 1;
  const int start = rg.lo > cs ? rg.lo : cs;
  const int end = rg.hi < ce ? rg.hi : ce;
  const int g_last = end >> 5;

  // Query operand: lane (j + 16c) holds dims 32s + 8c .. +7 of head j of the group (0 beyond G).
  u32x4 qreg[KS];
  {
    const int j = lane & 15, c = lane >> 4;
    const uint16_t* qp = static_cast<const uint16_t*>(p.q) +
                         ((int64_t)b * p.Hq + (int64_t)hkv * p.G + j) * D + 8 * c;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const u32x4 zero = {0u, 0u, 0u, 0u};
      qreg[s] = j < p.G ? *reinterpret_cast<const u32x4*>(qp + 32 * s) : zero;
    }
  }

  WaveState<D> st;
  st.m = -INFINITY;
  st.l = 0.f;
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) st.acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Two register images of a group, used alternately: the next group's loads are
  // in flight while the current one is consumed.
  int grp = (start >> 5) + wave;
  Group<D> ga, gb;
  if (grp <= g_last) load_group<D>(p, b, hkv, grp, lane, ga);
  while (grp <= g_last) {
    if (grp + nwaves <= g_last) load_group<D>(p, b, hkv, grp + nwaves, lane, gb);
    consume_group<D>(p, grp, start, end, lane, qreg, ga, st);
    grp += nwaves;
    if (grp > g_last) break;
    if (grp + nwaves <= g_last) load_group<D>(p, b, hkv, grp + nwaves, lane, ga);
    consume_group<D>(p, grp, start, end, lane, qreg, gb, st);
    grp += nwaves;
  }

  // Wave result -> LDS.  Heads live in lane&15 for (m, l) and in (4c + r) for acc.
  float l_tot = st.l + __shfl_xor(st.l, 16);
  l_tot += __shfl_xor(l_tot, 32);
  float* sm_m = smem;                       // [nwaves][16]
  float* sm_l = smem + nwaves * 16;         // [nwaves][16]
  float* sm_acc = smem + nwaves * 32;       // [nwaves][G][D]
  if (lane < 16) {
    sm_m[wave * 16 + lane] = st.m;
    sm_l[wave * 16 + lane] = l_tot;
  }
  {
    const int n = lane & 15, c = lane >> 4;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int g = 4 * c + r;
      if (g < p.G) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) sm_acc[(wave * p.G + g) * D + 16 * dt + n] = st.acc[dt][r];
      }
    }
  }
  __syncthreads();

  // Merge the wavefronts of the workgroup (same rule the split combine uses).
  for (int idx = threadIdx.x; idx < p.G * D; idx += blockDim.x) {
    const int g = idx / D, d = idx - g * D;
    float M = -INFINITY;
    for (int w = 0; w < nwaves; ++w) M = fmaxf(M, sm_m[w * 16 + g]);
    float num = 0.f, den = 0.f;
    for (int w = 0; w < nwaves; ++w) {
      const float mw = sm_m[w * 16 + g];
      if (mw == -INFINITY) continue;  // a wavefront that had no group
      const float wgt = fast_exp2(mw - M);
      num += wgt * sm_acc[(w * p.G + g) * D + d];
      den += wgt * sm_l[w * 16 + g];
    }
    const int64_t row = (int64_t)b * p.Hq + (int64_t)hkv * p.G + g;
    if (p.direct) {
      static_cast<__bf16*>(p.out)[row * D + d] = (__bf16)(num / den);
    } else {
      const int64_t part = row * p.num_splits + split;
      p.ws_acc[part * D + d] = num;
      if (d == 0) {
        p.ws_ml[part * 2] = M;
        p.ws_ml[part * 2 + 1] = den;
      }
    }
  }
}

}  // namespace

hipError_t launch_partial_bf16(const AttnParams& p, int batch, int D, int grid_splits, int waves,
                               hipStream_t stream) {
  const dim3 grid(grid_splits, p.Hkv, batch);
  const dim3 block(64 * waves);
  const size_t lds = (size_t)waves * (32 + (size_t)p.G * D) * sizeof(float);
  if (D == 128) return launch(attn_partial_bf16<128>, grid, block, lds, stream, p);
  else return launch(attn_partial_bf16<64>, grid, block, lds, stream, p);
}

}  // namespace tempo
