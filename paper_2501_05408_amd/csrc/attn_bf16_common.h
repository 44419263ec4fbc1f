// Pieces shared by the bf16 attention kernels (decode / block partial attention and
// prompt processing): operand register types, the block-store addressing of a
// 32-slot group, and the phases of one group (Q.K^T, index masks of Section 4.3,
// online softmax).  See attn_partial_bf16.hip for the operand layouts.
#pragma once

#include "tempo_internal.h"

namespace tempo {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// The block table is not written while a launch is in flight.  Reading it
// through the constant address space lets the compiler use scalar loads, whose
// completion is tracked apart from the key/value vector loads, although the
// kernel also stores to global memory.
typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr;

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int D>
struct Group {
  u32x4 k[2 * (D / 32)];
  u32x4 v[D / 16];
};

template <int D>
struct WaveState {
  float m;              // running max (log2 units) of head lane&15
  float l;              // running sum over this lane's slots
  f32x4 acc[D / 16];    // lane (n + 16c): dims 16*dt + n of heads 4c..4c+3
};

// Element offset, in either pool, of 32-slot group `grp` of (sequence b, kv head hkv).
template <int D>
__device__ inline int64_t group_base(const AttnParams& p, int b, int hkv, int grp) {
  const int Z = 1 << p.z_log2;
  const_i32_ptr table = (const_i32_ptr)p.block_table;
  const int entry = table[(int64_t)b * p.max_blocks_per_seq + (((grp << 5) >> p.z_log2) & p.tile_mask)];
  const int phys = clamp_block(entry, p.num_blocks);
  return (((int64_t)phys * p.Hkv + hkv) << p.z_log2) * D + (int64_t)((grp << 5) & (Z - 1)) * D;
}

// Keys and values are read once per step and never again by this kernel:
// non-temporal loads keep them from displacing anything in the caches.
template <int D>
__device__ inline void load_keys(const AttnParams& p, int64_t base, int lane, Group<D>& g) {
  const u32x4* kp = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.k_pool) + base) + lane;
#pragma unroll
  for (int i = 0; i < 2 * (D / 32); ++i) g.k[i] = __builtin_nontemporal_load(kp + i * 64);
}

template <int D>
__device__ inline void load_values(const AttnParams& p, int64_t base, int lane, Group<D>& g) {
  const u32x4* vp = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.v_pool) + base) + lane;
#pragma unroll
  for (int i = 0; i < D / 16; ++i) g.v[i] = __builtin_nontemporal_load(vp + i * 64);
}

// ---- the phases of a group ---------------------------------------------------------

// ---- rotary embedding on 16-byte pieces ----------------------------------------------
__device__ inline void unpack8(u32x4 v, float* f) {
  const bf16x8 b = as_bf16x8(v);
#pragma unroll
  for (int e = 0; e < 8; ++e) f[e] = (float)b[e];
}
__device__ inline u32x4 pack8(const float* f) {
  bf16x8 b;
#pragma unroll
  for (int e = 0; e < 8; ++e) b[e] = (__bf16)f[e];  // round to nearest even
  return __builtin_bit_cast(u32x4, b);
}
// 8 consecutive table entries starting at entry i0 of row `pos`.
__device__ inline void load_angles(const float* table, int64_t pos, int half, int i0, float* f) {
  const float4* src = reinterpret_cast<const float4*>(table + pos * half + i0);
  const float4 a = src[0], b = src[1];
  f[0] = a.x; f[1] = a.y; f[2] = a.z; f[3] = a.w;
  f[4] = b.x; f[5] = b.y; f[6] = b.z; f[7] = b.w;
}
// Two pieces of one head vector, dims i0 .. i0+7 (`lo`) and i0 + half .. (`hi`), turned
// to position `pos`; the one place where bf16 pieces are rotated, so that every kernel
// produces the same bits.
__device__ inline void rotate_pieces(const float* rope_cos, const float* rope_sin, int64_t pos, int half, int i0,
                                     u32x4& lo, u32x4& hi) {
  float cs[8], sn[8], x[8], y[8], xl[8], yh[8];
  load_angles(rope_cos, pos, half, i0, cs);
  load_angles(rope_sin, pos, half, i0, sn);
  unpack8(lo, x);
  unpack8(hi, y);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    xl[e] = rope_lo(x[e], y[e], cs[e], sn[e]);
    yh[e] = rope_hi(x[e], y[e], cs[e], sn[e]);
  }
  lo = pack8(xl);
  hi = pack8(yh);
}

// Query operand registers: qreg[s] holds dims 32s + 8c .. +7, its partner qreg[s + KS/2].
template <int D>
__device__ inline void rotate_query(const AttnParams& p, int pos, int lane, u32x4* qreg) {
  constexpr int KS = D / 32;
  const int c = lane >> 4;
#pragma unroll
  for (int s = 0; s < KS / 2; ++s)
    rotate_pieces(p.rope_cos, p.rope_sin, pos, D / 2, 32 * s + 8 * c, qreg[s], qreg[s + KS / 2]);
}

// Q.K^T for the group's two row tiles; logits in base-2 units.
template <int D>
__device__ inline void logits_of_group(const AttnParams& p, const u32x4* qreg, const Group<D>& g, float* x) {
  constexpr int KS = D / 32;
  f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int s = 0; s < KS; ++s) {
    sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(g.k[s]), as_bf16x8(qreg[s]), sa, 0, 0, 0);
    sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(g.k[KS + s]), as_bf16x8(qreg[s]), sb, 0, 0, 0);
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    x[r] = sa[r] * p.scale_log2e;
    x[4 + r] = sb[r] * p.scale_log2e;
  }
}

// Index masks for a group that some column's range cuts (wave-uniform decision by
// the caller).  Logits: -inf outside THIS lane's column range [lo_col, hi_col].
__device__ inline void mask_logits(int grp, int lo_col, int hi_col, int lane, float* x) {
  const int j0 = grp << 5;
  const int c = lane >> 4;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int ja = j0 + 4 * c + r, jb = ja + 16;
    x[r] = (ja >= lo_col && ja <= hi_col) ? x[r] : -INFINITY;          // -inf mask under the max
    x[4 + r] = (jb >= lo_col && jb <= hi_col) ? x[4 + r] : -INFINITY;
  }
}

// Values: `keep` zeroes the slots outside [v_lo, v_hi], the union of all columns'
// ranges (a slot another column still sees must keep its value; this column's
// weight for it is exactly 0).
__device__ inline void value_masks(int grp, int v_lo, int v_hi, int lane, uint32_t* keep) {
  const int j0 = grp << 5;
  const int c = lane >> 4;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int ja = j0 + 4 * c + r, jb = ja + 16;
    // value slot e of this lane: e<4 -> slot 4c+e, e>=4 -> slot 16+4c+e-4
    const uint32_t ma = (ja >= v_lo && ja <= v_hi) ? 0xFFFFu : 0u, mb = (jb >= v_lo && jb <= v_hi) ? 0xFFFFu : 0u;
    if ((r & 1) == 0) { keep[r >> 1] = ma; keep[2 + (r >> 1)] = mb; }
    else { keep[r >> 1] |= ma << 16; keep[2 + (r >> 1)] |= mb << 16; }
  }
}

// Maximum over the four lanes {l, l^16, l^32, l^48} that hold one column's logits,
// left in all four.  Two lane-swap instructions of gfx950 instead of two trips
// through the LDS permute unit: v_permlane16_swap exchanges the odd 16-lane rows of
// its first operand with the even rows of its second, v_permlane32_swap the upper
// half of the first with the lower half of the second; with both operands holding
// the same values, the maximum of the two results is the exchange-and-reduce step.
__device__ inline float column_max(float v) {
  float a = v, b = v;
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 0\n\tv_max_f32 %0, %0, %1" : "+v"(a), "+v"(b));
  float c = a, d = a;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 0\n\tv_max_f32 %0, %0, %1" : "+v"(c), "+v"(d));
  return c;
}

// The same exchange with a sum: the total over the four lanes that hold one column's partial sums.
__device__ inline float column_sum(float v) {
  float a = v, b = v;
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 0\n\tv_add_f32 %0, %0, %1" : "+v"(a), "+v"(b));
  float c = a, d = a;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 0\n\tv_add_f32 %0, %0, %1" : "+v"(c), "+v"(d));
  return c;
}

// Online-softmax update of (m, l), rescale of acc, and the bf16 weights of this group.
template <int D>
__device__ inline bf16x8 softmax_update(const float* x, int lane, WaveState<D>& st) {
  constexpr int DT = D / 16;
  const int c = lane >> 4;
  float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
  mx = column_max(mx);  // lane swaps, not two trips through the LDS permute unit
  const float m_new = fmaxf(st.m, mx);
  // A column may have seen no key yet (block of queries: a group beyond an early
  // query's step): keep -inf as its max but exponentiate against 0, never -inf - -inf.
  const float m_ref = m_new == -INFINITY ? 0.f : m_new;
  const float alpha = fast_exp2(st.m - m_ref);  // first keys of a column: exp2(-inf) = 0
  bf16x8 pa;
  float psum = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const __bf16 pb = (__bf16)fast_exp2(x[i] - m_ref);
    pa[i] = pb;
    psum += (float)pb;  // the sum uses the rounded weights, so out stays a convex combination
  }
  st.l = st.l * alpha + psum;
  const bool rescale = alpha != 1.0f && st.m != -INFINITY;  // a column that had seen no key holds zeros: nothing to scale
  st.m = m_new;
  if (__any(rescale)) {
    float a[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) a[r] = __shfl(alpha, 4 * c + r);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int r = 0; r < 4; ++r) st.acc[dt][r] *= a[r];
    }
  }
  return pa;
}

}  // namespace
}  // namespace tempo
