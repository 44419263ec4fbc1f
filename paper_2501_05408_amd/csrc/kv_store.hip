// Block store: in-place write of one timestep, and slice read-back.
//
// The paper's block store (Section 6) keeps a recurrent tensor in pre-allocated
// block-sized buffers that are written one timestep at a time, in place; its
// "in-place writes" kernel wrapper lets the producer write at index t directly.
// Here step t of sequence b goes to physical block block_table[b][t div Z],
// slot t mod Z (Section 4.3: tile n holds keys [nZ, (n+1)Z)).  An append may
// carry `count` consecutive steps per sequence (rows [B][count][Hkv][D]): row c
// goes to step t + c.
#include "attn_bf16_common.h"

namespace tempo {
namespace {

// Rows of the call that sequence b writes (all of them unless per-sequence counts are given).
__device__ inline int rows_of(const StoreParams& p, int b) {
  if (!p.count_per_seq) return INT32_MAX;
  const int n = p.count_per_seq[b];
  return n < 0 ? 0 : n;
}

__device__ inline int step_of(const StoreParams& p, int b) {
  int t = p.t_per_seq ? p.t_per_seq[b] : p.t;
  t = t > p.t ? p.t : t;  // the host validated p.t; never index past it
  return t < 0 ? 0 : t;
}

// bf16: one thread per (b, c, head, d).  V is written element by element (the
// operand-major value layout interleaves 8 slots per 16-byte unit); the thread
// with d % 8 == 0 also moves the 16-byte key unit that starts at d.
template <int D>
__global__ __launch_bounds__(256) void kv_append_bf16(StoreParams p, const uint16_t* __restrict__ k_new,
                                                      const uint16_t* __restrict__ v_new) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int total = p.batch * p.count * p.Hkv * D;
  if (idx >= total) return;
  const int d = idx % D;
  const int head = (idx / D) % p.Hkv;
  const int c = (idx / (D * p.Hkv)) % p.count;
  const int b = idx / (D * p.Hkv * p.count);
  if (p.row0 + c >= rows_of(p, b)) return;
  const int t = step_of(p, b) + c;
  const int Z = 1 << p.z_log2;
  const int tile = t >> p.z_log2, slot = t & (Z - 1);
  const int phys = clamp_block(p.block_table[(int64_t)b * p.max_blocks_per_seq + (tile & p.tile_mask)], p.num_blocks);
  const int64_t base = ((int64_t)phys * p.Hkv + head) * Z * D;
  uint16_t* vp = static_cast<uint16_t*>(p.v_pool);
  const int64_t src = (((int64_t)b * p.src_steps + c) * p.Hkv + head) * D + d;
  vp[base + tile_off_v_bf16(D, slot, d)] = v_new[src];
  if ((d & 7) == 0) {
    uint16_t* kp = static_cast<uint16_t*>(p.k_pool);
    if (!p.rope_cos) {
      const uint4 unit = *reinterpret_cast<const uint4*>(k_new + src);
      *reinterpret_cast<uint4*>(kp + base + tile_off_k_bf16(D, slot, d)) = unit;
    } else if (d < D / 2) {  // rotary: the piece at d and its partner at d + D/2 are turned together
      u32x4 lo = *reinterpret_cast<const u32x4*>(k_new + src);
      u32x4 hi = *reinterpret_cast<const u32x4*>(k_new + src + D / 2);
      rotate_pieces(p.rope_cos, p.rope_sin, t, D / 2, d, lo, hi);
      *reinterpret_cast<u32x4*>(kp + base + tile_off_k_bf16(D, slot, d)) = lo;
      *reinterpret_cast<u32x4*>(kp + base + tile_off_k_bf16(D, slot, d + D / 2)) = hi;
    }
  }
}

// bf16, whole 32-slot groups: one wavefront per (sequence, head, group) turns 32
// consecutive rows of k_new / v_new into the group's operand-major image and writes
// it as full 1 KiB units.  Keys: every 16-byte piece of a unit is 8 consecutive dims
// of one row, so it is a gather of 16-byte pieces.  Values: a 16-byte piece holds one
// dim of 8 slots, so the 32 x D tile goes through LDS (row stride D + 2 elements,
// which spreads the four rows a column tile's lanes read over different banks).
// p.t is the first step of the first group (a multiple of 32), p.count the number of
// groups times 32; rows of sequence b start at k_new[b][0].
template <int D>
__global__ __launch_bounds__(64) void kv_append_groups_bf16(StoreParams p, const uint16_t* __restrict__ k_new,
                                                            const uint16_t* __restrict__ v_new) {
  constexpr int KS = D / 32, DT = D / 16, LD = D + 2;
  __shared__ uint16_t tile[32 * LD];
  const int lane = threadIdx.x;
  const int g = blockIdx.x, head = blockIdx.y, b = blockIdx.z;
  // slots of this group that sequence b writes: all 32, or fewer where its rows end inside the group
  const int rows_b = rows_of(p, b);
  const int valid = rows_b == INT32_MAX ? 32 : rows_b - (p.row0 + 32 * g);
  if (valid <= 0) return;  // uniform over the workgroup
  const int t0 = p.t + 32 * g;  // first step of this group
  const int Z = 1 << p.z_log2;
  const int phys = clamp_block(p.block_table[(int64_t)b * p.max_blocks_per_seq + ((t0 >> p.z_log2) & p.tile_mask)],
                               p.num_blocks);
  const int64_t base = (((int64_t)phys * p.Hkv + head) << p.z_log2) * D + (int64_t)(t0 & (Z - 1)) * D;
  const int64_t row0 = ((int64_t)b * p.src_steps + 32 * g) * p.Hkv + head;  // source row of slot 0 (rows are Hkv apart)

  // values -> LDS, 16 bytes per lane and load
#pragma unroll
  for (int i = 0; i < (32 * D / 8) / 64; ++i) {
    const int piece = lane + 64 * i, row = piece / (D / 8), d8 = (piece % (D / 8)) * 8;
    const u32x4 v = *reinterpret_cast<const u32x4*>(v_new + (row0 + (int64_t)row * p.Hkv) * D + d8);
    uint32_t* dst = reinterpret_cast<uint32_t*>(tile + row * LD + d8);  // 4-byte aligned: LD and d8 are even
    dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
  }
  // keys: lane (row + 16c) of unit (tile, s) = dims 32s + 8c .. +7 of slot 16*tile + row
  {
    const int row = lane & 15, c = lane >> 4;
    u32x4* kp = reinterpret_cast<u32x4*>(static_cast<uint16_t*>(p.k_pool) + base) + lane;
#pragma unroll
    for (int tl = 0; tl < 2; ++tl) {
#pragma unroll
      for (int s = 0; s < KS / 2; ++s) {
        if (16 * tl + row < valid) {
          const uint16_t* src = k_new + (row0 + (int64_t)(16 * tl + row) * p.Hkv) * D + 32 * s + 8 * c;
          u32x4 lo = *reinterpret_cast<const u32x4*>(src);            // dims 32s + 8c .. +7
          u32x4 hi = *reinterpret_cast<const u32x4*>(src + D / 2);    // the same dims + D/2: unit s + KS/2
          if (p.rope_cos) rotate_pieces(p.rope_cos, p.rope_sin, t0 + 16 * tl + row, D / 2, 32 * s + 8 * c, lo, hi);
          kp[(tl * KS + s) * 64] = lo;
          kp[(tl * KS + s + KS / 2) * 64] = hi;
        }
      }
    }
  }
  __syncthreads();
  // values: lane (n + 16c) of unit dt = dim 16dt + n of slots {4c..4c+3, 16+4c..16+4c+3}
  {
    const int n = lane & 15, c = lane >> 4;
    u32x4* vp = reinterpret_cast<u32x4*>(static_cast<uint16_t*>(p.v_pool) + base) + lane;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
      const uint16_t* col = tile + 16 * dt + n;
      uint32_t e[8];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        e[r] = col[(4 * c + r) * LD];
        e[4 + r] = col[(16 + 4 * c + r) * LD];
      }
      u32x4 o;
      o.x = e[0] | (e[1] << 16); o.y = e[2] | (e[3] << 16);
      o.z = e[4] | (e[5] << 16); o.w = e[6] | (e[7] << 16);
      if (valid < 32) {  // the rows end inside this group: keep what the pool holds in the other slots
        uint32_t m[8];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          m[r] = (4 * c + r) < valid ? 0xFFFFu : 0u;
          m[4 + r] = (16 + 4 * c + r) < valid ? 0xFFFFu : 0u;
        }
        const u32x4 old = vp[dt * 64];
        const uint32_t mx = m[0] | (m[1] << 16), my = m[2] | (m[3] << 16);
        const uint32_t mz = m[4] | (m[5] << 16), mw = m[6] | (m[7] << 16);
        o.x = (o.x & mx) | (old.x & ~mx); o.y = (o.y & my) | (old.y & ~my);
        o.z = (o.z & mz) | (old.z & ~mz); o.w = (o.w & mw) | (old.w & ~mw);
      }
      vp[dt * 64] = o;
    }
  }
}

// f32: one thread per float4 of (b, c, head, d..d+3); both pools are row-major.
template <int D>
__global__ __launch_bounds__(256) void kv_append_f32(StoreParams p, const float* __restrict__ k_new,
                                                     const float* __restrict__ v_new) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  const int total = p.batch * p.count * p.Hkv * (D / 4);
  if (idx >= total) return;
  const int d = (idx % (D / 4)) * 4;
  const int head = (idx / (D / 4)) % p.Hkv;
  const int c = (idx / ((D / 4) * p.Hkv)) % p.count;
  const int b = idx / ((D / 4) * p.Hkv * p.count);
  if (p.row0 + c >= rows_of(p, b)) return;
  const int t = step_of(p, b) + c;
  const int Z = 1 << p.z_log2;
  const int tile = t >> p.z_log2, slot = t & (Z - 1);
  const int phys = clamp_block(p.block_table[(int64_t)b * p.max_blocks_per_seq + (tile & p.tile_mask)], p.num_blocks);
  const int64_t off = ((int64_t)phys * p.Hkv + head) * Z * D + tile_off_f32(D, slot, d);
  const int64_t src = (((int64_t)b * p.src_steps + c) * p.Hkv + head) * D + d;
  *reinterpret_cast<float4*>(static_cast<float*>(p.k_pool) + off) =
      *reinterpret_cast<const float4*>(k_new + src);
  *reinterpret_cast<float4*>(static_cast<float*>(p.v_pool) + off) =
      *reinterpret_cast<const float4*>(v_new + src);
}

// Slice read: out[b][j - j0][head][d] for j in [j0, j0 + count).  One thread per element.
template <typename T, bool kBf16>
__global__ __launch_bounds__(256) void kv_gather(StoreParams p, T* __restrict__ k_out,
                                                 T* __restrict__ v_out, int D, int j0, int count) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t total = (int64_t)p.batch * count * p.Hkv * D;
  if (idx >= total) return;
  const int d = (int)(idx % D);
  const int head = (int)((idx / D) % p.Hkv);
  const int jj = (int)((idx / ((int64_t)D * p.Hkv)) % count);
  const int b = (int)(idx / ((int64_t)D * p.Hkv * count));
  const int j = j0 + jj;
  const int Z = 1 << p.z_log2;
  const int tile = j >> p.z_log2, slot = j & (Z - 1);
  const int phys = clamp_block(p.block_table[(int64_t)b * p.max_blocks_per_seq + (tile & p.tile_mask)], p.num_blocks);
  const int64_t base = ((int64_t)phys * p.Hkv + head) * Z * D;
  if (k_out) {
    const int64_t off = kBf16 ? tile_off_k_bf16(D, slot, d) : tile_off_f32(D, slot, d);
    k_out[idx] = static_cast<const T*>(p.k_pool)[base + off];
  }
  if (v_out) {
    const int64_t off = kBf16 ? tile_off_v_bf16(D, slot, d) : tile_off_f32(D, slot, d);
    v_out[idx] = static_cast<const T*>(p.v_pool)[base + off];
  }
}

}  // namespace

hipError_t launch_append(const StoreParams& p, const void* k_new, const void* v_new, int D,
                         int dtype, hipStream_t stream) {
  // bf16, uniform first step, at least one whole 32-slot group: the groups go through
  // the group kernel, the rows before the first and after the last whole group
  // through the element-wise kernel.
  if (dtype == TEMPO_BF16 && !p.t_per_seq && p.count >= 32) {
    const int g0 = (p.t + 31) >> 5, g1 = ((p.t + p.count) >> 5) - 1;  // whole groups g0 .. g1
    if (g1 >= g0) {
      const uint16_t* k = static_cast<const uint16_t*>(k_new);
      const uint16_t* v = static_cast<const uint16_t*>(v_new);
      const int64_t row_elems = (int64_t)p.Hkv * D;
      const int head_rows = 32 * g0 - p.t, tail_first = 32 * (g1 + 1), tail_rows = p.t + p.count - tail_first;
      hipError_t e = hipSuccess;
      if (head_rows > 0) {
        StoreParams h = p;
        h.count = head_rows;  // row0 stays: these are the call's first rows
        e = launch_append(h, k, v, D, dtype, stream);
        if (e != hipSuccess) return e;
      }
      StoreParams m = p;
      m.t = 32 * g0;
      m.count = 32 * (g1 - g0 + 1);
      m.row0 = p.row0 + head_rows;
      const dim3 grid(g1 - g0 + 1, p.Hkv, p.batch);
      const uint16_t* km = k + head_rows * row_elems;
      const uint16_t* vm = v + head_rows * row_elems;
      e = D == 128 ? launch(kv_append_groups_bf16<128>, grid, dim3(64), 0, stream, m, km, vm)
                   : launch(kv_append_groups_bf16<64>, grid, dim3(64), 0, stream, m, km, vm);
      if (e != hipSuccess) return e;
      if (tail_rows > 0) {
        StoreParams tl = p;
        tl.t = tail_first;
        tl.count = tail_rows;
        tl.row0 = p.row0 + (tail_first - p.t);
        e = launch_append(tl, k + (tail_first - p.t) * row_elems, v + (tail_first - p.t) * row_elems, D, dtype, stream);
      }
      return e;
    }
  }
  const int threads = 256;
  if (dtype == TEMPO_BF16) {
    const int total = p.batch * p.count * p.Hkv * D;
    const dim3 grid((total + threads - 1) / threads);
    const uint16_t* k = static_cast<const uint16_t*>(k_new);
    const uint16_t* v = static_cast<const uint16_t*>(v_new);
    if (D == 128) return launch(kv_append_bf16<128>, grid, dim3(threads), 0, stream, p, k, v);
    else return launch(kv_append_bf16<64>, grid, dim3(threads), 0, stream, p, k, v);
  } else {
    const int total = p.batch * p.count * p.Hkv * (D / 4);
    const dim3 grid((total + threads - 1) / threads);
    const float* k = static_cast<const float*>(k_new);
    const float* v = static_cast<const float*>(v_new);
    if (D == 128) return launch(kv_append_f32<128>, grid, dim3(threads), 0, stream, p, k, v);
    else return launch(kv_append_f32<64>, grid, dim3(threads), 0, stream, p, k, v);
  }
}

hipError_t launch_gather(const StoreParams& p, void* k_out, void* v_out, int D, int dtype, int j0,
                         int count, hipStream_t stream) {
  const int threads = 256;
  const int64_t total = (int64_t)p.batch * count * p.Hkv * D;
  if (total == 0) return hipSuccess;
  const dim3 grid((unsigned)((total + threads - 1) / threads));
  if (dtype == TEMPO_BF16) {
    return launch((kv_gather<uint16_t, true>), grid, dim3(threads), 0, stream, p,
                       static_cast<uint16_t*>(k_out), static_cast<uint16_t*>(v_out), D, j0, count);
  } else {
    return launch((kv_gather<float, false>), grid, dim3(threads), 0, stream, p,
                       static_cast<float*>(k_out), static_cast<float*>(v_out), D, j0, count);
  }
}

}  // namespace tempo
