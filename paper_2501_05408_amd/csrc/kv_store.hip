// Block store: in-place write of one timestep, and slice read-back.
//
// The paper's block store (Section 6) keeps a recurrent tensor in pre-allocated
// block-sized buffers that are written one timestep at a time, in place; its
// "in-place writes" kernel wrapper lets the producer write at index t directly.
// Here step t of sequence b goes to physical block block_table[b][t div Z],
// slot t mod Z (Section 4.3: tile n holds keys [nZ, (n+1)Z)).  An append may
// carry `count` consecutive steps per sequence (rows [B][count][Hkv][D]): row c
// goes to step t + c.
#include "tempo_internal.h"

namespace tempo {
namespace {

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
    const uint4 unit = *reinterpret_cast<const uint4*>(k_new + src);
    *reinterpret_cast<uint4*>(kp + base + tile_off_k_bf16(D, slot, d)) = unit;
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
