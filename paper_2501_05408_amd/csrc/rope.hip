// Rotary position embedding of the producer step, as its own launches: rotate a
// [B][H][D] tensor, and rotate-and-write a key row straight into its block-store
// slot (Section 6, "in-place writes": the producer's output goes to index t of the
// pre-allocated buffer without an intermediate tensor or copy).
//
// Dimension i < D/2 is paired with i + D/2 and the pair is turned by the angle of
// (position, i); cosines and sines come from caller-provided tables
// [positions][D/2] in fp32.  The arithmetic is fp32; bf16 results are rounded to
// nearest even once.  The attention kernels contain the same rotation for the
// fully fused decode step.
#include "tempo_internal.h"

namespace tempo {
namespace {

__device__ inline int position_of(const int32_t* t_per_seq, int t, int b) {
  int tb = t_per_seq ? t_per_seq[b] : t;
  tb = tb > t ? t : tb;  // the host validated t against the tables; never index past it
  return tb < 0 ? 0 : tb;
}

template <typename T>
__device__ inline float to_f32(T v);
template <>
__device__ inline float to_f32<float>(float v) { return v; }
template <>
__device__ inline float to_f32<__bf16>(__bf16 v) { return (float)v; }

// One thread per (b, head, i): y[i], y[i + D/2] from x[i], x[i + D/2].  x may be y.
template <typename T>
__global__ __launch_bounds__(256) void rope_rotate(const float* __restrict__ rope_cos,
                                                   const float* __restrict__ rope_sin, const T* x, T* y,
                                                   int batch, int heads, int D, int t,
                                                   const int32_t* __restrict__ t_per_seq) {
  const int half = D >> 1;
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= batch * heads * half) return;
  const int i = idx % half;
  const int row = idx / half;  // b * heads + head
  const int b = row / heads;
  const int pos = position_of(t_per_seq, t, b);
  const float c = rope_cos[(int64_t)pos * half + i], s = rope_sin[(int64_t)pos * half + i];
  const float lo = to_f32<T>(x[(int64_t)row * D + i]), hi = to_f32<T>(x[(int64_t)row * D + i + half]);
  y[(int64_t)row * D + i] = (T)rope_lo(lo, hi, c, s);
  y[(int64_t)row * D + i + half] = (T)rope_hi(lo, hi, c, s);
}

// One thread per (b, head, i): rotated key elements i and i + D/2 and value elements
// i and i + D/2 of step t go to their slots.
template <typename T, bool kBf16>
__global__ __launch_bounds__(256) void kv_rope_append(StoreParams p, const float* __restrict__ rope_cos,
                                                      const float* __restrict__ rope_sin,
                                                      const T* __restrict__ k_raw,
                                                      const T* __restrict__ v_new, int D) {
  const int half = D >> 1;
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= p.batch * p.Hkv * half) return;
  const int i = idx % half;
  const int row = idx / half;  // b * Hkv + head
  const int head = row % p.Hkv, b = row / p.Hkv;
  const int t = position_of(p.t_per_seq, p.t, b);
  const int Z = 1 << p.z_log2;
  const int tile = t >> p.z_log2, slot = t & (Z - 1);
  const int phys = clamp_block(p.block_table[(int64_t)b * p.max_blocks_per_seq + (tile & p.tile_mask)], p.num_blocks);
  const int64_t base = ((int64_t)phys * p.Hkv + head) * Z * D;
  const float c = rope_cos[(int64_t)t * half + i], s = rope_sin[(int64_t)t * half + i];
  const float lo = to_f32<T>(k_raw[(int64_t)row * D + i]), hi = to_f32<T>(k_raw[(int64_t)row * D + i + half]);
  T* kp = static_cast<T*>(p.k_pool);
  T* vp = static_cast<T*>(p.v_pool);
  const int64_t k_lo = kBf16 ? tile_off_k_bf16(D, slot, i) : tile_off_f32(D, slot, i);
  const int64_t k_hi = kBf16 ? tile_off_k_bf16(D, slot, i + half) : tile_off_f32(D, slot, i + half);
  const int64_t v_lo = kBf16 ? tile_off_v_bf16(D, slot, i) : tile_off_f32(D, slot, i);
  const int64_t v_hi = kBf16 ? tile_off_v_bf16(D, slot, i + half) : tile_off_f32(D, slot, i + half);
  kp[base + k_lo] = (T)rope_lo(lo, hi, c, s);
  kp[base + k_hi] = (T)rope_hi(lo, hi, c, s);
  vp[base + v_lo] = v_new[(int64_t)row * D + i];
  vp[base + v_hi] = v_new[(int64_t)row * D + i + half];
}

}  // namespace

hipError_t launch_rope_rotate(const float* rope_cos, const float* rope_sin, const void* x, void* y,
                              int dtype, int batch, int heads, int D, int t, const int32_t* t_per_seq,
                              hipStream_t stream) {
  const int total = batch * heads * (D / 2);
  const dim3 grid((total + 255) / 256), block(256);
  if (dtype == TEMPO_BF16)
    return launch(rope_rotate<__bf16>, grid, block, 0, stream, rope_cos, rope_sin,
                  static_cast<const __bf16*>(x), static_cast<__bf16*>(y), batch, heads, D, t, t_per_seq);
  return launch(rope_rotate<float>, grid, block, 0, stream, rope_cos, rope_sin, static_cast<const float*>(x),
                static_cast<float*>(y), batch, heads, D, t, t_per_seq);
}

hipError_t launch_rope_append(const StoreParams& p, const float* rope_cos, const float* rope_sin,
                              const void* k_raw, const void* v_new, int D, int dtype, hipStream_t stream) {
  const int total = p.batch * p.Hkv * (D / 2);
  const dim3 grid((total + 255) / 256), block(256);
  if (dtype == TEMPO_BF16)
    return launch((kv_rope_append<__bf16, true>), grid, block, 0, stream, p, rope_cos, rope_sin,
                  static_cast<const __bf16*>(k_raw), static_cast<const __bf16*>(v_new), D);
  return launch((kv_rope_append<float, false>), grid, block, 0, stream, p, rope_cos, rope_sin,
                static_cast<const float*>(k_raw), static_cast<const float*>(v_new), D);
}

}  // namespace tempo
