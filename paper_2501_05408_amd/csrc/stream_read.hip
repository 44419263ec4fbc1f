// A plain streaming read of a device buffer: the achievable-bandwidth yardstick
// the attention kernel is compared with (same bytes, same 16-byte-per-lane
// non-temporal loads, no arithmetic beyond an XOR that keeps the loads alive).  Also the
// "copy kernel of known size" that hardware traffic counters are scaled by.
#include "tempo_internal.h"

namespace tempo {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// One workgroup of 256 threads reads kUnroll consecutive 4 KiB slabs per trip.
constexpr int kUnroll = 8;

__global__ __launch_bounds__(256) void stream_read(const u32x4* __restrict__ src, size_t n_vec,
                                                   uint32_t* __restrict__ sink) {
  const size_t per_wg = (size_t)256 * kUnroll;
  u32x4 acc = {0u, 0u, 0u, 0u};
  for (size_t base = (size_t)blockIdx.x * per_wg; base < n_vec; base += (size_t)gridDim.x * per_wg) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const size_t idx = base + (size_t)i * 256 + threadIdx.x;
      const u32x4 zero = {0u, 0u, 0u, 0u};
      v[i] = idx < n_vec ? __builtin_nontemporal_load(src + idx) : zero;
    }
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) acc ^= v[i];
  }
  // never true for real data in practice; keeps the loads from being optimised away
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u && sink) sink[0] = acc.x;
}

// The same walk, writing what it reads to dst: a copy of known size.
__global__ __launch_bounds__(256) void stream_copy(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                   size_t n_vec) {
  const size_t per_wg = (size_t)256 * kUnroll;
  for (size_t base = (size_t)blockIdx.x * per_wg; base < n_vec; base += (size_t)gridDim.x * per_wg) {
    u32x4 v[kUnroll];
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const size_t idx = base + (size_t)i * 256 + threadIdx.x;
      const u32x4 zero = {0u, 0u, 0u, 0u};
      v[i] = idx < n_vec ? __builtin_nontemporal_load(src + idx) : zero;
    }
#pragma unroll
    for (int i = 0; i < kUnroll; ++i) {
      const size_t idx = base + (size_t)i * 256 + threadIdx.x;
      if (idx < n_vec) __builtin_nontemporal_store(v[i], dst + idx);
    }
  }
}

}  // namespace

hipError_t launch_stream_copy(const void* src, void* dst, size_t bytes, int workgroups,
                              hipStream_t stream) {
  const size_t n_vec = bytes / 16;
  return launch(stream_copy, dim3(workgroups), dim3(256), 0, stream,
                static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), n_vec);
}

hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, int workgroups,
                              hipStream_t stream) {
  const size_t n_vec = bytes / 16;
  return launch(stream_read, dim3(workgroups), dim3(256), 0, stream,
                static_cast<const u32x4*>(src), n_vec, static_cast<uint32_t*>(sink));
}

}  // namespace tempo
