// Internal declarations shared by the translation units of libtempo.
// Nothing here crosses the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tempo.h"

namespace tempo {

// ---- block-store layout ----------------------------------------------------
// Offsets are in elements, inside the tile of one (block, kv head) pair, which
// holds block_size * head_dim elements.

// f32: row-major [slot][d].
__host__ __device__ inline int64_t tile_off_f32(int D, int slot, int d) {
  return (int64_t)slot * D + d;
}

// bf16 keys.  Groups of 32 slots; a group is 2 row-tiles (slots 0..15, 16..31)
// x D/32 contraction steps, each a 1 KiB unit of 64 lanes x 8 elements: lane
// (row + 16*c) holds dims 32*s + 8*c .. +7 of slot `row` of the tile.  That is
// the A-operand image of a 16x16x32 MFMA (rows = slots, contraction = dims).
__host__ __device__ inline int64_t tile_off_k_bf16(int D, int slot, int d) {
  const int grp = slot >> 5, u = slot & 31, tile = u >> 4, row = u & 15;
  const int s = d >> 5, c = (d & 31) >> 3, e = d & 7;
  return (int64_t)grp * 32 * D + (int64_t)(((tile * (D >> 5) + s) * 64) + c * 16 + row) * 8 + e;
}

// bf16 values.  Same groups of 32 slots; a group is D/16 column-tiles, each a
// 1 KiB unit: lane (n + 16*c) holds dim 16*dt + n of the 8 slots
// {4c..4c+3, 16+4c..16+4c+3}.  That is the B-operand image of a 16x16x32 MFMA
// (contraction = slots, columns = dims) whose contraction order matches the
// accumulator image of the two key row-tiles above.
__host__ __device__ inline int64_t tile_off_v_bf16(int D, int slot, int d) {
  const int grp = slot >> 5, u = slot & 31, half = u >> 4, uu = u & 15;
  const int c = uu >> 2, e = (uu & 3) + 4 * half;
  const int dt = d >> 4, n = d & 15;
  return (int64_t)grp * 32 * D + (int64_t)((dt * 64) + c * 16 + n) * 8 + e;
}

__host__ __device__ inline int clamp_block(int phys, int num_blocks) {
  return phys < 0 ? 0 : (phys >= num_blocks ? num_blocks - 1 : phys);
}

// ---- rotary embedding of one (i, i + D/2) pair ---------------------------------
// Every kernel that rotates uses these two expressions, so the fused and the
// separate launches store the same bits: one product, then one fused multiply-add.
__device__ inline float rope_lo(float lo, float hi, float c, float s) { return fmaf(-hi, s, lo * c); }
__device__ inline float rope_hi(float lo, float hi, float c, float s) { return fmaf(lo, s, hi * c); }

// ---- kernel parameter blocks -------------------------------------------------
struct StoreParams {
  void* k_pool;
  void* v_pool;
  const int32_t* block_table;
  const int32_t* t_per_seq;  // may be null
  int32_t t;                 // uniform step / upper bound
  int32_t z_log2;
  int32_t max_blocks_per_seq;
  int32_t tile_mask;         // ring_blocks-1 for a ring store, INT32_MAX otherwise: table column = tile & mask
  int32_t num_blocks;
  int32_t Hkv;
  int32_t batch;
  int32_t count;             // append: consecutive steps per sequence, rows [B][count][Hkv][D]
  int32_t src_steps;         // steps per sequence in the caller's k_new / v_new (>= count; == count normally)
  const int32_t* count_per_seq;  // may be null; sequence b writes only its first count_per_seq[b] rows of the call
  int32_t row0;              // index, on the call's step axis, of this launch's first row (for that test)
  const float* rope_cos;     // bf16 append: non-null = keys arrive unrotated and are turned to their step's
  const float* rope_sin;     //   position on the way into the store ([positions][D/2] tables)
};

struct AttnParams {
  void* k_pool;              // written only when k_new is set
  void* v_pool;
  const int32_t* block_table;
  const void* q;
  const void* k_new;         // [B][Hkv][D]; non-null: append step t inside the attention kernel (queries == 1)
  const void* v_new;
  const int32_t* t_per_seq;  // may be null
  const int32_t* count_per_seq;  // prompt kernel: may be null; sequence b answers only its first count_per_seq[b] steps
  const float* rope_cos;     // [positions][D/2]; non-null: q (and k_new) arrive unrotated and are
  const float* rope_sin;     //   rotated to their step's position inside the kernel
  const int32_t* worklist;   // bf16 decode kernel: may be null; [0] = number of items, then one item per
                             //   workgroup row: sequence in the low 16 bits, split in the high 16
  float* ws_ml;              // [B][C][Hq][S][2]  (running max in log2 units, running sum)
  float* ws_acc;             // [B][C][Hq][S][D]
  void* out;                 // [B][C][Hq][D]
  int32_t t;                 // uniform step / upper bound
  int32_t window;            // 0 = causal
  int32_t z_log2;
  int32_t max_blocks_per_seq;
  int32_t tile_mask;         // as in StoreParams
  int32_t num_blocks;
  int32_t Hkv;
  int32_t Hq;
  int32_t G;                 // Hq / Hkv
  int32_t tps_log2;          // log2(tokens per split)
  int32_t num_splits;        // S: stride of the split axis in the workspace
  int32_t queries;           // C: consecutive query steps per sequence (q, out, workspace rows are [B][C][Hq])
  int32_t io_steps;          // steps per sequence in the caller's q / out ([B][io_steps][Hq][D]); the block is
                             //   `queries` consecutive ones of them (pointers pre-offset); == queries normally
  int32_t pad_t;             // padded baseline: keys up to pad_t are read and masked; 0 = none
  int32_t direct;            // 1: single split, write `out` and skip the combine
  float scale_log2e;         // s * log2(e)
};

// Visible range and split bookkeeping of one sequence, identical on host and device.
// With a block of C queries (steps t_b .. t_b+C-1) the range is the union of the
// queries' ranges: from the first query's lo to the last query's step.  The padded
// baseline reads on to key pad_t (masked beyond each query's own step).
struct SeqRange {
  int lo, hi, chunk0, nchunks;
};
__host__ __device__ inline SeqRange seq_range(int t_b, int window, int tps_log2, int queries = 1,
                                              int pad_t = 0) {
  SeqRange r;
  r.hi = t_b + queries - 1;
  r.hi = r.hi > pad_t ? r.hi : pad_t;
  r.lo = (window > 0 && t_b - window + 1 > 0) ? t_b - window + 1 : 0;
  r.chunk0 = r.lo >> tps_log2;
  r.nchunks = (r.hi >> tps_log2) - r.chunk0 + 1;
  return r;
}

// Launch and return the launch's own status.  hipGetLastError() is not used: it
// reports the last error of any HIP call on the thread, including benign ones
// left behind by the caller's framework (an event query that was "not ready").
template <typename... Params>
inline hipError_t launch_converted(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds,
                                   hipStream_t stream, Params... vals) {
  void* argv[] = {(void*)&vals...};
  return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, argv, lds, stream);
}
template <typename... Params, typename... Args>
inline hipError_t launch(void (*kernel)(Params...), dim3 grid, dim3 block, size_t lds,
                         hipStream_t stream, Args... args) {
  static_assert(sizeof...(Params) == sizeof...(Args), "kernel argument count");
  return launch_converted<Params...>(kernel, grid, block, lds, stream, static_cast<Params>(args)...);
}

// ---- launchers (defined next to their kernels) -------------------------------
hipError_t launch_append(const StoreParams& p, const void* k_new, const void* v_new, int D,
                         int dtype, hipStream_t stream);
hipError_t launch_gather(const StoreParams& p, void* k_out, void* v_out, int D, int dtype, int j0,
                         int count, hipStream_t stream);
hipError_t launch_partial_bf16(const AttnParams& p, int batch, int D, int grid_splits, int waves,
                               hipStream_t stream);
size_t partial_bf16_lds_bytes(int waves, int columns, int D);      // dynamic LDS of that launch
int prefill_bf16_block_steps(int G);                               // query steps per workgroup of the prompt kernel
hipError_t launch_prefill_bf16(const AttnParams& p, int batch, int D, int grid_splits, hipStream_t stream);
hipError_t launch_partial_f32(const AttnParams& p, int batch, int D, int grid_splits, int waves,
                              hipStream_t stream);

hipError_t launch_rope_rotate(const float* rope_cos, const float* rope_sin, const void* x, void* y,
                              int dtype, int batch, int heads, int D, int t, const int32_t* t_per_seq,
                              hipStream_t stream);
hipError_t launch_rope_append(const StoreParams& p, const float* rope_cos, const float* rope_sin,
                              const void* k_raw, const void* v_new, int D, int dtype, hipStream_t stream);
hipError_t launch_combine(const AttnParams& p, int batch, int D, int dtype, hipStream_t stream);
hipError_t launch_worklist_build(const int32_t* t_per_seq, int batch, int t_max, int window, int tps_log2,
                                 int num_splits, int32_t* worklist, hipStream_t stream);
hipError_t launch_discounted_sum(const float* r, float* g, int batch, int T, int n, float gamma, hipStream_t stream);
int discounted_sum_max_window();
hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, int workgroups,
                              hipStream_t stream);
hipError_t launch_stream_copy(const void* src, void* dst, size_t bytes, int workgroups,
                              hipStream_t stream);

}  // namespace tempo
