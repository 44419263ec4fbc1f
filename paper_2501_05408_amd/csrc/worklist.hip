// Work list of a ragged decode step: the non-empty (sequence, split) items of a batch
// whose sequences are at different steps, longest first.
//
// Static tiling (Section 4.3) turns a dynamic range into a dynamic NUMBER of static
// tiles; with per-sequence steps that number differs per sequence, and a dense grid over
// (sequence, largest split count) launches many workgroups that find nothing to do, in
// an order that leaves the shortest items of the long sequences for last.  The list
// names only the items that exist: first every full split of every sequence, then the
// newest split of every sequence (the one the step cuts short) in eight size classes,
// largest class first, so that what remains for the launch's tail are its smallest items.
// It depends on the steps only: one list serves every layer of a decode step.
#include "tempo_internal.h"

namespace tempo {
namespace {

constexpr int kThreads = 256;
constexpr int kClasses = 8;

// Splits of sequence b and the size class of its newest split (0 = longest).
__device__ inline void seq_items(const int32_t* t_per_seq, int b, int t_max, int window, int tps_log2,
                                 int num_splits, int& n, int& size_class) {
  int t_b = t_per_seq[b];
  t_b = t_b > t_max ? t_max : (t_b < 0 ? 0 : t_b);
  const SeqRange rg = seq_range(t_b, window, tps_log2);
  n = rg.nchunks < num_splits ? rg.nchunks : num_splits;
  const int first = (rg.chunk0 + rg.nchunks - 1) << tps_log2;          // first key of the newest split
  const int len = rg.hi - (rg.lo > first ? rg.lo : first) + 1;        // 1 .. tokens per split
  size_class = (kClasses - 1) - (int)(((int64_t)(len - 1) * kClasses) >> tps_log2);
}

// One workgroup.  Thread i owns sequences i, i + 256, ...; its items of each kind are
// contiguous in the list, at the offset an exclusive scan over the threads gives.
__global__ __launch_bounds__(kThreads) void worklist_build(const int32_t* __restrict__ t_per_seq, int batch, int t_max,
                                                           int window, int tps_log2, int num_splits,
                                                           int32_t* __restrict__ list) {
  __shared__ int counts[kClasses + 1][kThreads];   // [0]: full splits; [1 + c]: newest splits of class c
  __shared__ int bases[kClasses + 1];
  const int tid = threadIdx.x;
  int mine[kClasses + 1];
#pragma unroll
  for (int k = 0; k <= kClasses; ++k) mine[k] = 0;
  for (int b = tid; b < batch; b += kThreads) {
    int n, c;
    seq_items(t_per_seq, b, t_max, window, tps_log2, num_splits, n, c);
    mine[0] += n - 1;
#pragma unroll
    for (int k = 0; k < kClasses; ++k) mine[1 + k] += (k == c) ? 1 : 0;
  }
#pragma unroll
  for (int k = 0; k <= kClasses; ++k) counts[k][tid] = mine[k];
  __syncthreads();
  if (tid <= kClasses) {   // one thread per kind turns its row of counts into exclusive offsets
    int run = 0;
    for (int i = 0; i < kThreads; ++i) {
      const int c = counts[tid][i];
      counts[tid][i] = run;
      run += c;
    }
    bases[tid] = run;      // total of this kind, for now
  }
  __syncthreads();
  if (tid == 0) {
    int run = 0;
    for (int k = 0; k <= kClasses; ++k) {
      const int total = bases[k];
      bases[k] = run;
      run += total;
    }
    list[0] = run;
  }
  __syncthreads();
  int at[kClasses + 1];
#pragma unroll
  for (int k = 0; k <= kClasses; ++k) at[k] = 1 + bases[k] + counts[k][tid];
  for (int b = tid; b < batch; b += kThreads) {
    int n, c;
    seq_items(t_per_seq, b, t_max, window, tps_log2, num_splits, n, c);
    for (int s = 0; s + 1 < n; ++s) list[at[0]++] = (int32_t)((uint32_t)b | ((uint32_t)s << 16));
#pragma unroll
    for (int k = 0; k < kClasses; ++k) {
      if (k == c) list[at[1 + k]++] = (int32_t)((uint32_t)b | ((uint32_t)(n - 1) << 16));
    }
  }
}

}  // namespace

hipError_t launch_worklist_build(const int32_t* t_per_seq, int batch, int t_max, int window, int tps_log2,
                                 int num_splits, int32_t* worklist, hipStream_t stream) {
  return launch(worklist_build, dim3(1), dim3(kThreads), 0, stream, t_per_seq, batch, t_max, window, tps_log2,
                num_splits, worklist);
}

}  // namespace tempo
