// Anti-causal window reduction (Section 3, Algorithm 1): the return of step t is the
// discounted sum of the rewards of the steps t .. min(t+n, T)-1, or of the whole future
// t .. T-1,
//     g[b][t] = sum_{k=0}^{m-1} gamma^k r[b][t+k],   m = min(n, T-t)  (n = 0: m = T-t).
// Like step t's attention over keys 0..t, it is a reduction over a range of the temporal
// dimension whose extent depends on t; here the range lies in the future and the
// reduction is a plain weighted sum, so no running maximum is needed.  fp32 in and out.
//
// Two kernels.
//   discounted_window   1 <= n <= 1024: one workgroup per tile of 256 steps of one sequence
//                       stages the tile and its n-step halo in LDS (zeros beyond T, which
//                       clip the slice) and every thread folds its window from the far end,
//                       g = r[t+k] + gamma * g.
//   discounted_suffix   the whole future: the recurrence g[t] = r[t] + gamma g[t+1] as a
//                       reverse scan, one workgroup per sequence.  A lane folds 4 consecutive
//                       steps; lanes are combined with the pairs (a, s) -> s + a * s', a * a'
//                       (a = gamma^4 to the number of lanes covered) in six shuffle steps,
//                       wavefronts through LDS, tiles of 1024 steps from the last to the first
//                       with a carried value.  O(T) work in one launch, whatever T is.
// The work is a few hundred KB at the paper's sizes (batch 64, T = 200 .. 1000): both kernels
// are bound by launch latency, not by any pipe.
#include "tempo_internal.h"

namespace tempo {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxWindow = 1024;

__global__ __launch_bounds__(kThreads) void discounted_window(const float* __restrict__ r, float* __restrict__ g, int T,
                                                              int n, float gamma) {
  __shared__ float tile[kThreads + kMaxWindow];
  const int b = blockIdx.y, t0 = blockIdx.x * kThreads, tid = threadIdx.x;
  const float* rb = r + (int64_t)b * T;
  for (int i = tid; i < kThreads + n - 1; i += kThreads) tile[i] = (t0 + i < T) ? rb[t0 + i] : 0.f;
  __syncthreads();
  if (t0 + tid >= T) return;
  float acc = 0.f;
  for (int k = n - 1; k >= 0; --k) acc = fmaf(acc, gamma, tile[tid + k]);  // steps beyond T hold 0: the slice is clipped
  g[(int64_t)b * T + t0 + tid] = acc;
}

constexpr int kChunk = 4;                       // steps per lane
constexpr int kTile = kThreads * kChunk;        // steps per trip of a workgroup

__global__ __launch_bounds__(kThreads) void discounted_suffix(const float* __restrict__ r, float* __restrict__ g, int T,
                                                              float gamma) {
  __shared__ float wave_sum[kThreads / 64], wave_pow[kThreads / 64], carried;
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float* rb = r + (int64_t)b * T;
  float* gb = g + (int64_t)b * T;
  const float g2 = gamma * gamma, A = g2 * g2;  // gamma^kChunk
  float carry = 0.f;                            // g at the first step after the current tile (0 beyond T)
  for (int first = ((T - 1) / kTile) * kTile; first >= 0; first -= kTile) {
    const int t0 = first + tid * kChunk;
    float x[kChunk];
#pragma unroll
    for (int c = 0; c < kChunk; ++c) x[c] = (t0 + c < T) ? rb[t0 + c] : 0.f;
    // this lane's steps folded from the far end, then all lanes behind it in the wavefront
    float s = x[kChunk - 1];
#pragma unroll
    for (int c = kChunk - 2; c >= 0; --c) s = fmaf(s, gamma, x[c]);
    float a = A;
#pragma unroll
    for (int d = 1; d < 64; d *= 2) {
      const float s2 = __shfl_down(s, d), a2 = __shfl_down(a, d);
      if (lane + d < 64) {
        s = fmaf(a, s2, s);
        a *= a2;
      }
    }
    if (lane == 0) {
      wave_sum[wave] = s;  // the wavefront's 256 steps folded; a = gamma^256 here
      wave_pow[wave] = a;
    }
    __syncthreads();
    // g at the first step after this wavefront's steps: the later wavefronts folded onto the carry
    float after = carry;
    for (int w = kThreads / 64 - 1; w > wave; --w) after = fmaf(wave_pow[w], after, wave_sum[w]);
    // ... and after this lane's steps
    const float s_next = __shfl_down(s, 1), a_next = __shfl_down(a, 1);
    float acc = lane == 63 ? after : fmaf(a_next, after, s_next);
    float out[kChunk];
#pragma unroll
    for (int c = kChunk - 1; c >= 0; --c) {
      acc = fmaf(acc, gamma, x[c]);
      out[c] = acc;
    }
#pragma unroll
    for (int c = 0; c < kChunk; ++c) {
      if (t0 + c < T) gb[t0 + c] = out[c];
    }
    if (tid == 0) carried = out[0];  // g at the tile's first step: what the tile before it continues from
    __syncthreads();
    carry = carried;
  }
}

}  // namespace

hipError_t launch_discounted_sum(const float* r, float* g, int batch, int T, int n, float gamma, hipStream_t stream) {
  if (n == 0 || n >= T)
    return launch(discounted_suffix, dim3(batch), dim3(kThreads), 0, stream, r, g, T, gamma);
  if (n > kMaxWindow) return hipErrorInvalidValue;
  return launch(discounted_window, dim3((T + kThreads - 1) / kThreads, batch), dim3(kThreads), 0, stream, r, g, T, n,
                gamma);
}

int discounted_sum_max_window() { return kMaxWindow; }

}  // namespace tempo
