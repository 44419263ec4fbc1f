// Split combine of query-head rows (the body of the combine kernel).
//
// Section 4.3 obtains the attention output by summing the masked per-tile terms.
// With per-split partials (m_s, l_s, acc_s) in base-2 units this is
//     M   = max_s m_s
//     out = sum_s 2^(m_s - M) acc_s  /  sum_s 2^(m_s - M) l_s
// Only splits that exist for the sequence are read, so no empty partial is ever
// touched.  The order of the sums depends only on the workgroup size, so the
// result is deterministic.
#pragma once

#include "tempo_internal.h"

namespace tempo {

// Floats of LDS combine_heads needs for a workgroup of `threads` threads.
__host__ __device__ inline int combine_lds_floats(int threads, int /*D*/) { return threads * 6; }

// Combine the n splits of G consecutive query-head rows.  All threads of the
// workgroup call this with the same arguments.
//   ml  [G][S][2]  (m_s, l_s);  acc [G][S][D];  out [G][D];  S = split stride.
// A thread owns one float4 column of one head in one of R split lanes; it reads
// its splits in batches of 8 independent loads (one memory round trip per batch,
// which is what the cost of this routine is made of), folds each batch into a
// running (max, sum, accumulator), and the R lanes are merged through LDS.
template <int D, bool kBf16>
__device__ inline void combine_heads(const float* ml, const float* acc, int S, int n, int G,
                                     void* out, float* smem) {
  constexpr int C4 = D / 4;
  constexpr int U = 8;
  const int threads = blockDim.x, tid = threadIdx.x;
  int GB = threads / C4 / 2;  // heads per pass: at least two split lanes when possible
  GB = GB < 1 ? 1 : (GB > G ? G : GB);
  const int cols = GB * C4;
  const int R = threads / cols;
  const int r = tid / cols, col = tid % cols, hg = col / C4, c4 = col % C4;
  for (int g0 = 0; g0 < G; g0 += GB) {
    const int g = g0 + hg;
    float mr = -INFINITY, lr = 0.f;
    float4 ar = {0.f, 0.f, 0.f, 0.f};
    if (r < R && g < G) {
      const float* mlr = ml + (int64_t)g * S * 2;
      const float* accr = acc + (int64_t)g * S * D + 4 * c4;
      for (int s0 = r; s0 < n; s0 += R * U) {
        float m[U], l[U];
        float4 a[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int s = s0 + u * R;
          const int ss = s < n ? s : s0;  // a valid split; its weight is forced to 0 below
          m[u] = mlr[2 * ss];
          l[u] = mlr[2 * ss + 1];
          a[u] = *reinterpret_cast<const float4*>(accr + (int64_t)ss * D);
          if (s >= n) m[u] = -INFINITY;
        }
        float mb = mr;
#pragma unroll
        for (int u = 0; u < U; ++u) mb = fmaxf(mb, m[u]);
        // With a block of queries a split may hold no key of this row (m = -inf,
        // l = acc = 0); while nothing finite has been seen, weigh against 0.
        const float ref = mb == -INFINITY ? 0.f : mb;
        const float keep = exp2f(mr - ref);  // first batch: exp2f(-inf) = 0
        lr *= keep;
        ar.x *= keep; ar.y *= keep; ar.z *= keep; ar.w *= keep;
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const float w = exp2f(m[u] - ref);
          lr = fmaf(w, l[u], lr);
          ar.x = fmaf(w, a[u].x, ar.x); ar.y = fmaf(w, a[u].y, ar.y);
          ar.z = fmaf(w, a[u].z, ar.z); ar.w = fmaf(w, a[u].w, ar.w);
        }
        mr = mb;
      }
    }
    if (r < R) {
      float* slot = smem + (r * cols + col) * 6;
      slot[0] = mr; slot[1] = lr; slot[2] = ar.x; slot[3] = ar.y; slot[4] = ar.z; slot[5] = ar.w;
    }
    __syncthreads();
    if (r == 0 && g < G) {
      float M = mr;
      for (int i = 1; i < R; ++i) M = fmaxf(M, smem[(i * cols + col) * 6]);
      float L = 0.f;
      float4 A = {0.f, 0.f, 0.f, 0.f};
      for (int i = 0; i < R; ++i) {
        const float* slot = smem + (i * cols + col) * 6;
        if (slot[0] == -INFINITY) continue;  // a lane that had no split
        const float w = exp2f(slot[0] - M);
        L = fmaf(w, slot[1], L);
        A.x = fmaf(w, slot[2], A.x); A.y = fmaf(w, slot[3], A.y);
        A.z = fmaf(w, slot[4], A.z); A.w = fmaf(w, slot[5], A.w);
      }
      const float inv = 1.0f / L;
      if (kBf16) {
        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
        bf16x4 o;
        o[0] = (__bf16)(A.x * inv); o[1] = (__bf16)(A.y * inv);
        o[2] = (__bf16)(A.z * inv); o[3] = (__bf16)(A.w * inv);
        *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(out) + (int64_t)g * D + 4 * c4) = o;
      } else {
        const float4 o = {A.x * inv, A.y * inv, A.z * inv, A.w * inv};
        *reinterpret_cast<float4*>(static_cast<float*>(out) + (int64_t)g * D + 4 * c4) = o;
      }
    }
    __syncthreads();  // smem is reused by the next pass
  }
}

}  // namespace tempo
