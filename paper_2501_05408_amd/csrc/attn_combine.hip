// Split combine: the second pass of split-KV decode attention.
//
// Section 4.3 obtains the attention output by summing the masked per-tile terms.
// With per-split partials (m_s, l_s, acc_s) in base-2 units this is
//     M   = max_s m_s
//     out = sum_s 2^(m_s - M) acc_s  /  sum_s 2^(m_s - M) l_s
// Only the splits that exist for the sequence are read (the partial kernel writes
// nothing for the others), so no empty partial is ever touched.
//
// One workgroup of 256 threads per (sequence, query head).  A thread owns one
// float4 of the head dimension in one of R = 256 / (D/4) split lanes; the R lanes
// stride over the splits and are merged through LDS.  The order of the sums is
// fixed, so the result is deterministic.
#include "tempo_internal.h"

namespace tempo {
namespace {

template <int D, bool kBf16>
__global__ __launch_bounds__(256) void attn_combine(AttnParams p) {
  constexpr int C4 = D / 4;       // float4 columns per row
  constexpr int R = 256 / C4;     // split lanes
  __shared__ float red[256];
  __shared__ float4 racc[R][C4];
  __shared__ float rl[R];
  const int hq = blockIdx.x, b = blockIdx.y;
  int t_b = p.t_per_seq ? p.t_per_seq[b] : p.t;
  t_b = t_b > p.t ? p.t : (t_b < 0 ? 0 : t_b);
  const SeqRange rg = seq_range(t_b, p.window, p.tps_log2);
  const int n = rg.nchunks < p.num_splits ? rg.nchunks : p.num_splits;
  const int64_t row = (int64_t)b * p.Hq + hq;
  const float* ml = p.ws_ml + row * p.num_splits * 2;
  const float* acc = p.ws_acc + row * p.num_splits * D;

  // global max over the sequence's splits
  float M = -INFINITY;
  for (int s = threadIdx.x; s < n; s += 256) M = fmaxf(M, ml[2 * s]);
  red[threadIdx.x] = M;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if (threadIdx.x < w) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + w]);
    __syncthreads();
  }
  M = red[0];

  const int r = threadIdx.x / C4, c4 = threadIdx.x % C4;
  float4 a = {0.f, 0.f, 0.f, 0.f};
  float l = 0.f;
  for (int s = r; s < n; s += R) {
    const float w = exp2f(ml[2 * s] - M);
    const float4 v = *reinterpret_cast<const float4*>(acc + (int64_t)s * D + 4 * c4);
    a.x = fmaf(w, v.x, a.x); a.y = fmaf(w, v.y, a.y); a.z = fmaf(w, v.z, a.z); a.w = fmaf(w, v.w, a.w);
    l = fmaf(w, ml[2 * s + 1], l);
  }
  racc[r][c4] = a;
  if (c4 == 0) rl[r] = l;
  __syncthreads();
  if (r == 0) {
    for (int i = 1; i < R; ++i) {
      const float4 v = racc[i][c4];
      a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
      l += rl[i];
    }
    const float inv = 1.0f / l;
    if (kBf16) {
      typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
      bf16x4 o;
      o[0] = (__bf16)(a.x * inv); o[1] = (__bf16)(a.y * inv);
      o[2] = (__bf16)(a.z * inv); o[3] = (__bf16)(a.w * inv);
      *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.out) + row * D + 4 * c4) = o;
    } else {
      float4 o = {a.x * inv, a.y * inv, a.z * inv, a.w * inv};
      *reinterpret_cast<float4*>(static_cast<float*>(p.out) + row * D + 4 * c4) = o;
    }
  }
}

}  // namespace

hipError_t launch_combine(const AttnParams& p, int batch, int D, int dtype, hipStream_t stream) {
  const dim3 grid(p.Hq, batch);
  const dim3 block(256);
  if (dtype == TEMPO_BF16) {
    if (D == 128) return launch((attn_combine<128, true>), grid, block, 0, stream, p);
    else return launch((attn_combine<64, true>), grid, block, 0, stream, p);
  } else {
    if (D == 128) return launch((attn_combine<128, false>), grid, block, 0, stream, p);
    else return launch((attn_combine<64, false>), grid, block, 0, stream, p);
  }
}

}  // namespace tempo
