// Split combine kernels: the second pass of split-KV decode attention
// (Section 4.3: the masked per-tile attention terms are summed).
//   attn_combine      one workgroup of 256 threads per (sequence, query head); split
//                     lanes merged through LDS.  Any number of splits.
//   attn_combine_few  at most 8 splits: one thread per float4 column of a row reads
//                     all of the row's splits in one batch of independent loads; no
//                     LDS, no barrier, a sixth of the workgroups.  The combine is a
//                     latency chain (launch, one memory round trip, store), so this is
//                     what the common case (1-8 long splits) uses.
#include "attn_combine.h"

namespace tempo {
namespace {

template <int D, bool kBf16>
__global__ __launch_bounds__(256) void attn_combine(AttnParams p) {
  extern __shared__ float smem[];
  const int b = blockIdx.y;  // blockIdx.x runs over the sequence's (query step, query head) rows
  int t_b = p.t_per_seq ? p.t_per_seq[b] : p.t;
  t_b = t_b > p.t ? p.t : (t_b < 0 ? 0 : t_b);
  const SeqRange rg = seq_range(t_b, p.window, p.tps_log2, p.queries, p.pad_t);
  const int n = rg.nchunks < p.num_splits ? rg.nchunks : p.num_splits;
  const int64_t row = (int64_t)b * gridDim.x + blockIdx.x;
  const int64_t orow = (int64_t)b * p.io_steps * p.Hq + blockIdx.x;  // rows of `out` may be strided per sequence
  const int esz = kBf16 ? 2 : 4;
  combine_heads<D, kBf16>(p.ws_ml + row * p.num_splits * 2, p.ws_acc + row * p.num_splits * D,
                                 p.num_splits, n, 1, static_cast<char*>(p.out) + orow * D * esz, smem);
}

template <int D, bool kBf16>
__global__ __launch_bounds__(256) void attn_combine_few(AttnParams p, int rows) {
  constexpr int C4 = D / 4;
  constexpr int U = 8;
  const int idx = blockIdx.x * 256 + threadIdx.x;
  const int row = idx / C4, c4 = idx - row * C4;
  if (row >= rows) return;
  const int b = row / (p.Hq * p.queries);
  const int64_t orow = (int64_t)b * p.io_steps * p.Hq + (row - b * (p.Hq * p.queries));
  int t_b = p.t_per_seq ? p.t_per_seq[b] : p.t;
  t_b = t_b > p.t ? p.t : (t_b < 0 ? 0 : t_b);
  const SeqRange rg = seq_range(t_b, p.window, p.tps_log2, p.queries, p.pad_t);
  const int n = rg.nchunks < p.num_splits ? rg.nchunks : p.num_splits;  // 1..8
  const float* ml = p.ws_ml + (int64_t)row * p.num_splits * 2;
  const float* acc = p.ws_acc + (int64_t)row * p.num_splits * D + 4 * c4;
  float m[U], l[U];
  float4 a[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int s = u < n ? u : 0;  // a valid split; its weight is forced to 0 below
    m[u] = ml[2 * s];
    l[u] = ml[2 * s + 1];
    a[u] = *reinterpret_cast<const float4*>(acc + (int64_t)s * D);
    if (u >= n) m[u] = -INFINITY;
  }
  // With a block of queries a split may hold no key of this row: its partial is
  // (-inf, 0, 0) and gets weight 0.  Every row sees its own key, so M is finite.
  float M = m[0];
#pragma unroll
  for (int u = 1; u < U; ++u) M = fmaxf(M, m[u]);
  float L = 0.f;
  float4 A = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const float w = exp2f(m[u] - M);
    L = fmaf(w, l[u], L);
    A.x = fmaf(w, a[u].x, A.x); A.y = fmaf(w, a[u].y, A.y);
    A.z = fmaf(w, a[u].z, A.z); A.w = fmaf(w, a[u].w, A.w);
  }
  const float inv = 1.0f / L;
  if (kBf16) {
    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
    bf16x4 o;
    o[0] = (__bf16)(A.x * inv); o[1] = (__bf16)(A.y * inv);
    o[2] = (__bf16)(A.z * inv); o[3] = (__bf16)(A.w * inv);
    *reinterpret_cast<bf16x4*>(static_cast<__bf16*>(p.out) + orow * D + 4 * c4) = o;
  } else {
    const float4 o = {A.x * inv, A.y * inv, A.z * inv, A.w * inv};
    *reinterpret_cast<float4*>(static_cast<float*>(p.out) + orow * D + 4 * c4) = o;
  }
}

}  // namespace

hipError_t launch_combine(const AttnParams& p, int batch, int D, int dtype, hipStream_t stream) {
  const dim3 block(256);
  if (p.num_splits <= 8) {
    const int rows = batch * p.queries * p.Hq;
    const dim3 few((unsigned)(((int64_t)rows * (D / 4) + 255) / 256));
    if (dtype == TEMPO_BF16) {
      if (D == 128) return launch((attn_combine_few<128, true>), few, block, 0, stream, p, rows);
      else return launch((attn_combine_few<64, true>), few, block, 0, stream, p, rows);
    } else {
      if (D == 128) return launch((attn_combine_few<128, false>), few, block, 0, stream, p, rows);
      else return launch((attn_combine_few<64, false>), few, block, 0, stream, p, rows);
    }
  }
  const dim3 grid(p.Hq * p.queries, batch);
  const size_t lds = (size_t)combine_lds_floats(256, D) * sizeof(float);
  if (dtype == TEMPO_BF16) {
    if (D == 128) return launch((attn_combine<128, true>), grid, block, lds, stream, p);
    else return launch((attn_combine<64, true>), grid, block, lds, stream, p);
  } else {
    if (D == 128) return launch((attn_combine<128, false>), grid, block, lds, stream, p);
    else return launch((attn_combine<64, false>), grid, block, lds, stream, p);
  }
}

}  // namespace tempo
