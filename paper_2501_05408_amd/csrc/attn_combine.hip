// Split combine as a kernel of its own: the second pass of split-KV decode
// attention when the partial kernel was launched without the fused tail.
// One workgroup of 256 threads per (sequence, query head).
#include "attn_combine.h"

namespace tempo {
namespace {

template <int D, bool kBf16>
__global__ __launch_bounds__(256) void attn_combine(AttnParams p) {
  extern __shared__ float smem[];
  const int hq = blockIdx.x, b = blockIdx.y;
  int t_b = p.t_per_seq ? p.t_per_seq[b] : p.t;
  t_b = t_b > p.t ? p.t : (t_b < 0 ? 0 : t_b);
  const SeqRange rg = seq_range(t_b, p.window, p.tps_log2);
  const int n = rg.nchunks < p.num_splits ? rg.nchunks : p.num_splits;
  const int64_t row = (int64_t)b * p.Hq + hq;
  const int esz = kBf16 ? 2 : 4;
  combine_heads<D, kBf16>(p.ws_ml + row * p.num_splits * 2, p.ws_acc + row * p.num_splits * D,
                                 p.num_splits, n, 1, static_cast<char*>(p.out) + row * D * esz, smem);
}

}  // namespace

hipError_t launch_combine(const AttnParams& p, int batch, int D, int dtype, hipStream_t stream) {
  const dim3 grid(p.Hq, batch);
  const dim3 block(256);
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
