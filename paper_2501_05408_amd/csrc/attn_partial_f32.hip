// Partial attention of one split, fp32 keys/values (row-major block store),
// plain vector arithmetic with wavefront reductions.
//
// Same quantities as the bf16 kernel (Section 2, Eq. 1 over one split; Section
// 4.3 masks): running max m, running sum l and accumulator acc in fp32, base-2
// units.  One workgroup = one (sequence, QUERY head, split): the fp32 path is the
// small-shape, tight-tolerance path, so it keeps every product in fp32 and does
// not share key/value reads across the query group.  With a block of C query
// steps the grid's first axis runs over (step, query head) and each workgroup
// masks by its own step's range inside the split.
//
// A wavefront looks at 4 key positions at a time: 16 lanes per position, each
// lane holding D/16 consecutive dims.  The dot product is a 16-lane butterfly
// (DPP row operations); each 16-lane row keeps its own (m, l, acc) and the rows
// and wavefronts are merged once, through LDS, at the end.
#include "tempo_internal.h"

namespace tempo {
namespace {

template <int D>
__global__ __launch_bounds__(512) void attn_partial_f32(AttnParams p) {
  constexpr int E = D / 16;  // dims per lane
  extern __shared__ float smem[];
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;
  const int cq = blockIdx.x / p.Hq, hq = blockIdx.x - cq * p.Hq, b = blockIdx.y;  // cq < p.queries
  const int hkv = hq / p.G;
  int t_b = p.t_per_seq ? p.t_per_seq[b] : p.t;
  t_b = t_b > p.t ? p.t : (t_b < 0 ? 0 : t_b);
  const SeqRange rg = seq_range(t_b, p.window, p.tps_log2, p.queries, p.pad_t);
  if ((int)blockIdx.z >= rg.nchunks) return;
  const int split = rg.nchunks - 1 - (int)blockIdx.z;  // newest split first, as in the bf16 kernel
  const int chunk = rg.chunk0 + split;
  const int cs = chunk << p.tps_log2, ce = ((chunk + 1) << p.tps_log2) - 1;
  // this query step's own range, cut to the split (empty if they do not meet)
  const int t_q = t_b + cq;
  const int lo_q = (p.window > 0 && t_q - p.window + 1 > 0) ? t_q - p.window + 1 : 0;
  const int start = lo_q > cs ? lo_q : cs;
  const int end = t_q < ce ? t_q : ce;

  const int row = lane >> 4, col = lane & 15;
  const int Z = 1 << p.z_log2;
  float* kpool = static_cast<float*>(p.k_pool);
  float* vpool = static_cast<float*>(p.v_pool);
  // Fused block-store write (Section 6, "in-place writes"): step t's own key/value
  // are taken from k_new / v_new, and the first query head of the group also stores
  // them into the pool for later steps.
  const float* kn = p.k_new ? static_cast<const float*>(p.k_new) + ((int64_t)b * p.Hkv + hkv) * D : nullptr;
  const float* vn = p.k_new ? static_cast<const float*>(p.v_new) + ((int64_t)b * p.Hkv + hkv) * D : nullptr;

  float qv[E];
  {
    const float* qp = static_cast<const float*>(p.q) + (((int64_t)b * p.io_steps + cq) * p.Hq + hq) * D + col * E;
#pragma unroll
    for (int e = 0; e < E; ++e) qv[e] = qp[e];
  }
  // Rotary embedding: dims col*E .. +E-1 pair with those of lane col ^ 8 of the same
  // 16-lane row; table entry (position, i) with i = (col & 7) * E + e.
  if (p.rope_cos) {
    const float* cs = p.rope_cos + (int64_t)t_q * (D / 2) + (col & 7) * E;
    const float* sn = p.rope_sin + (int64_t)t_q * (D / 2) + (col & 7) * E;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const float other = __shfl_xor(qv[e], 8);
      qv[e] = col < 8 ? rope_lo(qv[e], other, cs[e], sn[e]) : rope_hi(other, qv[e], cs[e], sn[e]);
    }
  }
  float m = -INFINITY, l = 0.f, acc[E];
#pragma unroll
  for (int e = 0; e < E; ++e) acc[e] = 0.f;

  // Rows of a wavefront may leave this loop at different trips; the butterfly
  // below only exchanges data inside one 16-lane row, whose lanes share j.
  for (int j = start + 4 * wave + row; j <= end; j += 4 * nwaves) {
    const int tile = j >> p.z_log2, slot = j & (Z - 1);
    const int phys = clamp_block(p.block_table[(int64_t)b * p.max_blocks_per_seq + (tile & p.tile_mask)], p.num_blocks);
    const int64_t off = ((int64_t)phys * p.Hkv + hkv) * Z * D + (int64_t)slot * D + col * E;
    const bool fresh = kn != nullptr && j == t_b;  // uniform over the 16-lane row
    const float* ksrc = fresh ? kn + col * E : kpool + off;
    const float* vsrc = fresh ? vn + col * E : vpool + off;
    float kx[E], vx[E];
#pragma unroll
    for (int e = 0; e < E; e += 4) {
      const float4 k4 = *reinterpret_cast<const float4*>(ksrc + e);
      const float4 v4 = *reinterpret_cast<const float4*>(vsrc + e);
      kx[e] = k4.x; kx[e + 1] = k4.y; kx[e + 2] = k4.z; kx[e + 3] = k4.w;
      vx[e] = v4.x; vx[e + 1] = v4.y; vx[e + 2] = v4.z; vx[e + 3] = v4.w;
    }
    if (fresh) {  // all 16 lanes of the row take this branch together
      if (p.rope_cos) {  // the new key arrives unrotated: turn it to position t_b
        const float* cs = p.rope_cos + (int64_t)t_b * (D / 2) + (col & 7) * E;
        const float* sn = p.rope_sin + (int64_t)t_b * (D / 2) + (col & 7) * E;
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const float other = __shfl_xor(kx[e], 8);
          kx[e] = col < 8 ? rope_lo(kx[e], other, cs[e], sn[e]) : rope_hi(other, kx[e], cs[e], sn[e]);
        }
      }
      if (hq == hkv * p.G) {
#pragma unroll
        for (int e = 0; e < E; e += 4) {
          *reinterpret_cast<float4*>(kpool + off + e) = float4{kx[e], kx[e + 1], kx[e + 2], kx[e + 3]};
          *reinterpret_cast<float4*>(vpool + off + e) = float4{vx[e], vx[e + 1], vx[e + 2], vx[e + 3]};
        }
      }
    }
    float dot = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) dot = fmaf(qv[e], kx[e], dot);
    // 16-lane butterfly: every lane of the row ends with the full dot product
    dot += __shfl_xor(dot, 8);
    dot += __shfl_xor(dot, 4);
    dot += __shfl_xor(dot, 2);
    dot += __shfl_xor(dot, 1);
    const float x = dot * p.scale_log2e;
    const float m_new = fmaxf(m, x);
    const float alpha = exp2f(m - m_new);  // exp2f(-inf) = 0 on the first key
    const float w = exp2f(x - m_new);
    l = l * alpha + w;
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = fmaf(w, vx[e], acc[e] * alpha);
    m = m_new;
  }

  // rows x wavefronts -> LDS, then one merge
  const int nrows = nwaves * 4;
  float* sm_m = smem;                 // [nrows]
  float* sm_l = smem + nrows;         // [nrows]
  float* sm_acc = smem + 2 * nrows;   // [nrows][D]
  const int r = wave * 4 + row;
  if (col == 0) { sm_m[r] = m; sm_l[r] = l; }
#pragma unroll
  for (int e = 0; e < E; ++e) sm_acc[r * D + col * E + e] = acc[e];
  __syncthreads();

  for (int d = threadIdx.x; d < D; d += blockDim.x) {
    float M = -INFINITY;
    for (int i = 0; i < nrows; ++i) M = fmaxf(M, sm_m[i]);
    float num = 0.f, den = 0.f;
    for (int i = 0; i < nrows; ++i) {
      const float mi = sm_m[i];
      if (mi == -INFINITY) continue;  // a row that saw no key (all rows: the partial is (-inf, 0, 0))
      const float wgt = exp2f(mi - M);
      num += wgt * sm_acc[i * D + d];
      den += wgt * sm_l[i];
    }
    const int64_t qrow = ((int64_t)b * p.queries + cq) * p.Hq + hq;
    if (p.direct) {
      const int64_t orow = ((int64_t)b * p.io_steps + cq) * p.Hq + hq;
      static_cast<float*>(p.out)[orow * D + d] = num / den;
    } else {
      const int64_t part = qrow * p.num_splits + split;
      p.ws_acc[part * D + d] = num;
      if (d == 0) {
        p.ws_ml[part * 2] = M;
        p.ws_ml[part * 2 + 1] = den;
      }
    }
  }
}

}  // namespace

hipError_t launch_partial_f32(const AttnParams& p, int batch, int D, int grid_splits, int waves,
                              hipStream_t stream) {
  const dim3 grid(p.Hq * p.queries, batch, grid_splits);
  const dim3 block(64 * waves);
  const size_t lds = (size_t)waves * 4 * (2 + (size_t)D) * sizeof(float);
  if (D == 128) return launch(attn_partial_f32<128>, grid, block, lds, stream, p);
  else return launch(attn_partial_f32<64>, grid, block, lds, stream, p);
}

}  // namespace tempo
