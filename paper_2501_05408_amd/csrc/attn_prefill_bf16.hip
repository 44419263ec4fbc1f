// Prompt processing: attention of many consecutive query steps over the tiled
// keys/values, bf16, MFMA on gfx950.
//
// What is computed (Section 2, Eq. 1 for every step t .. t+count-1 of a sequence,
// with the causal or window pattern; Section 4.3 index masks): exactly what the
// decode kernel computes for each of those steps, one after the other.  With many
// steps per key the products dominate the reads: this kernel is bound by the
// matrix cores and the softmax arithmetic, not by HBM.
//
// Mapping.  One workgroup = one (sequence, kv head, block of QB query steps); its
// columns are the block's (step, head) pairs, 16 per wavefront (column = c*G + g).
// Every wavefront walks ALL 32-slot groups of the block's key range, so each
// column's softmax is finished inside one wavefront: no partials, no combine, the
// output is written directly.  The key/value image of a group (16 KiB at D = 128)
// is the same for all wavefronts: the workgroup copies it once from the pool into
// LDS (it is already in MFMA operand order there, 1 KiB units) and every wavefront
// reads its operands from LDS.  Two key and two value buffers: the copies for later
// groups (global -> LDS loads issued at the top of an iteration, waited for at its
// end) overlap the arithmetic of the iteration; one barrier per group.
//
// Blocks against a long history.  The same kernel serves a block of up to 128
// columns in front of a long key range (chunked prompt processing, speculative
// decoding with many steps): the key range is then cut into splits as in the decode
// kernel, one workgroup per (sequence, kv head, split) writes a partial
// (reference, sum, accumulator) per column, and the split combine finishes.  The
// keys/values are read from HBM once per workgroup for all its columns.
//
// Workgroups of one (sequence, head) are adjacent in the work list and run together on
// one die, so the pool is streamed from HBM about once per (sequence, head) and the
// blocks that follow find it in that die's L2; the longest blocks come first.
#include "attn_bf16_common.h"


namespace tempo {
namespace {

typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* global_ptr;

__device__ inline float max3(float a, float b, float c) {
  float r;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}

// Online softmax of one group for this kernel, with a LAZY reference: weights are
// 2^(x - ref) where ref follows the running maximum only when the maximum has
// grown by more than kSlack (in log2 units) since ref was set, so weights stay
// below 2^kSlack (exact in fp32 sums, same relative rounding in bf16) and the
// accumulators are rescaled a few times per column instead of at every new
// maximum.  The result acc / sum does not depend on ref.  The running sum is one
// more accumulator tile (weights times a column of ones on the matrix cores).
constexpr float kSlack = 8.0f;

// First half: move the reference if this group's maximum calls for it.  x holds the
// RAW dot products (masked ones are -inf); `scale` > 0 is s * log2(e).
template <int D>
__device__ inline void softmax_reference(const float* x, float scale, int lane, float& ref, f32x4* acc,
                                         f32x4& acc_l) {
  constexpr int DT = D / 16;
  const int c = lane >> 4;
  // (three-operand maxima written out: fmaxf() first canonicalises each matrix-core result)
  float mx = max3(max3(max3(max3(x[0], x[1], x[2]), x[3], x[4]), x[5], x[6]), x[7], x[7]);
  mx = column_max(mx) * scale;
  // ref = -inf until the column sees its first key; -inf + kSlack = -inf, so any finite mx moves it
  const bool move = mx > ref + kSlack;
  if (__any(move)) {
    const float ref_new = move ? mx : ref;
    const float alpha = move ? fast_exp2(ref - ref_new) : 1.0f;  // exp2(-inf) = 0 on the first key
    ref = ref_new;
    float a[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) a[r] = __shfl(alpha, 4 * c + r);
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[dt][r] *= a[r];
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) acc_l[r] *= a[r];
  }
}

// Second half: the bf16 weights 2^(scale * x - ref), the scale applied inside one fused
// multiply-add.
__device__ inline bf16x8 softmax_weights(const float* x, float scale, float ref) {
  const float base = ref == -INFINITY ? 0.f : ref;  // a column that has seen no key yet: weights exp2(-inf) = 0
  bf16x8 pa;
#pragma unroll
  for (int i = 0; i < 8; ++i) pa[i] = (__bf16)fast_exp2(fmaf(x[i], scale, -base));
  return pa;
}

// Steps per workgroup for a query group of G heads: all 16 x `waves` columns.
__host__ __device__ inline int prefill_block_steps(int G, int waves) { return (16 * waves) / G; }

// NW wavefronts per workgroup, 16 columns per wavefront.  (Two column tiles per
// wavefront would halve the LDS reads per column, but the accumulators then cost a
// wavefront of occupancy: measured slower, 2.56 against 2.45 ms on the 4096-step prompt.)
//
// The loop is software-pipelined by one group: iteration n computes the logits of group
// n + 1 (matrix cores) next to the softmax of group n (vector ALU), then the
// weights x values products of group n.  The two kinds of work of one wavefront are
// independent inside an iteration, so they overlap instead of alternating.  Keys
// therefore run one group ahead of values through LDS: two key buffers (groups n + 1,
// n + 2) and two value buffers (groups n, n + 1).
template <int D, int NW, bool kRope, bool kStream>
__global__ __launch_bounds__(64 * NW) void attn_prefill_bf16(AttnParams p) {
  constexpr int KS = D / 32;
  constexpr int DT = D / 16;
  constexpr int KU = 2 * KS;                  // 1 KiB units of one group's keys
  constexpr int UNITS = KU + DT;              // ... and of its keys and values together
  constexpr int PER_THREAD = (UNITS + NW - 1) / NW;  // units each wavefront copies per iteration (at most)
  // A block in front of a long history reads every key/value once and no other workgroup reads
  // them again: non-temporal copies (the cache-policy bit the decode kernel's loads carry) keep
  // them from displacing anything.  The blocks of a prompt share keys/values through L2: cached.
  constexpr int kCachePolicy = kStream ? 2 : 0;
  extern __shared__ u32x4 lds[];              // keys [2][KU][64] x 16 bytes, then values [2][DT][64] x 16 bytes
  u32x4* const lds_k = lds;
  u32x4* const lds_v = lds + 2 * KU * 64;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int QB = prefill_block_steps(p.G, NW);
  const int nblocks = (p.queries + QB - 1) / QB;
  // Which (block, split, kv head, sequence) this workgroup takes.  Workgroups are handed
  // to the 8 accelerator dies (XCDs, each with its own L2) round-robin by linear index;
  // the blocks of one (sequence, head) read the same keys/values, so each die is given a
  // contiguous run of the work list instead: workgroup L takes item (L mod 8) * (n / 8)
  // + L / 8 (remainder items spread over the first dies), and the blocks that run
  // together on a die share its L2.
  const unsigned nx = gridDim.x, ny = gridDim.y, total = nx * ny * gridDim.z;
  const unsigned linear = blockIdx.x + nx * (blockIdx.y + ny * blockIdx.z);
  const unsigned die = linear & 7u, share = total >> 3, extra = total & 7u;
  const unsigned item = die * share + (die < extra ? die : extra) + (linear >> 3);
  const unsigned ix = item % nx, iyz = item / nx;
  const int qb = nblocks - 1 - (int)(ix % nblocks);           // longest range first
  const int zsplit = (int)(ix / nblocks);                     // 0 unless the key range is split
  const int hkv = (int)(iyz % ny), b = (int)(iyz / ny);
  const int c0 = qb * QB;                                           // first step of the block within the call
  // steps of this sequence in the call: all of them, or its own count
  int steps_b = p.queries;
  if (p.count_per_seq) {
    const int n = ((const_i32_ptr)p.count_per_seq)[b];
    steps_b = n < 0 ? 0 : (n < p.queries ? n : p.queries);
  }
  if (c0 >= steps_b) return;                                        // uniform over the workgroup, before any barrier
  const int C = steps_b - c0 < QB ? steps_b - c0 : QB;             // steps in this block
  const int ncols = C * p.G;
  int t_base = p.t_per_seq ? ((const_i32_ptr)p.t_per_seq)[b] : p.t; // first step of the call for this sequence
  t_base = t_base > p.t ? p.t : (t_base < 0 ? 0 : t_base);
  const int t_first = t_base + c0, t_last = t_first + C - 1;
  const int lo = (p.window > 0 && t_first - p.window + 1 > 0) ? t_first - p.window + 1 : 0;
  // The split of the key range this workgroup walks (the whole range when not split:
  // tps_log2 = 30), newest split first as in the decode kernel.
  const int chunk0 = lo >> p.tps_log2;
  const int nchunks = (t_last >> p.tps_log2) - chunk0 + 1;
  if (zsplit >= nchunks) return;                                    // uniform over the workgroup
  const int split = nchunks - 1 - zsplit;
  const int cs = (chunk0 + split) << p.tps_log2, ce = cs + ((1 << p.tps_log2) - 1);
  const int start = lo > cs ? lo : cs;
  const int end = t_last < ce ? t_last : ce;
  const int g_first = start >> 5, g_last = end >> 5;

  // wavefront-uniform bounds over this wavefront's 16 columns, cut to the split:
  // the groups it has any work in, and those no column cuts
  const int first_col = 16 * wave;
  const int last_col = (first_col + 15) < ncols - 1 ? (first_col + 15) : ncols - 1;
  const bool idle = first_col >= ncols;                             // a wavefront beyond the block's columns
  const int own_hi = t_first + (idle ? 0 : last_col / p.G);         // newest key any of its columns sees
  const int own_hi_min = t_first + (idle ? 0 : first_col / p.G);    // newest key ALL of its columns see
  const int own_lo_first = (p.window > 0 && own_hi_min - p.window + 1 > 0) ? own_hi_min - p.window + 1 : 0;
  const int own_lo_last = (p.window > 0 && own_hi - p.window + 1 > 0) ? own_hi - p.window + 1 : 0;
  const int w_hi = own_hi < end ? own_hi : end, w_hi_min = own_hi_min < end ? own_hi_min : end;
  const int w_lo_first = own_lo_first > start ? own_lo_first : start;
  const int w_lo_last = own_lo_last > start ? own_lo_last : start;
  // has this wavefront any work in group g / does some column's range cut group g?  (wave-uniform)
  auto active = [&](int g) { return !idle && (g << 5) <= w_hi && (g << 5) + 31 >= w_lo_first; };
  auto is_cut = [&](int g) { return (g << 5) < w_lo_last || (g << 5) + 31 > w_hi_min; };

  // This lane's column (unused columns behave like the block's last step with q = 0),
  // its range, its query operand, its softmax state.
  const int col = first_col + (lane & 15);
  const int cq = col < ncols ? col / p.G : C - 1;
  const int gq = col < ncols ? col - cq * p.G : 0;
  const int step = t_first + cq;               // the column's own step: its newest key and its position
  const int hi_col = step < end ? step : end;
  const int lo_own = (p.window > 0 && step - p.window + 1 > 0) ? step - p.window + 1 : 0;
  const int lo_col = lo_own > start ? lo_own : start;
  u32x4 qreg[KS];
  {
    const int c = lane >> 4;
    const uint16_t* qp = static_cast<const uint16_t*>(p.q) +
                         (((int64_t)b * p.io_steps + c0 + cq) * p.Hq + (int64_t)hkv * p.G + gq) * D + 8 * c;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const u32x4 zero = {0u, 0u, 0u, 0u};
      const u32x4 v = *reinterpret_cast<const u32x4*>(qp + 32 * s);
      qreg[s] = col < ncols ? v : zero;
    }
    if (kRope) rotate_query<D>(p, step, lane, qreg);  // queries arrive unrotated
  }
  float m_run = -INFINITY;                     // softmax reference of column lane&15 (log2 units)
  f32x4 acc[DT];                               // lane (n + 16c): dims 16dt + n of columns 4c .. 4c+3
  f32x4 acc_l = {0.f, 0.f, 0.f, 0.f};          // running sums of columns 4c .. 4c+3 (the same in every n)
#pragma unroll
  for (int dt = 0; dt < DT; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};  // bf16 1.0 x 8

  // Copy of a group: wavefront w moves units w, w + NW, ... of the group's 1 KiB units
  // (keys first, then values).  The pool image is already what the consumers read, so
  // the copy goes from global memory straight into LDS (gfx950's 16-byte global -> LDS
  // load: lane i's piece lands at the wavefront's LDS base + 16 i); completion is counted
  // by the vector-memory counter.
  // Where a group sits in either pool: its block-table entry (a scalar load, asked for
  // one iteration before it is needed so that nobody waits for it) and the offset that
  // follows from it.
  const_i32_ptr table = (const_i32_ptr)p.block_table + (int64_t)b * p.max_blocks_per_seq;
  auto entry_of = [&](int g) {
    const int gc = g < g_last ? g : g_last;  // never past the range's last tile
    return table[((gc << 5) >> p.z_log2) & p.tile_mask];
  };
  auto offset_of = [&](int entry, int g) -> int64_t {
    const int phys = clamp_block(entry, p.num_blocks);
    return (((int64_t)phys * p.Hkv + hkv) << p.z_log2) * D + (int64_t)((g << 5) & ((1 << p.z_log2) - 1)) * D;
  };
  auto issue_keys = [&](int gk, int64_t offset) {
    if (gk > g_last) return;  // uniform over the workgroup
    const char* from = reinterpret_cast<const char*>(static_cast<const uint16_t*>(p.k_pool) + offset);
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int u = wave + NW * i;  // wave-uniform
      if (u < KU)  // (wavefronts beyond the units copy nothing)
        __builtin_amdgcn_global_load_lds((global_ptr)(from + u * 1024 + lane * 16),
                                         (lds_ptr)(lds_k + ((gk & 1) * KU + u) * 64), 16, 0, kCachePolicy);
    }
  };
  auto issue_values = [&](int gv, int64_t offset) {
    if (gv > g_last) return;
    const char* from = reinterpret_cast<const char*>(static_cast<const uint16_t*>(p.v_pool) + offset);
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int u = wave + NW * i - KU;
      if (u >= 0 && u < DT)
        __builtin_amdgcn_global_load_lds((global_ptr)(from + u * 1024 + lane * 16),
                                         (lds_ptr)(lds_v + ((gv & 1) * DT + u) * 64), 16, 0, kCachePolicy);
    }
  };
  // Slots beyond the block's last step may be unwritten (NaN): the 0 mask under the
  // sums is applied once, to the value units of the range's last group, in LDS, by the
  // wavefront that copied the unit and after its copy has landed (the copy keeps the
  // lane of every 16-byte piece, so a lane masks the slots its consumers will read from
  // it).  Masked slots inside the range hold written data and weight 0.
  const bool tail = (g_last << 5) + 31 > t_last;  // uniform over the workgroup
  auto mask_values = [&](int gv) {  // gv == g_last, and tail
    uint32_t keep[4];
    value_masks(gv, 0, t_last, lane, keep);
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int u = wave + NW * i - KU;
      if (u < 0 || u >= DT) continue;
      u32x4* at = lds_v + ((gv & 1) * DT + u) * 64 + lane;
      u32x4 v = *at;
      v.x &= keep[0]; v.y &= keep[1]; v.z &= keep[2]; v.w &= keep[3];
      *at = v;
    }
  };
  // End of an iteration: wait until this wavefront's copies have landed, fix up what it
  // must, wait for its LDS stores, then meet the other wavefronts.  Written out instead
  // of __syncthreads() so that the waits are the ones this loop needs; the "memory"
  // clobbers keep the compiler from moving LDS accesses across.
  auto landed = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
  auto meet = [&]() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); };

  // Raw dot products of this wavefront's columns with the 32 keys of group g (two row tiles).
  auto logits = [&](int g, float* x) {
    const u32x4* src = lds_k + (g & 1) * KU * 64 + lane;
    f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(src[s * 64]), as_bf16x8(qreg[s]), sa, 0, 0, 0);
      sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(src[(KS + s) * 64]), as_bf16x8(qreg[s]), sb, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) { x[r] = sa[r]; x[4 + r] = sb[r]; }
  };

  int64_t off_v;     // offset of group n + 1: its keys were copied an iteration before its values
  int entry_next;    // block-table entry of group n + 2
  {
    const int e0 = entry_of(g_first), e1 = entry_of(g_first + 1);
    entry_next = entry_of(g_first + 2);
    const int64_t off0 = offset_of(e0, g_first);
    off_v = offset_of(e1, g_first + 1);
    issue_keys(g_first, off0);
    issue_keys(g_first + 1, off_v);
    issue_values(g_first, off0);
  }
  landed();
  if (tail && g_first == g_last) mask_values(g_first);
  meet();
  float xc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // logits of the current group
  if (active(g_first)) logits(g_first, xc);

  for (int grp = g_first; grp <= g_last; ++grp) {
    // Buffers (g + 2) & 1 of the keys and (g + 1) & 1 of the values held groups g and
    // g - 1, which everybody finished in the previous iteration.
    const int64_t off_k = offset_of(entry_next, grp + 2);
    entry_next = entry_of(grp + 3);
    issue_keys(grp + 2, off_k);
    issue_values(grp + 1, off_v);
    off_v = off_k;

    if (active(grp)) {
      if (is_cut(grp)) mask_logits(grp, lo_col, hi_col, lane, xc);
      softmax_reference<D>(xc, p.scale_log2e, lane, m_run, acc, acc_l);
      // The next group's logits: independent of the softmax below.  Beyond the last group
      // this reads a key buffer of an earlier group (or LDS nobody wrote); the result is unused.
      float xn[8];
      logits(grp + 1, xn);
      const bf16x8 pa = softmax_weights(xc, p.scale_log2e, m_run);
      acc_l = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, as_bf16x8(ones), acc_l, 0, 0, 0);
      const u32x4* src = lds_v + (grp & 1) * DT * 64 + lane;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
        acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, as_bf16x8(src[dt * 64]), acc[dt], 0, 0, 0);
#pragma unroll
      for (int i = 0; i < 8; ++i) xc[i] = xn[i];
    } else if (grp + 1 <= g_last && active(grp + 1)) {
      logits(grp + 1, xc);
    }

    landed();
    if (tail && grp + 1 == g_last) mask_values(grp + 1);
    meet();  // groups n + 1 (values) and n + 2 (keys) are in LDS; nobody reads group n any more
  }

  // Columns (4c + r) of acc, value dims 16dt + n.  Whole range: every column saw its own
  // key, so its sum is > 0 and the output is acc / sum.  One split of the range: the
  // column's partial (reference, sum, accumulator) goes to the workspace; a column
  // that saw no key in this split leaves (-inf, 0, 0).
  const int n = lane & 15, c = lane >> 4;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int j = first_col + 4 * c + r;
    const float l_j = acc_l[r];
    const float ref_j = __shfl(m_run, 4 * c + r);  // the reference lives in lane (column & 15)
    if (j < ncols) {
      const int jc = j / p.G, jg = j - jc * p.G;
      if (p.direct) {
        __bf16* orow = static_cast<__bf16*>(p.out) +
                       (((int64_t)b * p.io_steps + c0 + jc) * p.Hq + (int64_t)hkv * p.G + jg) * D;
        const float inv = 1.0f / l_j;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) orow[16 * dt + n] = (__bf16)(acc[dt][r] * inv);
      } else {
        const int64_t row = ((int64_t)b * p.queries + c0 + jc) * p.Hq + (int64_t)hkv * p.G + jg;
        const int64_t part = row * p.num_splits + split;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) p.ws_acc[part * D + 16 * dt + n] = acc[dt][r];
        if (n == 0) {
          p.ws_ml[part * 2] = ref_j;
          p.ws_ml[part * 2 + 1] = l_j;
        }
      }
    }
  }
}

}  // namespace

// The prompt path uses kPromptWaves wavefronts; a single block of fewer columns gets a
// workgroup of just enough wavefronts (2, 4 or 8), so that several workgroups share a
// compute unit and the kernel stays bound by HBM.
constexpr int kPromptWaves = 8;

int prefill_bf16_block_steps(int G) { return prefill_block_steps(G, kPromptWaves); }

namespace {
template <int NW>
hipError_t launch_prefill_nw(const AttnParams& p, int batch, int D, int grid_splits, hipStream_t stream) {
  const int QB = prefill_block_steps(p.G, NW);
  const int nblocks = (p.queries + QB - 1) / QB;
  // the kernel renumbers its workgroups with 32-bit arithmetic on the linear index
  if ((int64_t)nblocks * grid_splits * p.Hkv * batch > INT32_MAX) return hipErrorInvalidConfiguration;
  const dim3 grid(nblocks * grid_splits, p.Hkv, batch);
  const dim3 block(64 * NW);
  const size_t lds = 2 * (size_t)(2 * (D / 32) + D / 16) * 1024;
  const bool stream_once = !p.direct;  // split path: each workgroup's range is read by nobody else
  if (p.rope_cos) {
    if (D == 128) {
      return stream_once ? launch((attn_prefill_bf16<128, NW, true, true>), grid, block, lds, stream, p)
                         : launch((attn_prefill_bf16<128, NW, true, false>), grid, block, lds, stream, p);
    }
    return stream_once ? launch((attn_prefill_bf16<64, NW, true, true>), grid, block, lds, stream, p)
                       : launch((attn_prefill_bf16<64, NW, true, false>), grid, block, lds, stream, p);
  }
  if (D == 128) {
    return stream_once ? launch((attn_prefill_bf16<128, NW, false, true>), grid, block, lds, stream, p)
                       : launch((attn_prefill_bf16<128, NW, false, false>), grid, block, lds, stream, p);
  }
  return stream_once ? launch((attn_prefill_bf16<64, NW, false, true>), grid, block, lds, stream, p)
                     : launch((attn_prefill_bf16<64, NW, false, false>), grid, block, lds, stream, p);
}
}  // namespace

// grid_splits: splits of the key range to launch (1 = every workgroup walks its
// block's whole range and writes `out`; p.tps_log2 must then be 30).
hipError_t launch_prefill_bf16(const AttnParams& p, int batch, int D, int grid_splits, hipStream_t stream) {
  const int columns = p.queries * p.G;
  if (columns <= 32) return launch_prefill_nw<2>(p, batch, D, grid_splits, stream);
  if (columns <= 64) return launch_prefill_nw<4>(p, batch, D, grid_splits, stream);
  return launch_prefill_nw<kPromptWaves>(p, batch, D, grid_splits, stream);
}

}  // namespace tempo
