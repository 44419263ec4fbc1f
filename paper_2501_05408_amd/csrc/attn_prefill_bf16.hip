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
// reads its operands from LDS.  LDS buffers in a ring: the copy of a later group
// (global -> LDS loads issued at the top of the iteration, waited for at its end)
// overlaps the arithmetic on group n; one barrier per group.
//
// Blocks against a long history.  The same kernel serves a block of up to 128
// columns in front of a long key range (chunked prompt processing, speculative
// decoding with many steps): the key range is then cut into splits as in the decode
// kernel, one workgroup per (sequence, kv head, split) writes a partial
// (reference, sum, accumulator) per column, and the split combine finishes.  The
// keys/values are read from HBM once per workgroup for all its columns.
//
// Workgroups of one (sequence, head) are adjacent in the grid and run together, so
// the pool is streamed from HBM about once per (sequence, head) and the blocks that
// follow find it in the caches; the longest blocks are dispatched first.
#include "attn_bf16_common.h"

// The instantiation that is built: wavefronts per workgroup, column tiles per
// wavefront, and the occupancy (wavefronts per SIMD) the register allocation must
// allow.  Measured on the 4096-step x 16-sequence prompt: 8 x 1 2.45 ms, 4 x 2 (two
// per SIMD) 2.56 ms, 8 x 2 2.70 ms, 4 x 1 3.14 ms.
#ifndef PROMPT_NW
#define PROMPT_NW 8
#define PROMPT_NT 1
#define PROMPT_MIN_WAVES 1
#endif
#ifndef PROMPT_NBUF_SMALL
#define PROMPT_NBUF_SMALL 2
#define PROMPT_NBUF_SPLIT 2
#endif
#ifndef PROMPT_NBUF_DIRECT
#define PROMPT_NBUF_DIRECT 2
#endif

namespace tempo {
namespace {

typedef __attribute__((address_space(3))) void* lds_ptr;
typedef const __attribute__((address_space(1))) void* global_ptr;

// Maximum over the four lanes {l, l^16, l^32, l^48} that hold one column's logits,
// left in all four.  Two lane-swap instructions of gfx950 instead of two trips
// through the LDS permute unit: v_permlane16_swap exchanges the odd 16-lane rows of
// its first operand with the even rows of its second, v_permlane32_swap the upper
// half of the first with the lower half of the second; with both operands holding
// the same values, the maximum of the two results is the exchange-and-reduce step.
__device__ inline float column_max(float v) {
  float a = v, b = v;
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 0\n\tv_max_f32 %0, %0, %1" : "+v"(a), "+v"(b));
  float c = a, d = a;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 0\n\tv_max_f32 %0, %0, %1" : "+v"(c), "+v"(d));
  return c;
}

// Online softmax of one group for this kernel, with a LAZY reference: weights are
// 2^(x - ref) where ref follows the running maximum only when the maximum has
// grown by more than kSlack (in log2 units) since ref was set, so weights stay
// below 2^kSlack (exact in fp32 sums, same relative rounding in bf16) and the
// accumulators are rescaled a few times per column instead of at every new
// maximum.  The result acc / sum does not depend on ref.  The running sum is one
// more accumulator tile (weights times a column of ones on the matrix cores).
constexpr float kSlack = 8.0f;

// x holds the RAW dot products (masked ones are -inf); `scale` > 0 is s * log2(e),
// applied to the maximum once and to the weights inside one fused multiply-add.
template <int D>
__device__ inline bf16x8 prompt_softmax(const float* x, float scale, int lane, float& ref, f32x4* acc,
                                        f32x4& acc_l) {
  constexpr int DT = D / 16;
  const int c = lane >> 4;
  float mx = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
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
  const float base = ref == -INFINITY ? 0.f : ref;  // a column that has seen no key yet: weights exp2(-inf) = 0
  bf16x8 pa;
#pragma unroll
  for (int i = 0; i < 8; ++i) pa[i] = (__bf16)fast_exp2(fmaf(x[i], scale, -base));
  return pa;
}

// Steps per workgroup for a query group of G heads: all `waves` x `tiles` x 16 columns.
__host__ __device__ inline int prefill_block_steps(int G, int waves, int tiles) { return (16 * waves * tiles) / G; }

// NW wavefronts per workgroup, NT column tiles (of 16 columns) per wavefront.  The
// key/value operands a wavefront reads from LDS serve all its NT tiles, so LDS
// traffic per column falls with NT; the accumulators (NT x (D/16 + 1) tiles) set
// the register budget.
template <int D, int NW, int NT, int NBUF, bool kRope>
__global__ __launch_bounds__(64 * NW, PROMPT_MIN_WAVES) void attn_prefill_bf16(AttnParams p) {
  constexpr int KS = D / 32;
  constexpr int DT = D / 16;
  constexpr int UNITS = 2 * KS + DT;          // 1 KiB units of one group: keys then values
  constexpr int PER_THREAD = UNITS / NW;      // units each wavefront copies per group
  static_assert(UNITS % NW == 0, "units must divide among the wavefronts");
  extern __shared__ u32x4 lds[];              // [NBUF][UNITS][64] x 16 bytes
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int QB = prefill_block_steps(p.G, NW, NT);
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

  // wavefront-uniform bounds over this wavefront's 16 * NT columns, cut to the split:
  // the groups it has any work in, and those no column cuts
  const int first_col = 16 * NT * wave;
  const int last_col = (first_col + 16 * NT - 1) < ncols - 1 ? (first_col + 16 * NT - 1) : ncols - 1;
  const bool idle = first_col >= ncols;                             // a wavefront beyond the block's columns
  const int own_hi = t_first + (idle ? 0 : last_col / p.G);         // newest key any of its columns sees
  const int own_hi_min = t_first + (idle ? 0 : first_col / p.G);    // newest key ALL of its columns see
  const int own_lo_first = (p.window > 0 && own_hi_min - p.window + 1 > 0) ? own_hi_min - p.window + 1 : 0;
  const int own_lo_last = (p.window > 0 && own_hi - p.window + 1 > 0) ? own_hi - p.window + 1 : 0;
  const int w_hi = own_hi < end ? own_hi : end, w_hi_min = own_hi_min < end ? own_hi_min : end;
  const int w_lo_first = own_lo_first > start ? own_lo_first : start;
  const int w_lo_last = own_lo_last > start ? own_lo_last : start;

  // Per column tile: this lane's column (unused columns behave like the block's last
  // step with q = 0), its range, its query operand, its softmax state.
  int lo_col[NT], hi_col[NT];
  u32x4 qreg[NT][KS];
  float m_run[NT];                             // softmax reference of column lane&15 (log2 units)
  f32x4 acc[NT][DT];                           // lane (n + 16c): dims 16dt + n of columns 4c .. 4c+3
  f32x4 acc_l[NT];                             // running sums of columns 4c .. 4c+3 (the same in every n)
#pragma unroll
  for (int jt = 0; jt < NT; ++jt) {
    const int col = first_col + 16 * jt + (lane & 15);
    const int cq = col < ncols ? col / p.G : C - 1;
    const int gq = col < ncols ? col - cq * p.G : 0;
    const int step = t_first + cq;             // the column's own step: its newest key and its position
    hi_col[jt] = step < end ? step : end;
    const int lo_own = (p.window > 0 && step - p.window + 1 > 0) ? step - p.window + 1 : 0;
    lo_col[jt] = lo_own > start ? lo_own : start;
    const int c = lane >> 4;
    const uint16_t* qp = static_cast<const uint16_t*>(p.q) +
                         (((int64_t)b * p.io_steps + c0 + cq) * p.Hq + (int64_t)hkv * p.G + gq) * D + 8 * c;
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      const u32x4 zero = {0u, 0u, 0u, 0u};
      const u32x4 v = *reinterpret_cast<const u32x4*>(qp + 32 * s);
      qreg[jt][s] = col < ncols ? v : zero;
    }
    if (kRope) rotate_query<D>(p, step, lane, qreg[jt]);  // queries arrive unrotated
    m_run[jt] = -INFINITY;
    acc_l[jt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) acc[jt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  const u32x4 ones = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};  // bf16 1.0 x 8

  // Copy of one group: wavefront w moves units w, w + NW, ... (keys are units
  // 0 .. 2KS-1 of the key pool's group, values units 2KS .. of the value pool's).
  // The pool image is already what the consumers read, so the copy goes from global
  // memory straight into LDS (gfx950's 16-byte global -> LDS load: lane i's piece lands
  // at the wavefront's LDS base + 16 i), two groups ahead of the arithmetic, through
  // three LDS buffers; completion is counted by the vector-memory counter.
  auto copy_direct = [&](int buf, int grp) {
    const int64_t base = group_base<D>(p, b, hkv, grp);
    const u32x4* kp = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.k_pool) + base) + lane;
    const u32x4* vp = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.v_pool) + base) + lane;
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int u = wave + NW * i;  // wave-uniform
      const u32x4* from = u < 2 * KS ? kp + u * 64 : vp + (u - 2 * KS) * 64;
      __builtin_amdgcn_global_load_lds((global_ptr)from, (lds_ptr)(lds + (buf * UNITS + u) * 64), 16, 0, 0);
    }
  };
  // Slots beyond the block's last step may be unwritten (NaN): the 0 mask under the
  // sums is applied once, to the value units of the range's last group.  That one group
  // goes through registers (load, mask, LDS store; the copy keeps the lane of every
  // 16-byte piece, so the lane's slots are the consumer's).  Masked slots inside the
  // range hold written data and weight 0.
  const bool tail = (g_last << 5) + 31 > t_last;  // uniform over the workgroup
  u32x4 stage[PER_THREAD];
  auto fetch = [&](int grp) {
    const int64_t base = group_base<D>(p, b, hkv, grp);
    const u32x4* kp = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.k_pool) + base) + lane;
    const u32x4* vp = reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.v_pool) + base) + lane;
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int u = wave + NW * i;
      stage[i] = u < 2 * KS ? kp[u * 64] : vp[(u - 2 * KS) * 64];
    }
  };
  auto stash = [&](int buf, int grp) {
    uint32_t keep[4];
    value_masks(grp, 0, t_last, lane, keep);
#pragma unroll
    for (int i = 0; i < PER_THREAD; ++i) {
      const int u = wave + NW * i;
      u32x4 v = stage[i];
      if (u >= 2 * KS) { v.x &= keep[0]; v.y &= keep[1]; v.z &= keep[2]; v.w &= keep[3]; }
      lds[(buf * UNITS + u) * 64 + lane] = v;
    }
  };
  // Wait until this wavefront's loads have landed (all of them, or all but the newest
  // group's) and its LDS stores are done, then meet the other wavefronts.  Written out
  // instead of __syncthreads(): its fence would wait for every outstanding global -> LDS
  // load, the ones for the group after next included, which is the overlap this loop is
  // built for.  The "memory" clobbers keep the compiler from moving LDS accesses across.
  auto meet = [&](bool newest_pending) {
    if (newest_pending && NBUF == 3) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PER_THREAD) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  };

  // Groups g_first and g_first + 1 before the loop, group n + 2 at the top of iteration n.
  bool second = false;
  if (tail && g_first == g_last) {
    fetch(g_first);
    stash(0, g_first);
  } else {
    copy_direct(0, g_first);
    second = NBUF == 3 && g_first + 1 <= g_last && !(tail && g_first + 1 == g_last);
    if (second) copy_direct(1, g_first + 1);
  }
  meet(second);

  int buf = 0;  // LDS buffer of the current group; group n + k sits in buffer (buf + k) mod NBUF
  for (int grp = g_first; grp <= g_last; ++grp) {
    const int buf1 = buf == NBUF - 1 ? 0 : buf + 1;               // buffer of group n + 1
    const int bufa = buf == 0 ? NBUF - 1 : buf - 1;                // buffer of group n + NBUF - 1
    const bool via_regs = tail && grp + 1 == g_last;               // the next group is the masked one
    const bool ahead = grp + NBUF - 1 <= g_last && !(tail && grp + NBUF - 1 == g_last);
    if (ahead) copy_direct(bufa, grp + NBUF - 1);  // that buffer held group n - 1: everybody is past it
    if (via_regs) fetch(grp + 1);

    // Has this wavefront anything to do in this group?  (Uniform over the wavefront.)
    const int j0 = grp << 5;
    if (!idle && j0 <= w_hi && j0 + 31 >= w_lo_first) {
      const u32x4* src = lds + buf * UNITS * 64 + lane;
      const bool cut = j0 < w_lo_last || j0 + 31 > w_hi_min;
      bf16x8 pa[NT];
      {
        Group<D> g;  // only the key half is used: the operands serve all NT tiles
#pragma unroll
        for (int i = 0; i < 2 * KS; ++i) g.k[i] = src[i * 64];
#pragma unroll
        for (int jt = 0; jt < NT; ++jt) {
          float x[8];  // raw dot products of the two row tiles
          f32x4 sa = {0.f, 0.f, 0.f, 0.f}, sb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int s = 0; s < KS; ++s) {
            sa = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(g.k[s]), as_bf16x8(qreg[jt][s]), sa, 0, 0, 0);
            sb = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(g.k[KS + s]), as_bf16x8(qreg[jt][s]), sb, 0, 0, 0);
          }
#pragma unroll
          for (int r = 0; r < 4; ++r) { x[r] = sa[r]; x[4 + r] = sb[r]; }
          if (cut) mask_logits(grp, lo_col[jt], hi_col[jt], lane, x);
          pa[jt] = prompt_softmax<D>(x, p.scale_log2e, lane, m_run[jt], acc[jt], acc_l[jt]);
          acc_l[jt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa[jt], as_bf16x8(ones), acc_l[jt], 0, 0, 0);
        }
      }
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const u32x4 vv = src[(2 * KS + dt) * 64];
#pragma unroll
        for (int jt = 0; jt < NT; ++jt)
          acc[jt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa[jt], as_bf16x8(vv), acc[jt][dt], 0, 0, 0);
      }
    }

    // group n + 1 must be in LDS before anybody starts on it; group n + 2 may still be in flight
    if (via_regs) stash(buf1, grp + 1);
    meet(ahead);  // via_regs implies !ahead: the masked group is the last one
    buf = buf1;
  }

  // Columns (4c + r) of acc, value dims 16dt + n.  Whole range: every column saw its own
  // key, so its sum is > 0 and the output is acc / sum.  One split of the range: the
  // column's partial (reference, sum, accumulator) goes to the workspace; a column
  // that saw no key in this split leaves (-inf, 0, 0).
  const int n = lane & 15, c = lane >> 4;
#pragma unroll
  for (int jt = 0; jt < NT; ++jt) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int j = first_col + 16 * jt + 4 * c + r;
      const float l_j = acc_l[jt][r];
      const float ref_j = __shfl(m_run[jt], 4 * c + r);  // the reference lives in lane (column & 15)
      if (j < ncols) {
        const int jc = j / p.G, jg = j - jc * p.G;
        if (p.direct) {
          __bf16* orow = static_cast<__bf16*>(p.out) +
                         (((int64_t)b * p.io_steps + c0 + jc) * p.Hq + (int64_t)hkv * p.G + jg) * D;
          const float inv = 1.0f / l_j;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) orow[16 * dt + n] = (__bf16)(acc[jt][dt][r] * inv);
        } else {
          const int64_t row = ((int64_t)b * p.queries + c0 + jc) * p.Hq + (int64_t)hkv * p.G + jg;
          const int64_t part = row * p.num_splits + split;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt) p.ws_acc[part * D + 16 * dt + n] = acc[jt][dt][r];
          if (n == 0) {
            p.ws_ml[part * 2] = ref_j;
            p.ws_ml[part * 2 + 1] = l_j;
          }
        }
      }
    }
  }
}

}  // namespace

// The prompt path uses kPromptWaves wavefronts of kPromptTiles tiles; a single block
// of fewer columns gets a workgroup of just enough wavefronts (2, 4 or 8), so that
// several workgroups share a compute unit and the kernel stays bound by HBM.
constexpr int kPromptWaves = PROMPT_NW, kPromptTiles = PROMPT_NT;

int prefill_bf16_block_steps(int G) { return prefill_block_steps(G, kPromptWaves, kPromptTiles); }

namespace {
template <int NW, int NBUF>
hipError_t launch_prefill_nw(const AttnParams& p, int batch, int D, int grid_splits, hipStream_t stream) {
  constexpr int NT = kPromptTiles;
  const int QB = prefill_block_steps(p.G, NW, NT);
  const int nblocks = (p.queries + QB - 1) / QB;
  const dim3 grid(nblocks * grid_splits, p.Hkv, batch);
  const dim3 block(64 * NW);
  const size_t lds = NBUF * (size_t)(2 * (D / 32) + D / 16) * 1024;
  if (p.rope_cos) {
    if (D == 128) return launch((attn_prefill_bf16<128, NW, NT, NBUF, true>), grid, block, lds, stream, p);
    return launch((attn_prefill_bf16<64, NW, NT, NBUF, true>), grid, block, lds, stream, p);
  }
  if (D == 128) return launch((attn_prefill_bf16<128, NW, NT, NBUF, false>), grid, block, lds, stream, p);
  return launch((attn_prefill_bf16<64, NW, NT, NBUF, false>), grid, block, lds, stream, p);
}
}  // namespace

// grid_splits: splits of the key range to launch (1 = every workgroup walks its
// block's whole range and writes `out`; p.tps_log2 must then be 30).
hipError_t launch_prefill_bf16(const AttnParams& p, int batch, int D, int grid_splits, hipStream_t stream) {
  const int columns = p.queries * p.G;
  if (kPromptTiles == 1 && columns <= 32) return launch_prefill_nw<2, PROMPT_NBUF_SMALL>(p, batch, D, grid_splits, stream);
  if (kPromptTiles == 1 && columns <= 64) return launch_prefill_nw<4, PROMPT_NBUF_SMALL>(p, batch, D, grid_splits, stream);
  if (!p.direct) return launch_prefill_nw<kPromptWaves, PROMPT_NBUF_SPLIT>(p, batch, D, grid_splits, stream);
  return launch_prefill_nw<kPromptWaves, PROMPT_NBUF_DIRECT>(p, batch, D, grid_splits, stream);
}

}  // namespace tempo
