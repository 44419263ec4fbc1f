// The C ABI declared in tempo.h: argument validation, split planning, launches.
// Host code only; every step of the path runs in the kernels this file launches.
#include <math.h>
#include <limits.h>
#include <stdio.h>

#include <mutex>

#include "tempo_internal.h"

namespace {

using namespace tempo;

int ilog2_exact(int32_t v) {  // log2 of a power of two, else -1
  if (v <= 0 || (v & (v - 1)) != 0) return -1;
  int k = 0;
  while ((1 << k) < v) ++k;
  return k;
}

// Layout fields only (no pointers): dtype, head_dim, block_size, heads, counts.
int check_layout(const tempo_kv* kv) {
  if (!kv) return TEMPO_ERR_NULL;
  if (kv->dtype != TEMPO_BF16 && kv->dtype != TEMPO_F32) return TEMPO_ERR_DTYPE;
  if (kv->head_dim != 64 && kv->head_dim != 128) return TEMPO_ERR_SHAPE;
  const int zl = ilog2_exact(kv->block_size);
  if (zl < 0) return TEMPO_ERR_SHAPE;
  if (kv->dtype == TEMPO_BF16 && kv->block_size < 32) return TEMPO_ERR_SHAPE;
  if (kv->dtype == TEMPO_F32 && kv->block_size < 4) return TEMPO_ERR_SHAPE;
  if (kv->num_kv_heads < 1 || kv->num_kv_heads > 65535) return TEMPO_ERR_SHAPE;
  if (kv->num_blocks < 1 || kv->max_blocks_per_seq < 1) return TEMPO_ERR_SHAPE;
  if (kv->ring_blocks != 0 &&
      (ilog2_exact(kv->ring_blocks) < 0 || kv->ring_blocks > kv->max_blocks_per_seq))
    return TEMPO_ERR_SHAPE;
  return TEMPO_OK;
}

int check_store(const tempo_kv* kv) {
  const int rc = check_layout(kv);
  if (rc != TEMPO_OK) return rc;
  if (!kv->k_pool || !kv->v_pool || !kv->block_table) return TEMPO_ERR_NULL;
  return TEMPO_OK;
}

// A block of C consecutive query steps: its C * (Hq / Hkv) (step, head) columns
// either ride in the 16-column tile of the decode kernel or, up to 128, are spread
// over the eight wavefronts of the LDS-staged kernel (the same limit for fp32).
// A single step of a group of more than 16 query heads is such a block of one step.
constexpr int kMaxColumns = 128;
// Up to this many columns the single-step kernel (one 16-column tile) serves the call.
constexpr int kNarrowColumns = 16;

int check_heads(const tempo_kv* kv, int32_t batch, int32_t Hq) {
  if (batch < 1 || batch > 65535) return TEMPO_ERR_SHAPE;
  if (Hq < 1 || Hq % kv->num_kv_heads != 0) return TEMPO_ERR_SHAPE;
  if (Hq / kv->num_kv_heads > kMaxColumns || Hq > 65535) return TEMPO_ERR_SHAPE;
  return TEMPO_OK;
}

int check_queries(const tempo_kv* kv, int32_t Hq, int32_t queries) {
  if (queries < 1 || queries > kMaxColumns) return TEMPO_ERR_SHAPE;
  if ((int64_t)queries * (Hq / kv->num_kv_heads) > kMaxColumns) return TEMPO_ERR_SHAPE;
  if ((int64_t)queries * Hq > 65535) return TEMPO_ERR_SHAPE;
  return TEMPO_OK;
}

// The constant s of Eq. 1: finite and positive (the kernels take maxima of raw dot
// products and scale afterwards).
int check_scale(float scale) { return (scale > 0.0f && scale <= 3.0e38f) ? TEMPO_OK : TEMPO_ERR_RANGE; }

// The steps a block of queries starting at t touches: the last step, and the
// window measured from the last step that spans the union of the queries' ranges.
int32_t last_step(int32_t t, int32_t queries) { return t + (queries - 1); }
int32_t union_window(int32_t window, int32_t queries) { return window > 0 ? window + (queries - 1) : 0; }

// A linear store must have a table column for step t's tile; a ring store reuses
// its columns, so any step can be written.
int check_step(const tempo_kv* kv, int32_t t) {
  if (t < 0) return TEMPO_ERR_RANGE;
  if (kv->ring_blocks == 0 && t / kv->block_size >= kv->max_blocks_per_seq) return TEMPO_ERR_RANGE;
  return TEMPO_OK;
}

// What a ring store can still answer: every tile of the visible range of step t
// (and of any earlier step with the same window) must be resident, i.e. the range
// may touch at most ring_blocks tiles.
int check_ring_covers(const tempo_kv* kv, int32_t t, int32_t window) {
  if (kv->ring_blocks == 0) return TEMPO_OK;
  const int64_t Z = kv->block_size;
  int64_t tiles;
  if (window == 0 || window > (int64_t)t + 1) tiles = t / Z + 1;           // the whole history
  else tiles = window <= 1 ? 1 : ((int64_t)window - 2 + Z) / Z + 1;         // worst alignment
  return tiles <= kv->ring_blocks ? TEMPO_OK : TEMPO_ERR_RANGE;
}

// Rotary tables: both present, made for this head_dim, and long enough for step t.
int check_rope(const tempo_rope* rope, int32_t head_dim, int32_t t_last) {
  if (!rope || !rope->cos || !rope->sin) return TEMPO_ERR_NULL;
  if (rope->head_dim != head_dim) return TEMPO_ERR_SHAPE;
  if ((reinterpret_cast<uintptr_t>(rope->cos) & 15u) != 0 || (reinterpret_cast<uintptr_t>(rope->sin) & 15u) != 0)
    return TEMPO_ERR_SHAPE;
  if (t_last < 0 || rope->positions < 1 || t_last >= rope->positions) return TEMPO_ERR_RANGE;
  return TEMPO_OK;
}

int32_t tile_mask_of(const tempo_kv* kv) { return kv->ring_blocks ? kv->ring_blocks - 1 : INT32_MAX; }

// Upper bound of the number of splits any step t' <= t can need with this tps.
int32_t splits_bound(int32_t t, int32_t window, int tps_log2) {
  const int32_t causal = (t >> tps_log2) + 1;
  if (window <= 0) return causal;
  // a run of `window` keys starting anywhere touches at most ceil((window-1)/tps)+1 chunks
  const int32_t tps = 1 << tps_log2;
  const int32_t win = (window <= 1) ? 1 : (int32_t)(((int64_t)window - 2 + tps) >> tps_log2) + 1;
  return causal < win ? causal : win;
}

// Compute units of the part this library is written for (MI355X).
constexpr int kComputeUnits = 256;
constexpr int kMaxSplits = 1024;

// Split planning: a small time model of the launch, in nanoseconds, with constants
// measured on MI355X.
//   - Workgroups are handed to compute units round-robin, so the busiest unit gets
//     rounds = ceil(workgroups / units) of them, one after the other.
//   - A unit streams keys/values at its share of what the memory system sustains for
//     this access pattern (about 6.9 TB/s over all units), but never faster than
//     about 40 GB/s, so fewer than ~170 busy units cannot use the whole bandwidth.
//   - A launch pays about 2 us once before its first key arrives (dispatch, kernel
//     arguments, block table, first loads), about 1 us per round (a workgroup's own
//     argument -> table -> data chain and its merge and partial write, as far as the other
//     workgroups resident on the unit do not hide them; fitted on steps that are not powers
//     of two, where short splits looked better than they are), and about 3 us for the
//     combine launch if there is more than one split.
// Short splits balance better; long splits mean fewer rounds, fewer partials and,
// at one split, no combine at all.  Take the LONGEST split length whose estimate is
// within 3% of the best one.
constexpr double kSustainedBytesPerNs = 6900.0;  // whole part, GB/s
constexpr double kUnitBytesPerNs = 40.0;         // one compute unit, GB/s
constexpr double kLaunchNs = 2000.0, kRoundNs = 1000.0, kCombineNs = 3000.0;

double plan_cost_ns(int64_t pairs, int64_t splits, int64_t keys_per_split, int bytes_per_key) {
  const int64_t workgroups = pairs * splits;
  const int64_t busy = workgroups < kComputeUnits ? workgroups : kComputeUnits;
  const double share = kSustainedBytesPerNs / (double)busy;
  const double rate = share < kUnitBytesPerNs ? share : kUnitBytesPerNs;
  const int64_t rounds = (workgroups + kComputeUnits - 1) / kComputeUnits;
  return kLaunchNs + (double)rounds * (kRoundNs + (double)keys_per_split * bytes_per_key / rate) +
         (splits > 1 ? kCombineNs : 0.0);
}

// Ragged batches (per-sequence steps below t_max) hold less work than the model
// assumes and it is unevenly spread, so their splits are capped at 1024 keys to
// keep the long sequences from becoming single long-running workgroups.
void make_plan(const tempo_kv* kv, int32_t batch, int32_t Hq, int32_t t_max, int32_t window,
               bool ragged, tempo_plan* plan) {
  // bf16 shares one key/value read across the query group; fp32 launches per query head.
  const int64_t pairs = (int64_t)batch * (kv->dtype == TEMPO_BF16 ? kv->num_kv_heads : Hq);
  const int64_t len = (window > 0 && window < (int64_t)t_max + 1) ? window : (int64_t)t_max + 1;
  const int bytes_per_key = 2 * kv->head_dim * (kv->dtype == TEMPO_BF16 ? 2 : 4);  // K and V of one head
  const int k_max = ragged ? 10 : 30;
  int best_k = -1;
  double best_cost = -1.0;
  double costs[26];
  for (int k = 5; k <= 30; ++k) costs[k - 5] = -1.0;
  for (int k = 5; k <= k_max; ++k) {
    const int64_t splits = splits_bound(t_max, window, k);
    if (splits > kMaxSplits) continue;
    const int64_t tps = (int64_t)1 << k;
    const int64_t per_split = tps < len ? tps : len;  // a split never holds more than the range
    costs[k - 5] = plan_cost_ns(pairs, splits, per_split, bytes_per_key);
    if (best_cost < 0.0 || costs[k - 5] < best_cost) best_cost = costs[k - 5];
    if (splits == 1) break;  // longer splits change nothing
  }
  for (int k = 5; k <= k_max; ++k) {
    if (costs[k - 5] >= 0.0 && costs[k - 5] <= best_cost * 1.03) best_k = k;
  }
  if (best_k < 0) {  // a ragged range too long for 1024 splits of 1024 keys: lengthen until it fits
    best_k = k_max;
    while (splits_bound(t_max, window, best_k) > kMaxSplits) ++best_k;
  }
  plan->tokens_per_split = 1 << best_k;
  plan->num_splits = splits_bound(t_max, window, best_k);
  // About 8 wavefronts per compute unit keep the memory pipe full: 4 per workgroup
  // when a unit gets two or more workgroups, 8 when it gets at most one (measured:
  // 256 workgroups x 8 waves 42.4 us, x 4 waves 43.4 us; 512 x 4 waves 42.7 us), down
  // to one 32-slot group per wavefront (256 keys at batch 16: 7.7 us with 8, 8.2 with 4).
  const int groups = plan->tokens_per_split / 32;
  const int64_t workgroups = pairs * plan->num_splits;
  if (workgroups <= kComputeUnits && groups >= 8) plan->waves = 8;
  else plan->waves = groups >= 4 ? 4 : groups;
}

// A uniform step needs its own split count; ragged steps (any t' <= t) need the bound.
int check_plan(const tempo_plan* plan, int32_t t, int32_t window, bool ragged, int32_t queries,
               int32_t pad_t = 0) {
  if (!plan) return TEMPO_ERR_NULL;
  const int k = ilog2_exact(plan->tokens_per_split);
  if (k < 5) return TEMPO_ERR_SHAPE;
  if (plan->waves != 1 && plan->waves != 2 && plan->waves != 4 && plan->waves != 8) return TEMPO_ERR_SHAPE;
  if (plan->num_splits < 1 || plan->num_splits > 65535) return TEMPO_ERR_SHAPE;
  const int32_t cover = last_step(t, queries) > pad_t ? last_step(t, queries) : pad_t;
  const int32_t need = ragged ? splits_bound(cover, union_window(window, queries), k)
                              : seq_range(t, window, k, queries, pad_t).nchunks;
  if (plan->num_splits < need) return TEMPO_ERR_RANGE;
  return TEMPO_OK;
}

// Map a launch status to the ABI's; say on stderr what the runtime said.
int launch_status(hipError_t e, const char* what) {
  if (e == hipSuccess) return TEMPO_OK;
  fprintf(stderr, "libtempo: launch of %s failed: %s\n", what, hipGetErrorString(e));
  return TEMPO_ERR_LAUNCH;
}

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- statically allocated partials for callers that cannot allocate -----------------
// tempo_decode_step_causal_noalloc keeps the split partials here instead of in a caller's
// workspace.  Each GPU holds its own copy of the array, at its own address, until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress:
// the address kernels are given is the one that call returned for the current device.
constexpr size_t kScratchBytes = (size_t)8 << 20;
__attribute__((used)) static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, resolved once per device.
int scratch_on_current_device(void** ptr) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    fprintf(stderr, "libtempo: no current device for the static scratch array: %s\n", hipGetErrorString(e));
    return TEMPO_ERR_LAUNCH;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      fprintf(stderr, "libtempo: hipGetSymbolAddress(scratch) failed on device %d: %s\n", dev, hipGetErrorString(e));
      return TEMPO_ERR_LAUNCH;
    }
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return TEMPO_OK;
}


// Workspace = [m,l: rows*S*2 f32] [acc: rows*S*D f32], each part padded to 256 bytes;
// rows = batch * queries * Hq.
size_t ml_bytes(int64_t rows, int32_t S) { return align_up((size_t)rows * S * 2 * sizeof(float), 256); }

size_t plan_bytes(const tempo_kv* kv, int64_t rows, int32_t S) {
  return ml_bytes(rows, S) + align_up((size_t)rows * S * kv->head_dim * sizeof(float), 256);
}

constexpr size_t kMaxLds = 64 * 1024;

AttnParams attn_params(const tempo_kv* kv, const void* q, void* out, int32_t Hq, int32_t t,
                       const int32_t* t_per_seq, int32_t window, float scale,
                       const tempo_plan* plan, void* workspace, int32_t batch, int32_t queries,
                       int32_t pad_t = 0) {
  AttnParams p;
  p.k_pool = kv->k_pool;
  p.v_pool = kv->v_pool;
  p.block_table = kv->block_table;
  p.q = q;
  p.k_new = nullptr;
  p.v_new = nullptr;
  p.t_per_seq = t_per_seq;
  p.count_per_seq = nullptr;
  p.rope_cos = nullptr;
  p.rope_sin = nullptr;
  p.worklist = nullptr;
  char* ws = static_cast<char*>(workspace);
  p.ws_ml = reinterpret_cast<float*>(ws);
  p.ws_acc = reinterpret_cast<float*>(ws + ml_bytes((int64_t)batch * queries * Hq, plan->num_splits));
  p.out = out;
  p.t = t;
  p.window = window;
  p.z_log2 = ilog2_exact(kv->block_size);
  p.max_blocks_per_seq = kv->max_blocks_per_seq;
  p.tile_mask = tile_mask_of(kv);
  p.num_blocks = kv->num_blocks;
  p.Hkv = kv->num_kv_heads;
  p.Hq = Hq;
  p.G = Hq / kv->num_kv_heads;
  p.tps_log2 = ilog2_exact(plan->tokens_per_split);
  p.num_splits = plan->num_splits;
  p.queries = queries;
  p.io_steps = queries;
  p.pad_t = pad_t;
  p.direct = 0;
  p.scale_log2e = scale * 1.44269504088896340736f;
  return p;
}

StoreParams store_params(const tempo_kv* kv, int32_t batch, int32_t t, const int32_t* t_per_seq,
                         int32_t count = 1) {
  StoreParams p;
  p.k_pool = kv->k_pool;
  p.v_pool = kv->v_pool;
  p.block_table = kv->block_table;
  p.t_per_seq = t_per_seq;
  p.t = t;
  p.z_log2 = ilog2_exact(kv->block_size);
  p.max_blocks_per_seq = kv->max_blocks_per_seq;
  p.tile_mask = tile_mask_of(kv);
  p.num_blocks = kv->num_blocks;
  p.Hkv = kv->num_kv_heads;
  p.batch = batch;
  p.count = count;
  p.src_steps = count;
  p.count_per_seq = nullptr;
  p.row0 = 0;
  p.rope_cos = nullptr;
  p.rope_sin = nullptr;
  return p;
}

// Splits to launch along grid.x: exact for a uniform step, the bound for ragged steps.
int32_t grid_splits(const tempo_plan* plan, int32_t t, const int32_t* t_per_seq, int32_t window,
                    int32_t queries, int32_t pad_t) {
  if (t_per_seq) return plan->num_splits;
  const int32_t exact = seq_range(t, window, ilog2_exact(plan->tokens_per_split), queries, pad_t).nchunks;
  return exact < plan->num_splits ? exact : plan->num_splits;
}

int check_attn(const tempo_kv* kv, int32_t batch, int32_t Hq, int32_t t, int32_t window, bool ragged,
               const tempo_plan* plan, const void* workspace, size_t workspace_bytes,
               int32_t queries = 1, int32_t pad_t = 0) {
  int rc = check_store(kv);
  if (rc != TEMPO_OK) return rc;
  if ((rc = check_heads(kv, batch, Hq)) != TEMPO_OK) return rc;
  if ((rc = check_queries(kv, Hq, queries)) != TEMPO_OK) return rc;
  if (window < 0 || t < 0 || t > INT32_MAX - 64) return TEMPO_ERR_RANGE;
  // the padded baseline is causal only: with a window the range's length would depend on the step
  if (pad_t < 0 || (pad_t > 0 && window != 0)) return TEMPO_ERR_RANGE;
  const int32_t cover = last_step(t, queries) > pad_t ? last_step(t, queries) : pad_t;
  if ((rc = check_step(kv, cover)) != TEMPO_OK) return rc;
  if ((rc = check_ring_covers(kv, cover, union_window(window, queries))) != TEMPO_OK) return rc;
  if ((rc = check_plan(plan, t, window, ragged, queries, pad_t)) != TEMPO_OK) return rc;
  if (kv->dtype == TEMPO_BF16) {
    const int columns = queries * (Hq / kv->num_kv_heads);
    // more than 16 columns go to the LDS-staged kernel, whose launch shape is fixed
    if (columns <= kNarrowColumns && partial_bf16_lds_bytes(plan->waves, columns, kv->head_dim) > kMaxLds) return TEMPO_ERR_SHAPE;
  }
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return TEMPO_ERR_WORKSPACE;
  if (workspace_bytes < plan_bytes(kv, (int64_t)batch * queries * Hq, plan->num_splits)) return TEMPO_ERR_WORKSPACE;
  return TEMPO_OK;
}

// out != nullptr and a single split: the launch writes `out` itself; otherwise it
// writes partials and the caller launches the combine.
// k_new/v_new != nullptr: step t's key/value are appended inside the same launch.
int do_partial(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new, void* out,
               int32_t batch, int32_t Hq, int32_t t, const int32_t* t_per_seq, int32_t window,
               float scale, const tempo_plan* plan, void* workspace, hipStream_t stream,
               int32_t queries = 1, const tempo_rope* rope = nullptr, int32_t pad_t = 0, int32_t io_steps = 0,
               const int32_t* worklist = nullptr) {
  AttnParams p = attn_params(kv, q, out, Hq, t, t_per_seq, window, scale, plan, workspace, batch, queries, pad_t);
  if (io_steps > 0) p.io_steps = io_steps;
  p.worklist = worklist;
  p.direct = (out != nullptr && plan->num_splits == 1) ? 1 : 0;
  p.k_new = k_new;
  p.v_new = v_new;
  if (rope) {
    p.rope_cos = rope->cos;
    p.rope_sin = rope->sin;
  }
  const int32_t gs = grid_splits(plan, t, t_per_seq, window, queries, pad_t);
  if (kv->dtype == TEMPO_BF16 && queries * p.G > kNarrowColumns)  // a wide block: the LDS-staged kernel, key range split as planned
    return launch_status(launch_prefill_bf16(p, batch, kv->head_dim, gs, stream), "attn_block_partial");
  const hipError_t e = kv->dtype == TEMPO_BF16
                           ? launch_partial_bf16(p, batch, kv->head_dim, gs, plan->waves, stream)
                           : launch_partial_f32(p, batch, kv->head_dim, gs, plan->waves, stream);
  return launch_status(e, "attn_decode_partial");
}

int do_combine(const tempo_kv* kv, void* out, int32_t batch, int32_t Hq, int32_t t,
               const int32_t* t_per_seq, int32_t window, const tempo_plan* plan, void* workspace,
               hipStream_t stream, int32_t queries = 1, int32_t pad_t = 0, int32_t io_steps = 0) {
  AttnParams p = attn_params(kv, nullptr, out, Hq, t, t_per_seq, window, 1.0f, plan, workspace, batch, queries,
                             pad_t);
  if (io_steps > 0) p.io_steps = io_steps;
  const hipError_t e = launch_combine(p, batch, kv->head_dim, kv->dtype, stream);
  return launch_status(e, "attn_decode_combine");
}

// Plan of a block of queries: the plan of the union range, with the wavefront count
// cut down until the bf16 kernel's wave-merge area (one accumulator row per column
// and wavefront) fits the LDS a workgroup may ask for.
void make_block_plan(const tempo_kv* kv, int32_t batch, int32_t Hq, int32_t t, int32_t window,
                     bool ragged, int32_t queries, tempo_plan* plan) {
  make_plan(kv, batch, Hq, last_step(t, queries), union_window(window, queries), ragged, plan);
  if (kv->dtype != TEMPO_BF16) return;
  const int columns = queries * (Hq / kv->num_kv_heads);
  if (columns > kNarrowColumns) {
    // The LDS-staged kernel: its workgroups do more arithmetic per key than the decode
    // kernel's, so two per compute unit are wanted (measured at batch 16 x 8 heads,
    // t = 4095: 4 splits of 1024 keys 59-68 us for 63-126 columns, 2 splits 82-83 us,
    // 8 splits 68-81 us).
    // Longest split length of at least 256 keys that gives >= 512 workgroups, else 256.
    // Up to 32 columns a workgroup has only two wavefronts: twice as many workgroups
    // (measured there: 8 splits of 512 keys 52.8-53.8 us, 4 splits of 1024 keys 55.5-56.1 us).
    const int32_t t_eff = last_step(t, queries), w_eff = union_window(window, queries);
    const int64_t pairs = (int64_t)batch * kv->num_kv_heads;
    const int64_t want = (columns <= 32 ? 4 : 2) * (int64_t)kComputeUnits;
    int k = 8;
    for (int cand = 30; cand >= 8; --cand) {
      if (pairs * splits_bound(t_eff, w_eff, cand) >= want) { k = cand; break; }
    }
    while (splits_bound(t_eff, w_eff, k) > kMaxSplits) ++k;
    if (ragged && k > 10 && splits_bound(t_eff, w_eff, 10) <= kMaxSplits) k = 10;  // as for single steps
    plan->tokens_per_split = 1 << k;
    plan->num_splits = splits_bound(t_eff, w_eff, k);
    plan->waves = 8;  // ignored: the launch picks 2, 4 or 8 wavefronts by the column count
    return;
  }
  while (plan->waves > 1 && partial_bf16_lds_bytes(plan->waves, columns, kv->head_dim) > kMaxLds) plan->waves /= 2;
}

int decode(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new, void* out,
           int32_t batch, int32_t Hq, int32_t t, const int32_t* t_per_seq, int32_t window, float scale,
           void* workspace, size_t workspace_bytes, void* stream, int32_t queries = 1,
           const tempo_rope* rope = nullptr, int32_t pad_t = 0, const int32_t* worklist = nullptr) {
  int rc = check_layout(kv);
  if (rc != TEMPO_OK) return rc;
  if (!q || !out) return TEMPO_ERR_NULL;
  if ((rc = check_heads(kv, batch, Hq)) != TEMPO_OK) return rc;
  if ((rc = check_queries(kv, Hq, queries)) != TEMPO_OK) return rc;
  if (t < 0 || window < 0 || t > INT32_MAX - 64) return TEMPO_ERR_RANGE;
  if ((rc = check_scale(scale)) != TEMPO_OK) return rc;
  if (rope && (rc = check_rope(rope, kv->head_dim, last_step(t, queries))) != TEMPO_OK) return rc;
  if (pad_t < 0 || pad_t > INT32_MAX - 64) return TEMPO_ERR_RANGE;
  tempo_plan plan;
  // the padded baseline is planned as the step it pretends every step to be
  make_block_plan(kv, batch, Hq, pad_t > t ? pad_t : t, window, t_per_seq != nullptr, queries, &plan);
  if ((rc = check_attn(kv, batch, Hq, t, window, t_per_seq != nullptr, &plan, workspace, workspace_bytes, queries,
                       pad_t)) != TEMPO_OK)
    return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // With more (sequence, head) pairs than compute units the in-kernel block-store write
  // costs more than a launch of its own (measured at 512 pairs: +7.5 us inside the
  // attention kernel, +4 us as a separate launch; at 128 pairs +1 us inside): write first.
  // A group of more than 16 query heads runs in the LDS-staged kernel, which reads the
  // store only: the write (rotating the key when tables are given) goes first there too,
  // and the kernel rotates the queries.
  const bool wide = kv->dtype == TEMPO_BF16 && queries * (Hq / kv->num_kv_heads) > kNarrowColumns;
  if (k_new && kv->dtype == TEMPO_BF16 && (wide || (!rope && (int64_t)batch * kv->num_kv_heads > kComputeUnits))) {
    const StoreParams sp = store_params(kv, batch, t, t_per_seq);
    const hipError_t e = rope ? launch_rope_append(sp, rope->cos, rope->sin, k_new, v_new, kv->head_dim, kv->dtype, s)
                              : launch_append(sp, k_new, v_new, kv->head_dim, kv->dtype, s);
    if ((rc = launch_status(e, "kv_append")) != TEMPO_OK) return rc;
    k_new = v_new = nullptr;
  }
  rc = do_partial(kv, q, k_new, v_new, out, batch, Hq, t, t_per_seq, window, scale, &plan, workspace, s, queries,
                  rope, pad_t, 0, worklist);
  if (rc != TEMPO_OK || plan.num_splits == 1) return rc;  // a single split wrote `out` itself
  return do_combine(kv, out, batch, Hq, t, t_per_seq, window, &plan, workspace, s, queries, pad_t);
}

}  // namespace

extern "C" {

int tempo_visible_range(int32_t t, int32_t window, int32_t Z, int32_t* lo, int32_t* hi,
                        int32_t* first_tile, int32_t* last_tile, int32_t* first_tile_skip,
                        int32_t* last_tile_valid) {
  if (t < 0 || window < 0 || Z < 1) return TEMPO_ERR_RANGE;
  const int32_t l = (window > 0 && t - window + 1 > 0) ? t - window + 1 : 0;
  if (lo) *lo = l;
  if (hi) *hi = t;
  if (first_tile) *first_tile = l / Z;
  if (last_tile) *last_tile = t / Z;
  if (first_tile_skip) *first_tile_skip = l % Z;
  if (last_tile_valid) *last_tile_valid = t % Z + 1;
  return TEMPO_OK;
}

int tempo_append_slot(int32_t t, int32_t Z, int32_t* tile, int32_t* slot) {
  if (t < 0 || Z < 1) return TEMPO_ERR_RANGE;
  if (tile) *tile = t / Z;
  if (slot) *slot = t % Z;
  return TEMPO_OK;
}

int tempo_kv_release(int32_t t, int32_t window, int32_t Z, int32_t* dead_keys, int32_t* dead_tiles) {
  if (t < 0 || t == INT32_MAX || window < 0 || Z < 1) return TEMPO_ERR_RANGE;  // t + 1 keys must be countable
  // the last reader of key j is step j + window - 1: dead after step t iff j <= t - window + 1
  int64_t dead = window == 0 ? 0 : (int64_t)t - window + 2;
  if (dead < 0) dead = 0;
  if (dead_keys) *dead_keys = (int32_t)dead;
  if (dead_tiles) *dead_tiles = (int32_t)(dead / Z);
  return TEMPO_OK;
}

int tempo_ring_blocks(int32_t window, int32_t Z, int32_t queries, int32_t* ring_blocks) {
  if (!ring_blocks) return TEMPO_ERR_NULL;
  if (window < 1 || Z < 1 || queries < 1) return TEMPO_ERR_RANGE;
  // the union of the queries' ranges, at its worst alignment to the tiles
  const int64_t span = (int64_t)window + queries - 1;
  const int64_t tiles = span <= 1 ? 1 : (span - 2 + Z) / Z + 1;
  if (tiles > (1 << 30)) return TEMPO_ERR_RANGE;
  int32_t ring = 1;
  while (ring < tiles) ring *= 2;
  *ring_blocks = ring;
  return TEMPO_OK;
}

int64_t tempo_kv_element_offset(const tempo_kv* kv, int32_t which, int32_t block, int32_t head,
                                int32_t slot, int32_t d) {
  if (check_layout(kv) != TEMPO_OK) return -1;
  if (which < 0 || which > 1 || block < 0 || block >= kv->num_blocks || head < 0 ||
      head >= kv->num_kv_heads || slot < 0 || slot >= kv->block_size || d < 0 || d >= kv->head_dim)
    return -1;
  const int D = kv->head_dim;
  const int64_t base = ((int64_t)block * kv->num_kv_heads + head) * kv->block_size * D;
  if (kv->dtype == TEMPO_F32) return base + tile_off_f32(D, slot, d);
  return base + (which == 0 ? tile_off_k_bf16(D, slot, d) : tile_off_v_bf16(D, slot, d));
}

size_t tempo_kv_pool_bytes(const tempo_kv* kv) {
  if (check_layout(kv) != TEMPO_OK) return 0;
  const size_t e = kv->dtype == TEMPO_BF16 ? 2 : 4;
  return (size_t)kv->num_blocks * kv->num_kv_heads * kv->block_size * kv->head_dim * e;
}

int tempo_attn_plan(const tempo_kv* kv, int32_t batch, int32_t num_q_heads, int32_t t_max,
                    int32_t window, int32_t ragged, tempo_plan* plan) {
  int rc = check_layout(kv);
  if (rc != TEMPO_OK) return rc;
  if (!plan) return TEMPO_ERR_NULL;
  if ((rc = check_heads(kv, batch, num_q_heads)) != TEMPO_OK) return rc;
  if (t_max < 0 || window < 0) return TEMPO_ERR_RANGE;
  make_block_plan(kv, batch, num_q_heads, t_max, window, ragged != 0, 1, plan);
  return TEMPO_OK;
}

size_t tempo_attn_plan_workspace_bytes(const tempo_kv* kv, int32_t batch, int32_t num_q_heads,
                                       const tempo_plan* plan) {
  if (check_layout(kv) != TEMPO_OK || !plan) return 0;
  if (check_heads(kv, batch, num_q_heads) != TEMPO_OK || plan->num_splits < 1) return 0;
  return plan_bytes(kv, (int64_t)batch * num_q_heads, plan->num_splits);
}

size_t tempo_attn_workspace_bytes(const tempo_kv* kv, int32_t batch, int32_t num_q_heads,
                                  int32_t max_t) {
  if (check_layout(kv) != TEMPO_OK || max_t < 0) return 0;
  if (check_heads(kv, batch, num_q_heads) != TEMPO_OK) return 0;
  // The planner's split count is not monotone in t, so take the largest count it
  // produces for any step up to max_t and any window.  A shorter range or a window
  // never needs more splits than the causal range of max_t at the same split
  // length, and the planner only chooses lengths of at least 32, so the causal
  // count at length 32, capped at the planner's own maximum, bounds them all.
  int64_t worst = splits_bound(max_t, 0, 5);
  if (worst > kMaxSplits) worst = kMaxSplits;
  return plan_bytes(kv, (int64_t)batch * num_q_heads, (int32_t)worst);
}

int tempo_attn_block_plan(const tempo_kv* kv, int32_t batch, int32_t num_q_heads, int32_t queries,
                          int32_t t_max, int32_t window, int32_t ragged, tempo_plan* plan) {
  int rc = check_layout(kv);
  if (rc != TEMPO_OK) return rc;
  if (!plan) return TEMPO_ERR_NULL;
  if ((rc = check_heads(kv, batch, num_q_heads)) != TEMPO_OK) return rc;
  if ((rc = check_queries(kv, num_q_heads, queries)) != TEMPO_OK) return rc;
  if (t_max < 0 || t_max > INT32_MAX - 64 || window < 0 || window > INT32_MAX - 64) return TEMPO_ERR_RANGE;
  make_block_plan(kv, batch, num_q_heads, t_max, window, ragged != 0, queries, plan);
  return TEMPO_OK;
}

size_t tempo_attn_block_workspace_bytes(const tempo_kv* kv, int32_t batch, int32_t num_q_heads,
                                        int32_t queries, int32_t max_t) {
  if (check_layout(kv) != TEMPO_OK || max_t < 0 || max_t > INT32_MAX - 64) return 0;
  if (check_heads(kv, batch, num_q_heads) != TEMPO_OK) return 0;
  if (check_queries(kv, num_q_heads, queries) != TEMPO_OK) return 0;
  // as tempo_attn_workspace_bytes, for the union range that ends at the last query's step
  int64_t worst = splits_bound(last_step(max_t, queries), 0, 5);
  if (worst > kMaxSplits) worst = kMaxSplits;
  return plan_bytes(kv, (int64_t)batch * queries * num_q_heads, (int32_t)worst);
}

const char* tempo_strerror(int status) {
  switch (status) {
    case TEMPO_OK: return "ok";
    case TEMPO_ERR_NULL: return "a required pointer is NULL";
    case TEMPO_ERR_SHAPE: return "unsupported shape (head_dim, block_size, head counts or batch)";
    case TEMPO_ERR_RANGE: return "step or window out of range for this block store";
    case TEMPO_ERR_WORKSPACE: return "workspace is NULL, misaligned or too small";
    case TEMPO_ERR_DTYPE: return "unknown dtype";
    case TEMPO_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

int tempo_kv_append(const tempo_kv* kv, const void* k_new, const void* v_new, int32_t batch,
                    int32_t t, const int32_t* t_per_seq, void* stream) {
  int rc = check_store(kv);
  if (rc != TEMPO_OK) return rc;
  if (!k_new || !v_new) return TEMPO_ERR_NULL;
  if (batch < 1 || batch > 65535) return TEMPO_ERR_SHAPE;
  if ((rc = check_step(kv, t)) != TEMPO_OK) return rc;
  if ((int64_t)batch * kv->num_kv_heads * kv->head_dim > INT32_MAX) return TEMPO_ERR_SHAPE;
  const StoreParams p = store_params(kv, batch, t, t_per_seq);
  const hipError_t e = launch_append(p, k_new, v_new, kv->head_dim, kv->dtype, static_cast<hipStream_t>(stream));
  return launch_status(e, "kv_append");
}

int tempo_kv_append_block(const tempo_kv* kv, const void* k_new, const void* v_new, int32_t batch,
                          int32_t t, const int32_t* t_per_seq, int32_t count, void* stream) {
  int rc = check_store(kv);
  if (rc != TEMPO_OK) return rc;
  if (!k_new || !v_new) return TEMPO_ERR_NULL;
  if (batch < 1 || batch > 65535) return TEMPO_ERR_SHAPE;
  if (count < 1 || count > 65536) return TEMPO_ERR_SHAPE;
  if (t < 0 || t > INT32_MAX - count) return TEMPO_ERR_RANGE;
  if ((rc = check_step(kv, t + count - 1)) != TEMPO_OK) return rc;
  // a ring store must not wrap onto rows of the same call
  if (kv->ring_blocks && (int64_t)count > (int64_t)kv->ring_blocks * kv->block_size) return TEMPO_ERR_RANGE;
  if ((int64_t)batch * count * kv->num_kv_heads * kv->head_dim > INT32_MAX) return TEMPO_ERR_SHAPE;
  const StoreParams p = store_params(kv, batch, t, t_per_seq, count);
  const hipError_t e = launch_append(p, k_new, v_new, kv->head_dim, kv->dtype, static_cast<hipStream_t>(stream));
  return launch_status(e, "kv_append_block");
}

int tempo_rope_kv_append_block(const tempo_kv* kv, const tempo_rope* rope, const void* k_raw, const void* v_new,
                               int32_t batch, int32_t t, const int32_t* t_per_seq, int32_t count, void* stream) {
  int rc = check_store(kv);
  if (rc != TEMPO_OK) return rc;
  if (!k_raw || !v_new) return TEMPO_ERR_NULL;
  if (kv->dtype != TEMPO_BF16) return TEMPO_ERR_DTYPE;  // the block write rotates in the bf16 kernels only
  if (batch < 1 || batch > 65535) return TEMPO_ERR_SHAPE;
  if (count < 1 || count > 65536) return TEMPO_ERR_SHAPE;
  if (t < 0 || t > INT32_MAX - count) return TEMPO_ERR_RANGE;
  if ((rc = check_step(kv, t + count - 1)) != TEMPO_OK) return rc;
  if ((rc = check_rope(rope, kv->head_dim, t + count - 1)) != TEMPO_OK) return rc;
  if (kv->ring_blocks && (int64_t)count > (int64_t)kv->ring_blocks * kv->block_size) return TEMPO_ERR_RANGE;
  if ((int64_t)batch * count * kv->num_kv_heads * kv->head_dim > INT32_MAX) return TEMPO_ERR_SHAPE;
  StoreParams p = store_params(kv, batch, t, t_per_seq, count);
  p.rope_cos = rope->cos;
  p.rope_sin = rope->sin;
  const hipError_t e = launch_append(p, k_raw, v_new, kv->head_dim, kv->dtype, static_cast<hipStream_t>(stream));
  return launch_status(e, "kv_rope_append_block");
}

int tempo_kv_gather(const tempo_kv* kv, void* k_out, void* v_out, int32_t batch, int32_t j0,
                    int32_t count, void* stream) {
  int rc = check_store(kv);
  if (rc != TEMPO_OK) return rc;
  if (batch < 1 || batch > 65535) return TEMPO_ERR_SHAPE;
  if (j0 < 0 || count < 0) return TEMPO_ERR_RANGE;
  if (count == 0) return TEMPO_OK;
  if ((int64_t)j0 + count - 1 > INT32_MAX) return TEMPO_ERR_RANGE;
  if ((rc = check_step(kv, j0 + count - 1)) != TEMPO_OK) return rc;
  if (kv->ring_blocks && (int64_t)count > (int64_t)kv->ring_blocks * kv->block_size) return TEMPO_ERR_RANGE;
  const StoreParams p = store_params(kv, batch, 0, nullptr);
  const hipError_t e = launch_gather(p, k_out, v_out, kv->head_dim, kv->dtype, j0, count,
                                     static_cast<hipStream_t>(stream));
  return launch_status(e, "kv_gather");
}

int tempo_attn_decode_causal(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                             int32_t num_q_heads, int32_t t, const int32_t* t_per_seq,
                             float scale, void* workspace, size_t workspace_bytes, void* stream) {
  return decode(kv, q, nullptr, nullptr, out, batch, num_q_heads, t, t_per_seq, 0, scale, workspace,
                workspace_bytes, stream);
}

int tempo_attn_decode_window(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                             int32_t num_q_heads, int32_t t, const int32_t* t_per_seq,
                             int32_t window, float scale, void* workspace,
                             size_t workspace_bytes, void* stream) {
  if (window < 1) return TEMPO_ERR_RANGE;
  return decode(kv, q, nullptr, nullptr, out, batch, num_q_heads, t, t_per_seq, window, scale, workspace,
                workspace_bytes, stream);
}

int tempo_decode_step_causal(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new,
                             void* out, int32_t batch, int32_t num_q_heads, int32_t t,
                             const int32_t* t_per_seq, float scale, void* workspace,
                             size_t workspace_bytes, void* stream) {
  if (!k_new || !v_new) return TEMPO_ERR_NULL;
  return decode(kv, q, k_new, v_new, out, batch, num_q_heads, t, t_per_seq, 0, scale, workspace,
                workspace_bytes, stream);
}

int tempo_decode_step_window(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new,
                             void* out, int32_t batch, int32_t num_q_heads, int32_t t,
                             const int32_t* t_per_seq, int32_t window, float scale, void* workspace,
                             size_t workspace_bytes, void* stream) {
  if (!k_new || !v_new) return TEMPO_ERR_NULL;
  if (window < 1) return TEMPO_ERR_RANGE;
  return decode(kv, q, k_new, v_new, out, batch, num_q_heads, t, t_per_seq, window, scale, workspace,
                workspace_bytes, stream);
}

int tempo_decode_step_causal_noalloc(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new,
                                     void* out, int32_t batch, int32_t num_q_heads, int32_t t,
                                     const int32_t* t_per_seq, float scale, void* stream) {
  if (!k_new || !v_new) return TEMPO_ERR_NULL;
  int rc = check_layout(kv);
  if (rc != TEMPO_OK) return rc;
  if (!q || !out) return TEMPO_ERR_NULL;
  if ((rc = check_heads(kv, batch, num_q_heads)) != TEMPO_OK) return rc;
  if (t < 0 || t > INT32_MAX - 64) return TEMPO_ERR_RANGE;
  // the partials of this call's own plan must fit the static array
  tempo_plan plan;
  make_block_plan(kv, batch, num_q_heads, t, 0, t_per_seq != nullptr, 1, &plan);
  const size_t need = plan_bytes(kv, (int64_t)batch * num_q_heads, plan.num_splits);
  if (need > kScratchBytes) {
    fprintf(stderr, "libtempo: tempo_decode_step_causal_noalloc: this step needs %zu bytes of split partials, "
                    "the static array holds %zu; use tempo_decode_step_causal with a workspace\n", need, kScratchBytes);
    return TEMPO_ERR_WORKSPACE;
  }
  void* ws = nullptr;
  if ((rc = scratch_on_current_device(&ws)) != TEMPO_OK) return rc;
  return decode(kv, q, k_new, v_new, out, batch, num_q_heads, t, t_per_seq, 0, scale, ws, kScratchBytes, stream);
}

// The work list of a ragged step is tied to the plan the step will use: both come from
// make_block_plan with the same arguments.
static int worklist_plan(const tempo_kv* kv, int32_t batch, int32_t Hq, int32_t t_max, int32_t window, tempo_plan* plan) {
  int rc = check_layout(kv);
  if (rc != TEMPO_OK) return rc;
  if ((rc = check_heads(kv, batch, Hq)) != TEMPO_OK) return rc;
  if (t_max < 0 || t_max > INT32_MAX - 64 || window < 0) return TEMPO_ERR_RANGE;
  // the list is read by the single-step bf16 kernel only
  if (kv->dtype != TEMPO_BF16) return TEMPO_ERR_DTYPE;
  if (Hq / kv->num_kv_heads > kNarrowColumns) return TEMPO_ERR_SHAPE;
  make_block_plan(kv, batch, Hq, t_max, window, true, 1, plan);
  if ((int64_t)batch * plan->num_splits > 65535) return TEMPO_ERR_SHAPE;  // one grid row per possible item
  return TEMPO_OK;
}

size_t tempo_attn_worklist_bytes(const tempo_kv* kv, int32_t batch, int32_t num_q_heads, int32_t t_max,
                                 int32_t window) {
  tempo_plan plan;
  if (worklist_plan(kv, batch, num_q_heads, t_max, window, &plan) != TEMPO_OK) return 0;
  return align_up(sizeof(int32_t) * (1 + (size_t)batch * plan.num_splits), 256);
}

int tempo_attn_worklist_build(const tempo_kv* kv, int32_t batch, int32_t num_q_heads, int32_t t_max,
                              const int32_t* t_per_seq, int32_t window, void* worklist, size_t worklist_bytes,
                              void* stream) {
  tempo_plan plan;
  const int rc = worklist_plan(kv, batch, num_q_heads, t_max, window, &plan);
  if (rc != TEMPO_OK) return rc;
  if (!t_per_seq || !worklist) return TEMPO_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(worklist) & 3u) != 0) return TEMPO_ERR_WORKSPACE;
  if (worklist_bytes < sizeof(int32_t) * (1 + (size_t)batch * plan.num_splits)) return TEMPO_ERR_WORKSPACE;
  const hipError_t e = launch_worklist_build(t_per_seq, batch, t_max, window, ilog2_exact(plan.tokens_per_split),
                                             plan.num_splits, static_cast<int32_t*>(worklist),
                                             static_cast<hipStream_t>(stream));
  return launch_status(e, "worklist_build");
}

int tempo_decode_step_ragged(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new, void* out,
                             int32_t batch, int32_t num_q_heads, int32_t t_max, const int32_t* t_per_seq,
                             int32_t window, float scale, const void* worklist, void* workspace,
                             size_t workspace_bytes, void* stream) {
  if (!t_per_seq || !worklist) return TEMPO_ERR_NULL;
  if ((k_new == nullptr) != (v_new == nullptr)) return TEMPO_ERR_NULL;
  tempo_plan plan;
  const int rc = worklist_plan(kv, batch, num_q_heads, t_max, window, &plan);
  if (rc != TEMPO_OK) return rc;
  return decode(kv, q, k_new, v_new, out, batch, num_q_heads, t_max, t_per_seq, window, scale, workspace,
                workspace_bytes, stream, 1, nullptr, 0, static_cast<const int32_t*>(worklist));
}

int tempo_attn_decode_padded_causal(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                                    int32_t num_q_heads, int32_t t, const int32_t* t_per_seq,
                                    int32_t t_pad, float scale, void* workspace, size_t workspace_bytes,
                                    void* stream) {
  if (kv && kv->dtype == TEMPO_F32) return TEMPO_ERR_DTYPE;  // the baseline exists for the bf16 kernel only
  // ... and in the single-step kernel only: the LDS-staged kernel that serves larger query
  // groups walks the step's own range and knows no padding bound
  if (kv && kv->num_kv_heads > 0 && num_q_heads / kv->num_kv_heads > kNarrowColumns) return TEMPO_ERR_SHAPE;
  if (t_pad < t) return TEMPO_ERR_RANGE;
  return decode(kv, q, nullptr, nullptr, out, batch, num_q_heads, t, t_per_seq, 0, scale, workspace,
                workspace_bytes, stream, 1, nullptr, t_pad);
}

int tempo_rope_rotate(const tempo_rope* rope, const void* x, void* y, int32_t dtype, int32_t batch,
                      int32_t heads, int32_t t, const int32_t* t_per_seq, void* stream) {
  if (!rope || !x || !y) return TEMPO_ERR_NULL;
  if (dtype != TEMPO_BF16 && dtype != TEMPO_F32) return TEMPO_ERR_DTYPE;
  if (rope->head_dim < 2 || rope->head_dim % 2 != 0 || rope->head_dim > 65536) return TEMPO_ERR_SHAPE;
  if (batch < 1 || heads < 1 || (int64_t)batch * heads * rope->head_dim > INT32_MAX) return TEMPO_ERR_SHAPE;
  const int rc = check_rope(rope, rope->head_dim, t);
  if (rc != TEMPO_OK) return rc;
  const hipError_t e = launch_rope_rotate(rope->cos, rope->sin, x, y, dtype, batch, heads, rope->head_dim, t,
                                          t_per_seq, static_cast<hipStream_t>(stream));
  return launch_status(e, "rope_rotate");
}

int tempo_rope_kv_append(const tempo_kv* kv, const tempo_rope* rope, const void* k_raw, const void* v_new,
                         int32_t batch, int32_t t, const int32_t* t_per_seq, void* stream) {
  int rc = check_store(kv);
  if (rc != TEMPO_OK) return rc;
  if (!k_raw || !v_new) return TEMPO_ERR_NULL;
  if (batch < 1 || batch > 65535) return TEMPO_ERR_SHAPE;
  if ((rc = check_step(kv, t)) != TEMPO_OK) return rc;
  if ((rc = check_rope(rope, kv->head_dim, t)) != TEMPO_OK) return rc;
  if ((int64_t)batch * kv->num_kv_heads * kv->head_dim > INT32_MAX) return TEMPO_ERR_SHAPE;
  const StoreParams p = store_params(kv, batch, t, t_per_seq);
  const hipError_t e = launch_rope_append(p, rope->cos, rope->sin, k_raw, v_new, kv->head_dim, kv->dtype,
                                          static_cast<hipStream_t>(stream));
  return launch_status(e, "kv_rope_append");
}

int tempo_rope_decode_step_causal(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw,
                                  const void* k_raw, const void* v_new, void* out, int32_t batch,
                                  int32_t num_q_heads, int32_t t, const int32_t* t_per_seq, float scale,
                                  void* workspace, size_t workspace_bytes, void* stream) {
  if (!rope || !k_raw || !v_new) return TEMPO_ERR_NULL;
  return decode(kv, q_raw, k_raw, v_new, out, batch, num_q_heads, t, t_per_seq, 0, scale, workspace,
                workspace_bytes, stream, 1, rope);
}

int tempo_rope_decode_step_window(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw,
                                  const void* k_raw, const void* v_new, void* out, int32_t batch,
                                  int32_t num_q_heads, int32_t t, const int32_t* t_per_seq,
                                  int32_t window, float scale, void* workspace, size_t workspace_bytes,
                                  void* stream) {
  if (!rope || !k_raw || !v_new) return TEMPO_ERR_NULL;
  if (window < 1) return TEMPO_ERR_RANGE;
  return decode(kv, q_raw, k_raw, v_new, out, batch, num_q_heads, t, t_per_seq, window, scale, workspace,
                workspace_bytes, stream, 1, rope);
}

// Does a prompt of `count` steps go through the prompt kernel (one launch after the
// block-store write) rather than block by block?  It does when its query blocks fill
// the part; a ring store and fp32 always go block by block.
bool prefill_in_one_launch(const tempo_kv* kv, int32_t batch, int32_t Hq, int32_t count) {
  if (kv->dtype != TEMPO_BF16 || kv->ring_blocks != 0) return false;
  if ((int64_t)batch * count * kv->num_kv_heads * kv->head_dim > INT32_MAX) return false;
  const int32_t qb = prefill_bf16_block_steps(Hq / kv->num_kv_heads);
  return (int64_t)((count + qb - 1) / qb) * kv->num_kv_heads * batch >= kComputeUnits;
}

// Prompt processing: `count` steps per sequence, written and answered in blocks of
// as many steps as the column tiles hold.
static int prefill(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new, void* out, int32_t batch,
            int32_t Hq, int32_t t, int32_t count, const int32_t* count_per_seq, int32_t window, float scale,
            void* workspace, size_t workspace_bytes, void* stream, const tempo_rope* rope = nullptr) {
  int rc = check_store(kv);
  if (rc != TEMPO_OK) return rc;
  if (!q || !k_new || !v_new || !out) return TEMPO_ERR_NULL;
  if ((rc = check_heads(kv, batch, Hq)) != TEMPO_OK) return rc;
  if (count < 1 || count > (1 << 24)) return TEMPO_ERR_SHAPE;
  if (t < 0 || window < 0 || t > INT32_MAX - 64 - count) return TEMPO_ERR_RANGE;
  if ((rc = check_scale(scale)) != TEMPO_OK) return rc;
  if ((rc = check_step(kv, t + count - 1)) != TEMPO_OK) return rc;
  const int G = Hq / kv->num_kv_heads;
  const int32_t block = kMaxColumns / G;  // steps per block: all four column tiles
  if ((int64_t)batch * block * Hq * kv->head_dim > INT32_MAX) return TEMPO_ERR_SHAPE;
  const size_t esz = kv->dtype == TEMPO_BF16 ? 2 : 4;
  const bool ragged = false;  // every sequence starts at step t
  const int32_t* t_per_seq = nullptr;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // validate every block before the first launch, so that an error leaves the store untouched
  for (int32_t c0 = 0; c0 < count; c0 += block) {
    const int32_t C = count - c0 < block ? count - c0 : block;
    tempo_plan plan;
    make_block_plan(kv, batch, Hq, t + c0, window, ragged, C, &plan);
    if ((rc = check_attn(kv, batch, Hq, t + c0, window, ragged, &plan, workspace, workspace_bytes, C)) != TEMPO_OK)
      return rc;
    if (kv->ring_blocks && (int64_t)C > (int64_t)kv->ring_blocks * kv->block_size) return TEMPO_ERR_RANGE;
  }

  // Enough query blocks to fill the part: write the whole prompt, then one launch of
  // the prompt kernel (each workgroup walks its block's whole key range; no partials).
  // per-sequence prompt lengths and the rotary producer exist in the prompt kernel only
  if ((count_per_seq || rope) && (kv->dtype != TEMPO_BF16 || kv->ring_blocks != 0 ||
                                  (int64_t)batch * count * kv->num_kv_heads * kv->head_dim > INT32_MAX))
    return TEMPO_ERR_SHAPE;
  if (rope && (rc = check_rope(rope, kv->head_dim, t + count - 1)) != TEMPO_OK) return rc;
  if (count_per_seq || rope || prefill_in_one_launch(kv, batch, Hq, count)) {
    StoreParams sp = store_params(kv, batch, t, nullptr, count);
    sp.count_per_seq = count_per_seq;
    if (rope) {
      sp.rope_cos = rope->cos;
      sp.rope_sin = rope->sin;
    }
    if ((rc = launch_status(launch_append(sp, k_new, v_new, kv->head_dim, kv->dtype, s), "kv_append_block")) != TEMPO_OK)
      return rc;
    const tempo_plan whole = {1 << 30, 1, 8};  // no split of the key range: every workgroup walks its block's own
    AttnParams p = attn_params(kv, q, out, Hq, t, nullptr, window, scale, &whole, workspace, batch, count);
    p.direct = 1;
    p.count_per_seq = count_per_seq;
    if (rope) {
      p.rope_cos = rope->cos;
      p.rope_sin = rope->sin;
    }
    return launch_status(launch_prefill_bf16(p, batch, kv->head_dim, 1, s), "attn_prefill");
  }

  // Otherwise block by block: split-KV partial attention keeps the part busy when the
  // blocks are few and the history is long.
  for (int32_t c0 = 0; c0 < count; c0 += block) {
    const int32_t C = count - c0 < block ? count - c0 : block;
    tempo_plan plan;
    make_block_plan(kv, batch, Hq, t + c0, window, ragged, C, &plan);
    const char* kc = static_cast<const char*>(k_new) + (size_t)c0 * kv->num_kv_heads * kv->head_dim * esz;
    const char* vc = static_cast<const char*>(v_new) + (size_t)c0 * kv->num_kv_heads * kv->head_dim * esz;
    const char* qc = static_cast<const char*>(q) + (size_t)c0 * Hq * kv->head_dim * esz;
    char* oc = static_cast<char*>(out) + (size_t)c0 * Hq * kv->head_dim * esz;
    StoreParams sp = store_params(kv, batch, t + c0, t_per_seq, C);
    sp.src_steps = count;
    hipError_t e = launch_append(sp, kc, vc, kv->head_dim, kv->dtype, s);
    if ((rc = launch_status(e, "kv_append_block")) != TEMPO_OK) return rc;
    rc = do_partial(kv, qc, nullptr, nullptr, oc, batch, Hq, t + c0, t_per_seq, window, scale, &plan, workspace, s,
                    C, nullptr, 0, count);
    if (rc != TEMPO_OK) return rc;
    if (plan.num_splits > 1) {
      rc = do_combine(kv, oc, batch, Hq, t + c0, t_per_seq, window, &plan, workspace, s, C, 0, count);
      if (rc != TEMPO_OK) return rc;
    }
  }
  return TEMPO_OK;
}

int tempo_prefill_causal(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new, void* out,
                         int32_t batch, int32_t num_q_heads, int32_t t, int32_t count,
                         const int32_t* count_per_seq, float scale, void* workspace, size_t workspace_bytes,
                         void* stream) {
  return prefill(kv, q, k_new, v_new, out, batch, num_q_heads, t, count, count_per_seq, 0, scale, workspace,
                 workspace_bytes, stream);
}

int tempo_prefill_window(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new, void* out,
                         int32_t batch, int32_t num_q_heads, int32_t t, int32_t count,
                         const int32_t* count_per_seq, int32_t window, float scale, void* workspace,
                         size_t workspace_bytes, void* stream) {
  if (window < 1 || window > INT32_MAX - 128) return TEMPO_ERR_RANGE;
  return prefill(kv, q, k_new, v_new, out, batch, num_q_heads, t, count, count_per_seq, window, scale, workspace,
                 workspace_bytes, stream);
}

int tempo_rope_prefill_causal(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw, const void* k_raw,
                              const void* v_new, void* out, int32_t batch, int32_t num_q_heads, int32_t t,
                              int32_t count, const int32_t* count_per_seq, float scale, void* workspace,
                              size_t workspace_bytes, void* stream) {
  if (!rope) return TEMPO_ERR_NULL;
  return prefill(kv, q_raw, k_raw, v_new, out, batch, num_q_heads, t, count, count_per_seq, 0, scale, workspace,
                 workspace_bytes, stream, rope);
}

int tempo_rope_prefill_window(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw, const void* k_raw,
                              const void* v_new, void* out, int32_t batch, int32_t num_q_heads, int32_t t,
                              int32_t count, const int32_t* count_per_seq, int32_t window, float scale,
                              void* workspace, size_t workspace_bytes, void* stream) {
  if (!rope) return TEMPO_ERR_NULL;
  if (window < 1 || window > INT32_MAX - 128) return TEMPO_ERR_RANGE;
  return prefill(kv, q_raw, k_raw, v_new, out, batch, num_q_heads, t, count, count_per_seq, window, scale,
                 workspace, workspace_bytes, stream, rope);
}

int tempo_prefill_launches(const tempo_kv* kv, int32_t batch, int32_t num_q_heads, int32_t count) {
  if (check_layout(kv) != TEMPO_OK || check_heads(kv, batch, num_q_heads) != TEMPO_OK || count < 1) return 0;
  if (prefill_in_one_launch(kv, batch, num_q_heads, count)) return 2;
  const int32_t block = kMaxColumns / (num_q_heads / kv->num_kv_heads);
  return 3 * ((count + block - 1) / block);
}

size_t tempo_prefill_workspace_bytes(const tempo_kv* kv, int32_t batch, int32_t num_q_heads, int32_t max_t) {
  if (check_layout(kv) != TEMPO_OK || check_heads(kv, batch, num_q_heads) != TEMPO_OK) return 0;
  const int32_t block = kMaxColumns / (num_q_heads / kv->num_kv_heads);
  return tempo_attn_block_workspace_bytes(kv, batch, num_q_heads, block, max_t);
}

int tempo_attn_block_with_plan(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                               int32_t num_q_heads, int32_t queries, int32_t t, const int32_t* t_per_seq,
                               int32_t window, float scale, const tempo_plan* plan, void* workspace,
                               size_t workspace_bytes, void* stream) {
  int rc = check_layout(kv);
  if (rc != TEMPO_OK) return rc;
  if (!q || !out || !plan) return TEMPO_ERR_NULL;
  if ((rc = check_scale(scale)) != TEMPO_OK) return rc;
  if ((rc = check_attn(kv, batch, num_q_heads, t, window, t_per_seq != nullptr, plan, workspace, workspace_bytes,
                       queries)) != TEMPO_OK)
    return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  rc = do_partial(kv, q, nullptr, nullptr, out, batch, num_q_heads, t, t_per_seq, window, scale, plan, workspace, s,
                  queries);
  if (rc != TEMPO_OK || plan->num_splits == 1) return rc;
  return do_combine(kv, out, batch, num_q_heads, t, t_per_seq, window, plan, workspace, s, queries);
}

int tempo_attn_block_causal(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                            int32_t num_q_heads, int32_t queries, int32_t t, const int32_t* t_per_seq,
                            float scale, void* workspace, size_t workspace_bytes, void* stream) {
  return decode(kv, q, nullptr, nullptr, out, batch, num_q_heads, t, t_per_seq, 0, scale, workspace,
                workspace_bytes, stream, queries);
}

int tempo_attn_block_window(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                            int32_t num_q_heads, int32_t queries, int32_t t, const int32_t* t_per_seq,
                            int32_t window, float scale, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (window < 1 || window > INT32_MAX - 64) return TEMPO_ERR_RANGE;
  return decode(kv, q, nullptr, nullptr, out, batch, num_q_heads, t, t_per_seq, window, scale, workspace,
                workspace_bytes, stream, queries);
}

int tempo_rope_attn_block_causal(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw, void* out,
                                 int32_t batch, int32_t num_q_heads, int32_t queries, int32_t t,
                                 const int32_t* t_per_seq, float scale, void* workspace, size_t workspace_bytes,
                                 void* stream) {
  if (!rope) return TEMPO_ERR_NULL;
  return decode(kv, q_raw, nullptr, nullptr, out, batch, num_q_heads, t, t_per_seq, 0, scale, workspace,
                workspace_bytes, stream, queries, rope);
}

int tempo_rope_attn_block_window(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw, void* out,
                                 int32_t batch, int32_t num_q_heads, int32_t queries, int32_t t,
                                 const int32_t* t_per_seq, int32_t window, float scale, void* workspace,
                                 size_t workspace_bytes, void* stream) {
  if (!rope) return TEMPO_ERR_NULL;
  if (window < 1 || window > INT32_MAX - 64) return TEMPO_ERR_RANGE;
  return decode(kv, q_raw, nullptr, nullptr, out, batch, num_q_heads, t, t_per_seq, window, scale, workspace,
                workspace_bytes, stream, queries, rope);
}

int tempo_attn_decode_partial(const tempo_kv* kv, const void* q, const void* k_new,
                              const void* v_new, int32_t batch, int32_t num_q_heads, int32_t t,
                              const int32_t* t_per_seq, int32_t window, float scale,
                              const tempo_plan* plan, void* workspace, size_t workspace_bytes,
                              void* stream) {
  int rc = check_layout(kv);
  if (rc != TEMPO_OK) return rc;
  if (!q || ((k_new == nullptr) != (v_new == nullptr))) return TEMPO_ERR_NULL;
  if ((rc = check_scale(scale)) != TEMPO_OK) return rc;
  if ((rc = check_attn(kv, batch, num_q_heads, t, window, t_per_seq != nullptr, plan, workspace, workspace_bytes)) != TEMPO_OK) return rc;
  // the kernel that serves a group of more than 16 heads does not write the store
  if (k_new && kv->dtype == TEMPO_BF16 && num_q_heads / kv->num_kv_heads > kNarrowColumns) return TEMPO_ERR_SHAPE;
  return do_partial(kv, q, k_new, v_new, nullptr, batch, num_q_heads, t, t_per_seq, window, scale, plan,
                    workspace, static_cast<hipStream_t>(stream));
}

int tempo_attn_decode_combine(const tempo_kv* kv, void* out, int32_t batch, int32_t num_q_heads,
                              int32_t t, const int32_t* t_per_seq, int32_t window,
                              const tempo_plan* plan, const void* workspace,
                              size_t workspace_bytes, void* stream) {
  int rc = check_layout(kv);
  if (rc != TEMPO_OK) return rc;
  if (!out) return TEMPO_ERR_NULL;
  if ((rc = check_attn(kv, batch, num_q_heads, t, window, t_per_seq != nullptr, plan, workspace, workspace_bytes)) != TEMPO_OK) return rc;
  return do_combine(kv, out, batch, num_q_heads, t, t_per_seq, window, plan,
                    const_cast<void*>(workspace), static_cast<hipStream_t>(stream));
}

int tempo_discounted_sum(const float* r, float* g, int32_t batch, int32_t T, int32_t n, float gamma, void* stream) {
  if (!r || !g) return TEMPO_ERR_NULL;
  if (batch < 1 || batch > 65535 || T < 1) return TEMPO_ERR_SHAPE;
  if (n < 0 || !(gamma >= -3.0e38f && gamma <= 3.0e38f)) return TEMPO_ERR_RANGE;       // a finite discount
  if (n > discounted_sum_max_window() && n < T) return TEMPO_ERR_RANGE;                 // neither a short window nor the whole future
  if (r == g) return TEMPO_ERR_SHAPE;                                                   // a step reads rewards of later steps
  if ((int64_t)T > INT32_MAX - 4096) return TEMPO_ERR_SHAPE;
  const hipError_t e = launch_discounted_sum(r, g, batch, T, n, gamma, static_cast<hipStream_t>(stream));
  return launch_status(e, "discounted_sum");
}

int tempo_stream_read(const void* src, size_t bytes, void* sink, int32_t workgroups, void* stream) {
  if (!src || !sink) return TEMPO_ERR_NULL;
  if (bytes < 16 || bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(src) & 15u) != 0) return TEMPO_ERR_SHAPE;
  if (workgroups < 1 || workgroups > (1 << 24)) return TEMPO_ERR_SHAPE;
  const hipError_t e = launch_stream_read(src, bytes, sink, workgroups, static_cast<hipStream_t>(stream));
  return launch_status(e, "stream_read");
}

int tempo_stream_copy(const void* src, void* dst, size_t bytes, int32_t workgroups, void* stream) {
  if (!src || !dst) return TEMPO_ERR_NULL;
  if (bytes < 16 || bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(src) & 15u) != 0 ||
      (reinterpret_cast<uintptr_t>(dst) & 15u) != 0)
    return TEMPO_ERR_SHAPE;
  if (workgroups < 1 || workgroups > (1 << 24)) return TEMPO_ERR_SHAPE;
  const hipError_t e = launch_stream_copy(src, dst, bytes, workgroups, static_cast<hipStream_t>(stream));
  return launch_status(e, "stream_copy");
}

}  // extern "C"
