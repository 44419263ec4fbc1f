/*
 * tempo.h -- C ABI of the decode-attention library for MI355X (gfx950).
 *
 * One hot path, from the Tempo paper's dynamic-tensor method: at decode step t
 * the query q_t attends over a key/value tensor whose temporal extent depends
 * on t (Section 2, Eq. 1):
 *
 *     a_t = softmax(q_t . k_phi(t)^T * s) . v_phi(t)
 *     causal:  phi(t) = 0 : t+1                 keys 0..t, key t included
 *     window:  phi(t) = max(t-w', 0) : t+1      a backward window
 *
 * Keys and values are kept as temporal tiles of a static size Z (Section 4.3,
 * "static tiling": ceil((t+1)/Z) tiles, tile n = keys [nZ, min((n+1)Z, t+1)),
 * the unfilled tail of the last tile masked), held in pre-allocated blocks that
 * are written in place one timestep at a time (Section 6, "block store" and the
 * "in-place writes" kernel wrapper).  A block table maps a sequence's logical
 * tile n to a physical block of a shared pool.
 *
 * Conventions
 *  - `window` is the NUMBER OF VISIBLE KEYS: lo = max(0, t-window+1), hi = t.
 *    The paper's slice with window size w' is window = w'+1.
 *  - Grouped-query attention: query head h reads key/value head
 *    h div (num_q_heads / num_kv_heads).
 *  - Order: step t's key/value must be appended before step t attends.
 *  - Pointers marked "device" are HIP device pointers; `stream` is a
 *    hipStream_t passed as void* (NULL = the default stream).  Everything else
 *    is host memory.  The caller owns every buffer.  The library allocates
 *    nothing, never synchronises, keeps no state between calls (one exception:
 *    tempo_decode_step_causal_noalloc, see there), and every launch is
 *    asynchronous on `stream`; calls may be captured in a HIP graph.
 *  - `out` must not alias q, the pools or the workspace.
 *  - Results are deterministic: same inputs and same arguments, same bits.
 *  - Every entry point validates its arguments on the host and returns a
 *    negative tempo_status before launching anything if they are bad.  Block
 *    ids read from the table on the device are clamped into [0, num_blocks),
 *    so a corrupt table gives wrong numbers, not a memory fault.
 *  - The result never depends on pool contents outside the visible range:
 *    masking is by index (the paper's -inf mask under max, 0 mask under sums).
 *
 * Supported shapes: head_dim in {64, 128}; block_size a power of two, >= 32
 * for bf16 and >= 4 for f32; num_q_heads a multiple of num_kv_heads with a
 * group of at most 128 query heads per key/value head (bf16: a group of up to
 * 16 heads is served by the single-step kernel, which can write the step's
 * key/value itself; a larger group by the LDS-staged kernel of the block entry
 * points, with the store written by a launch of its own first).
 */
#ifndef TEMPO_H
#define TEMPO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { TEMPO_BF16 = 0, TEMPO_F32 = 1 } tempo_dtype;

typedef enum {
  TEMPO_OK = 0,
  TEMPO_ERR_NULL = -1,      /* a required pointer is NULL */
  TEMPO_ERR_SHAPE = -2,     /* unsupported head_dim / block_size / head counts / batch */
  TEMPO_ERR_RANGE = -3,     /* t < 0, window < 1, step t does not fit max_blocks_per_seq, or a
                               ring store no longer holds the visible range */
  TEMPO_ERR_WORKSPACE = -4, /* workspace NULL, misaligned or too small */
  TEMPO_ERR_DTYPE = -5,     /* dtype is not a tempo_dtype */
  TEMPO_ERR_LAUNCH = -6     /* the HIP runtime refused a launch */
} tempo_status;

/*
 * The block store.  k_pool and v_pool each hold
 * num_blocks * num_kv_heads * block_size * head_dim elements of `dtype`.
 * Within the pool, the elements of one (block, kv head) pair are contiguous
 * (block_size*head_dim of them); their order inside that tile depends on dtype
 * and is defined by tempo_kv_element_offset():
 *
 *   TEMPO_F32   row-major [slot][d].
 *   TEMPO_BF16  "operand-major": the tile is cut into groups of 32 consecutive
 *               slots, and inside a group the 16-byte units are ordered so that
 *               a 64-lane wavefront loading consecutive units receives exactly
 *               the register image of a 16x16x32 bf16 MFMA operand (K: 16 slots
 *               x 32 dims per unit group; V: 32 slots x 16 dims).  A decode step
 *               therefore streams K and V with contiguous 1 KiB loads and no
 *               transposition; the price is paid once per token at append time.
 *
 * The pools are opaque to the caller: write them with tempo_kv_append, read
 * them back with tempo_kv_gather.  Slots that were never appended may hold
 * anything (NaN included).
 */
typedef struct tempo_kv {
  void* k_pool;               /* device */
  void* v_pool;               /* device */
  const int32_t* block_table; /* device; [batch][max_blocks_per_seq]; tile n -> physical block */
  int32_t num_blocks;
  int32_t max_blocks_per_seq;
  int32_t block_size;         /* Z, the static tile size of Section 4.3 */
  int32_t num_kv_heads;       /* Hkv */
  int32_t head_dim;           /* D */
  int32_t dtype;              /* tempo_dtype of pools, q, k_new, v_new and out */
  int32_t ring_blocks;        /* 0: linear store, tile n -> block_table[b][n].
                                 R > 0 (a power of two, <= max_blocks_per_seq): window store,
                                 tile n -> block_table[b][n mod R]; see below */
} tempo_kv;

/*
 * Window store (Section 6: a window-accessed tensor lives in a pre-allocated
 * circular buffer, so windowed decode runs in constant memory for any number of
 * steps).  With ring_blocks = R a sequence owns R blocks that are reused in turn:
 * step t is written to block_table[b][(t div Z) mod R], over the block that held
 * steps t-R*Z.. .  No mirrored second write is needed: reads are per tile with index
 * masks, never one contiguous slice.  A ring answers a step only if every tile of
 * its visible range is still resident: windowed attention needs
 * ceil((window-1)/Z)+1 <= R, causal attention needs (t div Z)+1 <= R; otherwise the
 * attention entry points return TEMPO_ERR_RANGE.  tempo_kv_gather on a ring returns
 * whatever the addressed slots hold now.
 */

/* How a step's visible range is cut into independent partial-attention work
 * items ("splits"), each a run of tokens_per_split consecutive key positions
 * aligned to a multiple of tokens_per_split; one workgroup of `waves` 64-lane
 * wavefronts handles the query group of one (sequence, kv head, split). */
typedef struct tempo_plan {
  int32_t tokens_per_split;   /* power of two, >= 32 */
  int32_t num_splits;         /* splits launched per (sequence, kv head) for the longest range */
  int32_t waves;              /* 1, 2, 4 or 8 */
} tempo_plan;

/* ---- pure host functions (no GPU needed) -------------------------------- */

/*
 * Integer quantities of step t (Section 2 patterns, Section 4.3 tiles).
 * window = 0 selects the causal pattern.  Writes: lo, hi (first/last visible
 * key, hi = t); first_tile = lo div Z and last_tile = t div Z; first_tile_skip
 * = keys of first_tile before lo; last_tile_valid = (t mod Z)+1 keys of the
 * last tile that exist (the rest is the padding Section 4.3 masks).  Any output
 * pointer may be NULL.  Returns TEMPO_ERR_RANGE for t < 0, window < 0, Z < 1.
 */
int tempo_visible_range(int32_t t, int32_t window, int32_t Z, int32_t* lo, int32_t* hi,
                        int32_t* first_tile, int32_t* last_tile, int32_t* first_tile_skip,
                        int32_t* last_tile_valid);

/* Where step t is written (block store, Section 6): tile = t div Z, slot = t mod Z. */
int tempo_append_slot(int32_t t, int32_t Z, int32_t* tile, int32_t* slot);

/*
 * Which stored steps may be released once step t has been answered (Section 5.2,
 * scheduling deallocations: what a step produced is released after the last step
 * that reads it, found from the inverse of the consumer's dependence).  With a
 * window of `window` visible keys, key j is read by steps j .. j+window-1, so after
 * step t the keys 0 .. t-window+1 are dead.  Writes: dead_keys = their number
 * (clamped to [0, t+1]), dead_tiles = dead_keys div Z = the leading blocks of a
 * linear store that no later step reads and the caller may hand to another
 * sequence.  window = 0 (causal): nothing is ever dead, both are 0.  Either
 * pointer may be NULL.  Pure host function; TEMPO_ERR_RANGE for t < 0, t = INT32_MAX,
 * window < 0, Z < 1.
 */
int tempo_kv_release(int32_t t, int32_t window, int32_t Z, int32_t* dead_keys, int32_t* dead_tiles);

/*
 * Size of a window store (Section 6: a window-accessed tensor lives in a
 * pre-allocated circular buffer sized by the window): the smallest ring_blocks (a
 * power of two) with which calls that answer `queries` consecutive steps with this
 * window always find their visible range resident, wherever the steps fall
 * relative to the tile boundaries: floor((window + queries - 3) / Z) + 2 tiles
 * (1 if window + queries = 2), rounded up to a power of two.  Pure host function;
 * TEMPO_ERR_RANGE for window < 1, Z < 1, queries < 1 or a result beyond 2^30;
 * ring_blocks must not be NULL.
 */
int tempo_ring_blocks(int32_t window, int32_t Z, int32_t queries, int32_t* ring_blocks);

/*
 * Element offset, from the start of k_pool (which = 0) or v_pool (which = 1),
 * of dimension d of slot `slot` of kv head `head` of physical block `block`.
 * Only the layout fields of kv are read.  Returns -1 for arguments out of range.
 */
int64_t tempo_kv_element_offset(const tempo_kv* kv, int32_t which, int32_t block, int32_t head,
                                int32_t slot, int32_t d);

/* Bytes of one pool (k_pool or v_pool); 0 if the layout fields are invalid. */
size_t tempo_kv_pool_bytes(const tempo_kv* kv);

/*
 * The split plan the attention entry points use for a batch whose longest
 * step is t_max (window = 0: causal; ragged != 0: the plan used when t_per_seq
 * is given).  Deterministic function of its arguments.
 */
int tempo_attn_plan(const tempo_kv* kv, int32_t batch, int32_t num_q_heads, int32_t t_max,
                    int32_t window, int32_t ragged, tempo_plan* plan);

/*
 * Workspace bytes that tempo_attn_decode_causal / _window need for any step
 * t <= max_t of `batch` sequences (partials: running max, running sum and
 * fp32 accumulator per (sequence, query head, split)).  0 on invalid arguments.
 */
size_t tempo_attn_workspace_bytes(const tempo_kv* kv, int32_t batch, int32_t num_q_heads,
                                  int32_t max_t);

const char* tempo_strerror(int status);

/* ---- device entry points ------------------------------------------------ */

/*
 * Block-store write of one timestep (Section 6): k_new, v_new (device,
 * [batch][Hkv][D] of dtype) go to physical block block_table[b][t div Z], slot
 * t mod Z.  If t_per_seq (device, [batch]) is not NULL each sequence b is
 * written at its own step t_per_seq[b], and t must be an upper bound of those
 * steps (it is only used for validation).
 */
int tempo_kv_append(const tempo_kv* kv, const void* k_new, const void* v_new, int32_t batch,
                    int32_t t, const int32_t* t_per_seq, void* stream);

/*
 * Read keys/values of steps j0 .. j0+count-1 of every sequence back out of the
 * block store into flat arrays k_out, v_out (device, [batch][count][Hkv][D] of
 * dtype; either may be NULL).  The "slice read" of the block store; used by
 * tests and for inspection, not by the decode path.
 */
int tempo_kv_gather(const tempo_kv* kv, void* k_out, void* v_out, int32_t batch, int32_t j0,
                    int32_t count, void* stream);

/*
 * Eq. 1 with the causal pattern: out[b][h][:] (device, [batch][Hq][D] of dtype)
 * = attention of q[b][h][:] (device, same shape) over keys/values 0..t of
 * sequence b.  If t_per_seq (device, [batch]) is not NULL, sequence b is at step
 * t_per_seq[b] and t must be an upper bound of those steps (it fixes the launch
 * geometry).  scale is the constant s of Eq. 1, finite and > 0 (TEMPO_ERR_RANGE
 * otherwise, in every entry point that takes it).  workspace: device, 256-byte
 * aligned, at least tempo_attn_workspace_bytes(kv, batch, num_q_heads, t) bytes;
 * its contents need no initialisation and one workspace serves one call at a
 * time.  Launches: partial attention per split, then the split combine (a step
 * that fits one split writes out directly and launches nothing else).
 */
int tempo_attn_decode_causal(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                             int32_t num_q_heads, int32_t t, const int32_t* t_per_seq,
                             float scale, void* workspace, size_t workspace_bytes, void* stream);

/* Same with the window pattern: keys max(0, t-window+1) .. t; window >= 1. */
int tempo_attn_decode_window(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                             int32_t num_q_heads, int32_t t, const int32_t* t_per_seq,
                             int32_t window, float scale, void* workspace,
                             size_t workspace_bytes, void* stream);

/*
 * One decode step with one launch fewer: tempo_kv_append(k_new, v_new at step t)
 * followed by tempo_attn_decode_causal / _window at step t, with the same
 * arguments and the same results as those two calls.  The block-store write is
 * done by the attention kernel itself (the paper's "in-place writes" wrapper,
 * Section 6, applied to the consumer): the workgroup that owns step t's slot
 * stores k_new / v_new there and attends over them from registers.
 */
int tempo_decode_step_causal(const tempo_kv* kv, const void* q, const void* k_new,
                             const void* v_new, void* out, int32_t batch, int32_t num_q_heads,
                             int32_t t, const int32_t* t_per_seq, float scale, void* workspace,
                             size_t workspace_bytes, void* stream);

int tempo_decode_step_window(const tempo_kv* kv, const void* q, const void* k_new,
                             const void* v_new, void* out, int32_t batch, int32_t num_q_heads,
                             int32_t t, const int32_t* t_per_seq, int32_t window, float scale,
                             void* workspace, size_t workspace_bytes, void* stream);

/*
 * Ragged decode steps with a work list.  Static tiling (Section 4.3) trades a dynamic range
 * for a dynamic NUMBER of static tiles; when every sequence of a batch is at its own step
 * (t_per_seq), that number differs per sequence.  tempo_decode_step_causal / _window then
 * launch a dense grid over (sequence, largest split count) whose surplus workgroups exit at
 * once.  The work list names only the (sequence, split) items that exist, longest first (all
 * full splits, then each sequence's newest split by size), so the launch holds no empty
 * workgroups and ends on its smallest items.  The list depends on the steps only, not on the
 * pools or the block table: build it once per decode step and pass it to every layer's call.
 *
 * tempo_attn_worklist_bytes   bytes of a list for steps up to t_max (host only; 0 on
 *                             unsupported arguments).
 * tempo_attn_worklist_build   one small launch that writes the list (device, 4-byte aligned,
 *                             at least tempo_attn_worklist_bytes bytes) from t_per_seq (device,
 *                             [batch]; each clamped to [0, t_max]).  window = 0: causal.
 * tempo_decode_step_ragged    tempo_decode_step_causal (window = 0) or _window at per-sequence
 *                             steps, its partial-attention launch driven by the list; k_new
 *                             and v_new may both be NULL (the store already holds the steps).
 *                             Same results, bit for bit, as the entry points without a list.
 * The list is valid for exactly the batch, head counts, t_max, window and t_per_seq VALUES it
 * was built from; a stale list gives wrong results (never a fault: an item outside a
 * sequence's range is skipped).  bf16 stores with at most 16 query heads per key/value head
 * (TEMPO_ERR_DTYPE / TEMPO_ERR_SHAPE otherwise), batch * splits <= 65535 (TEMPO_ERR_SHAPE).
 */
size_t tempo_attn_worklist_bytes(const tempo_kv* kv, int32_t batch, int32_t num_q_heads,
                                 int32_t t_max, int32_t window);

int tempo_attn_worklist_build(const tempo_kv* kv, int32_t batch, int32_t num_q_heads, int32_t t_max,
                              const int32_t* t_per_seq, int32_t window, void* worklist,
                              size_t worklist_bytes, void* stream);

int tempo_decode_step_ragged(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new,
                             void* out, int32_t batch, int32_t num_q_heads, int32_t t_max,
                             const int32_t* t_per_seq, int32_t window, float scale,
                             const void* worklist, void* workspace, size_t workspace_bytes,
                             void* stream);

/*
 * tempo_decode_step_causal for callers that cannot allocate device memory at all, not
 * even a workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, launches and results (bit for bit) as
 * tempo_decode_step_causal, but the split partials live in an 8 MiB array that is part
 * of the library's device code (one copy per GPU, held until the process ends) instead
 * of a caller's workspace.  The call allocates and frees nothing.
 *   - A step whose partials (tempo_attn_plan_workspace_bytes of the plan tempo_attn_plan
 *     returns for it) exceed 8 MiB is refused with TEMPO_ERR_WORKSPACE and a message on
 *     stderr; nothing is launched.  (The headline shape needs 0.4 MiB, a single sequence
 *     at t = 65535 3.2 MiB, a ragged batch of 64 at t <= 8191 6.4 MiB.)
 *   - The device that `stream` belongs to must be the current device.  The first call on
 *     a device looks the array's address up (hipGetSymbolAddress) and keeps it: this is
 *     the one piece of state the library holds.  Make that first call outside stream
 *     capture.
 *   - Every call on a GPU uses that GPU's one array, so calls that overlap in time on one
 *     GPU (different streams, or threads) race; calls on one stream are ordered and safe.
 *     The array's contents need no initialisation and mean nothing between calls.
 */
int tempo_decode_step_causal_noalloc(const tempo_kv* kv, const void* q, const void* k_new,
                                     const void* v_new, void* out, int32_t batch,
                                     int32_t num_q_heads, int32_t t, const int32_t* t_per_seq,
                                     float scale, void* stream);

/*
 * Padded + masked baseline (Section 2.1, workaround (c): pad the dynamic dimension
 * to a static bound and mask; Section 7.2 measures the dynamic formulation against
 * it).  Same result as tempo_attn_decode_causal at step t, but the kernel reads and
 * multiplies keys/values 0 .. t_pad of every sequence and masks those beyond the
 * step by index (their contents never matter).  For measurement: its time is that
 * of step t_pad whatever t is.  bf16 stores only (TEMPO_ERR_DTYPE otherwise) and
 * groups of at most 16 query heads per key/value head (TEMPO_ERR_SHAPE otherwise:
 * the kernel that serves larger groups has no padded form); t <= t_pad, and step
 * t_pad must fit the store (TEMPO_ERR_RANGE).  workspace as for step t_pad.
 */
int tempo_attn_decode_padded_causal(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                                    int32_t num_q_heads, int32_t t, const int32_t* t_per_seq,
                                    int32_t t_pad, float scale, void* workspace,
                                    size_t workspace_bytes, void* stream);

/*
 * Rotary position embedding of the producer step, fused with the block-store
 * write (Section 6, kernel wrappers / "in-place writes": the kernel that produces
 * a value writes it straight to index t of the pre-allocated buffer; here the
 * producer is the position encoding of the Llama decoding workload of Section 7.2,
 * which the paper leaves to the model).  A head vector x at position t becomes
 *     y[i]       = x[i] * cos[t][i] - x[i + D/2] * sin[t][i]
 *     y[i + D/2] = x[i + D/2] * cos[t][i] + x[i] * sin[t][i],     i = 0 .. D/2-1,
 * with the caller's tables (normally cos / sin of t * theta^(-2i/D)).  Arithmetic
 * is fp32; bf16 results are rounded to nearest even once.
 *   cos, sin   device, [positions][head_dim/2] float, 16-byte aligned; read only;
 *              owned by the caller and unchanged
 *   head_dim   must equal the store's head_dim where a store is involved
 * Errors: TEMPO_ERR_NULL (rope or a table is NULL), TEMPO_ERR_SHAPE (head_dim
 * mismatch, misaligned table), TEMPO_ERR_RANGE (a step >= positions).
 */
typedef struct tempo_rope {
  const float* cos;
  const float* sin;
  int32_t positions;
  int32_t head_dim;
} tempo_rope;

/* y = x rotated to position t (t_per_seq[b] if given, t their upper bound).
 * x, y: device, [batch][heads][rope->head_dim] of `dtype`; y may be x. */
int tempo_rope_rotate(const tempo_rope* rope, const void* x, void* y, int32_t dtype, int32_t batch,
                      int32_t heads, int32_t t, const int32_t* t_per_seq, void* stream);

/* tempo_kv_append of (rotate(k_raw, t), v_new): the rotated key is written to its
 * slot directly and never exists as a tensor.  Arguments as tempo_kv_append. */
int tempo_rope_kv_append(const tempo_kv* kv, const tempo_rope* rope, const void* k_raw,
                         const void* v_new, int32_t batch, int32_t t, const int32_t* t_per_seq,
                         void* stream);

/*
 * The whole producer + consumer step in the launches of tempo_decode_step_*:
 * q_raw and k_raw (both unrotated) are turned to position t inside the attention
 * kernel, the rotated key and v_new are written to step t's slot, and the rotated
 * query attends over the visible range.  Same result as tempo_rope_rotate(q),
 * tempo_rope_kv_append, tempo_attn_decode_*, bit for bit in the store.
 * Arguments otherwise as tempo_decode_step_causal / _window.
 */
int tempo_rope_decode_step_causal(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw,
                                  const void* k_raw, const void* v_new, void* out, int32_t batch,
                                  int32_t num_q_heads, int32_t t, const int32_t* t_per_seq,
                                  float scale, void* workspace, size_t workspace_bytes,
                                  void* stream);

int tempo_rope_decode_step_window(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw,
                                  const void* k_raw, const void* v_new, void* out, int32_t batch,
                                  int32_t num_q_heads, int32_t t, const int32_t* t_per_seq,
                                  int32_t window, float scale, void* workspace,
                                  size_t workspace_bytes, void* stream);

/*
 * Block of queries (Section 2: the block access pattern and prompt processing;
 * Section 4.3: a tile of timesteps evaluated together).  `queries` = C consecutive
 * steps t .. t+C-1 of every sequence are answered by one call: query c attends
 * over keys 0 .. t+c (causal) or max(0, t+c-window+1) .. t+c (window), exactly as
 * C single-step calls would, while the keys and values are read once.  The store
 * must already hold keys/values up to step t+C-1 (tempo_kv_append_block).
 *   q, out   device, [batch][queries][num_q_heads][head_dim], kv->dtype
 *   t        first step of the block (uniform), or with t_per_seq the upper bound of
 *            the per-sequence first steps t_per_seq[b]
 * Limits: queries >= 1 and queries * (num_q_heads / num_kv_heads) <= 128
 * (TEMPO_ERR_SHAPE otherwise): up to 16 such (step, head) columns ride in the
 * padding of the single-step kernel's tiles, 17..128 use the LDS-staged kernel
 * (eight wavefronts of 16 columns share one copy of every key/value group).  workspace: device, 256-byte aligned, at least
 * tempo_attn_block_workspace_bytes(kv, batch, num_q_heads, queries, t) bytes.
 * Other arguments, launches and errors as tempo_attn_decode_causal / _window.
 */
int tempo_attn_block_causal(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                            int32_t num_q_heads, int32_t queries, int32_t t,
                            const int32_t* t_per_seq, float scale, void* workspace,
                            size_t workspace_bytes, void* stream);

int tempo_attn_block_window(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                            int32_t num_q_heads, int32_t queries, int32_t t,
                            const int32_t* t_per_seq, int32_t window, float scale, void* workspace,
                            size_t workspace_bytes, void* stream);

/*
 * The block entry points with unrotated queries: query c of sequence b is turned to its
 * own position t + c (t_per_seq[b] + c) when the kernel loads it, with the arithmetic of
 * tempo_rope_rotate (same bits as rotating first).  The store must already hold the
 * rotated keys of steps up to t + queries - 1 (tempo_rope_kv_append_block).  rope as in
 * tempo_rope_decode_step_*; everything else as tempo_attn_block_*.
 */
int tempo_rope_attn_block_causal(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw,
                                 void* out, int32_t batch, int32_t num_q_heads, int32_t queries,
                                 int32_t t, const int32_t* t_per_seq, float scale, void* workspace,
                                 size_t workspace_bytes, void* stream);
int tempo_rope_attn_block_window(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw,
                                 void* out, int32_t batch, int32_t num_q_heads, int32_t queries,
                                 int32_t t, const int32_t* t_per_seq, int32_t window, float scale,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * Prompt processing (Section 2: prompt tokens are processed before decoding
 * starts; Section 4.3: the temporal dimension evaluated in tiles): steps
 * t .. t+count-1 of every sequence in ONE call.  The keys/values of those steps are
 * written to the store and every step's query attends over its own range (keys
 * 0 .. t+c, or its window), exactly as `count` single decode steps would.  Work is
 * issued in blocks of 128 / (num_q_heads / num_kv_heads) steps: per block one
 * tempo_kv_append_block and one tempo_attn_block_* (all launches asynchronous on
 * `stream`, nothing allocated).
 *   q, out        device, [batch][count][num_q_heads][head_dim]
 *   k_new, v_new  device, [batch][count][num_kv_heads][head_dim]
 *   count_per_seq device, int32 [batch], or NULL: sequence b has only count_per_seq[b]
 *                 (0 .. count) prompt steps; its later rows of q / k_new / v_new are not
 *                 read into the store, its later rows of out and its later slots in
 *                 the store are left as they are.  bf16 linear stores only
 *                 (TEMPO_ERR_SHAPE otherwise); always the prompt kernel.
 *   workspace     device, 256-byte aligned, >= tempo_prefill_workspace_bytes(kv, batch,
 *                 num_q_heads, t + count - 1) bytes
 * All arguments are validated for every block before the first launch.
 */
int tempo_prefill_causal(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new,
                         void* out, int32_t batch, int32_t num_q_heads, int32_t t, int32_t count,
                         const int32_t* count_per_seq, float scale, void* workspace,
                         size_t workspace_bytes, void* stream);

int tempo_prefill_window(const tempo_kv* kv, const void* q, const void* k_new, const void* v_new,
                         void* out, int32_t batch, int32_t num_q_heads, int32_t t, int32_t count,
                         const int32_t* count_per_seq, int32_t window, float scale, void* workspace,
                         size_t workspace_bytes, void* stream);

/* tempo_prefill_* with the rotary producer fused in: q_raw and k_raw arrive
 * unrotated; keys are turned to their step's position on the way into the store
 * (the same bits tempo_rope_kv_append stores), queries when the prompt kernel loads
 * them.  bf16 linear stores only (TEMPO_ERR_SHAPE otherwise); always the prompt
 * kernel; rope->positions must exceed t + count - 1.  Other arguments as
 * tempo_prefill_causal / _window. */
int tempo_rope_prefill_causal(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw,
                              const void* k_raw, const void* v_new, void* out, int32_t batch,
                              int32_t num_q_heads, int32_t t, int32_t count,
                              const int32_t* count_per_seq, float scale, void* workspace,
                              size_t workspace_bytes, void* stream);

int tempo_rope_prefill_window(const tempo_kv* kv, const tempo_rope* rope, const void* q_raw,
                              const void* k_raw, const void* v_new, void* out, int32_t batch,
                              int32_t num_q_heads, int32_t t, int32_t count,
                              const int32_t* count_per_seq, int32_t window, float scale,
                              void* workspace, size_t workspace_bytes, void* stream);

/* How many launches a tempo_prefill_* call of `count` steps issues at most (host
 * only; 0 on unsupported arguments): 2 when the prompt's query blocks fill the part
 * (bf16, linear store: one block-store write, then one launch of the prompt kernel,
 * in which every workgroup walks the whole key range of its 128 (step, head)
 * columns through LDS and writes `out` directly), else 3 per block of steps. */
int tempo_prefill_launches(const tempo_kv* kv, int32_t batch, int32_t num_q_heads, int32_t count);

/* Workspace bound for tempo_prefill_* calls whose last step is at most max_t (host only). */
size_t tempo_prefill_workspace_bytes(const tempo_kv* kv, int32_t batch, int32_t num_q_heads,
                                     int32_t max_t);

/* tempo_attn_block_causal (window = 0) or _window with the caller's plan instead of
 * the library's (for sweeping plans).  The plan must cover the union of the block's
 * ranges and satisfy the limits of tempo_attn_block_plan's results (up to 16
 * columns: wave-merge area within 64 KiB of LDS; above: waves is ignored); workspace at
 * least batch * queries * num_q_heads rows of plan->num_splits partials
 * (tempo_attn_plan_workspace_bytes with batch * queries as the batch). */
int tempo_attn_block_with_plan(const tempo_kv* kv, const void* q, void* out, int32_t batch,
                               int32_t num_q_heads, int32_t queries, int32_t t,
                               const int32_t* t_per_seq, int32_t window, float scale,
                               const tempo_plan* plan, void* workspace, size_t workspace_bytes,
                               void* stream);

/* The plan tempo_attn_block_* use for a block whose first step is t_max (host
 * only): tempo_attn_plan for the union of the queries' ranges, with fewer
 * wavefronts where the per-column accumulators would not fit the workgroup's LDS.
 * Its workspace holds batch * queries * num_q_heads rows of num_splits partials. */
int tempo_attn_block_plan(const tempo_kv* kv, int32_t batch, int32_t num_q_heads, int32_t queries,
                          int32_t t_max, int32_t window, int32_t ragged, tempo_plan* plan);

/* Workspace bound for blocks of `queries` steps whose first step is at most max_t
 * (host only; 0 on unsupported arguments). */
size_t tempo_attn_block_workspace_bytes(const tempo_kv* kv, int32_t batch, int32_t num_q_heads,
                                        int32_t queries, int32_t max_t);

/*
 * In-place write of `count` consecutive steps per sequence (Section 6, block
 * store): row c of sequence b goes to step t + c (t_per_seq[b] + c if given, with
 * t their upper bound).  k_new, v_new: device, [batch][count][num_kv_heads][head_dim].
 * A ring store accepts at most ring_blocks * block_size steps per call.  Errors as
 * tempo_kv_append, for every step of the block.
 */
int tempo_kv_append_block(const tempo_kv* kv, const void* k_new, const void* v_new, int32_t batch,
                          int32_t t, const int32_t* t_per_seq, int32_t count, void* stream);

/*
 * The same write with the rotary producer fused in (Section 6, "in-place writes": the
 * kernel that produces the keys writes them into the store): row c of k_raw arrives
 * unrotated and is turned to its own position t + c (t_per_seq[b] + c) on the way in;
 * the store then holds the bits tempo_rope_kv_append would have written step by step.
 * bf16 stores only (TEMPO_ERR_DTYPE otherwise); rope as in tempo_rope_kv_append, its
 * tables must reach position t + count - 1.  Other errors as tempo_kv_append_block.
 */
int tempo_rope_kv_append_block(const tempo_kv* kv, const tempo_rope* rope, const void* k_raw,
                               const void* v_new, int32_t batch, int32_t t, const int32_t* t_per_seq,
                               int32_t count, void* stream);

/*
 * Partial attention and split combine as two separate launches, with an explicit
 * plan (for profiling one kernel at a time and for sweeping plans).  window = 0
 * is causal.  k_new / v_new are both NULL (the pool already holds step t) or both
 * set (step t is appended by this launch, as in tempo_decode_step_*; bf16 groups
 * of more than 16 query heads: TEMPO_ERR_SHAPE, write the store first).
 * tempo_attn_decode_partial writes one (max, sum, accumulator)
 * partial per (sequence, query head, non-empty split) into workspace
 * (Section 4.3: per-tile reductions under -inf / 0 masks);
 * tempo_attn_decode_combine adds the per-tile partial results up into out (the
 * final summation over masked tiles of Section 4.3).  plan->num_splits must cover the range
 * of step t, at least (t div tps) - (lo div tps) + 1 splits, and with t_per_seq
 * the range of any step up to t (what tempo_attn_plan returns).
 */
int tempo_attn_decode_partial(const tempo_kv* kv, const void* q, const void* k_new,
                              const void* v_new, int32_t batch, int32_t num_q_heads, int32_t t,
                              const int32_t* t_per_seq, int32_t window, float scale,
                              const tempo_plan* plan, void* workspace, size_t workspace_bytes,
                              void* stream);

int tempo_attn_decode_combine(const tempo_kv* kv, void* out, int32_t batch, int32_t num_q_heads,
                              int32_t t, const int32_t* t_per_seq, int32_t window,
                              const tempo_plan* plan, const void* workspace,
                              size_t workspace_bytes, void* stream);

/* Workspace bytes for an explicit plan. */
size_t tempo_attn_plan_workspace_bytes(const tempo_kv* kv, int32_t batch, int32_t num_q_heads,
                                       const tempo_plan* plan);

/*
 * Anti-causal window reduction (Section 3, Algorithm 1: the returns of the paper's
 * reinforcement-learning example, `r[t : min(t+n, T)].discounted_sum(gamma)` and
 * `r[t : T].discounted_sum(gamma)`): for every sequence b and step t
 *     g[b][t] = sum_{k=0}^{m-1} gamma^k * r[b][t+k],    m = min(n, T - t),
 * the first reward undiscounted; n = 0 (or any n >= T) means the whole future, m = T - t.
 * The forward counterpart of the attention windows above: a reduction over a range of the
 * temporal dimension whose extent depends on t.
 *   r, g    device, [batch][T] float, row-major; g must not be r (a step reads later rewards)
 *   n       0, or 1 .. 1024, or >= T (TEMPO_ERR_RANGE for a window between 1024 and T)
 *   gamma   any finite value (TEMPO_ERR_RANGE otherwise)
 * One launch: a short window is folded per step from a tile staged in LDS; the whole
 * future is a reverse scan of g[t] = r[t] + gamma g[t+1], O(T) work per sequence.  fp32
 * arithmetic; against exact arithmetic the error of g[b][t] stays within
 * 1e-5 * sum_k |gamma|^k |r[b][t+k]|.
 */
int tempo_discounted_sum(const float* r, float* g, int32_t batch, int32_t T, int32_t n, float gamma,
                         void* stream);

/*
 * Measurement aid, not part of the decode path: read `bytes` (a multiple of 16)
 * of device memory at src (16-byte aligned) once with 16-byte-per-lane loads,
 * using `workgroups` workgroups of 256 threads, and discard the data (sink:
 * device, at least 4 bytes, practically never written).  It is the streaming-read
 * yardstick the decode kernels' key/value bandwidth is compared with, and the kernel of known size that hardware traffic counters are
 * scaled by.
 */
int tempo_stream_read(const void* src, size_t bytes, void* sink, int32_t workgroups, void* stream);

/* The same walk, copying src to dst (both device, 16-byte aligned, `bytes` each):
 * reads `bytes` and writes `bytes`, which is what traffic counters are checked against. */
int tempo_stream_copy(const void* src, void* dst, size_t bytes, int32_t workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TEMPO_H */
