/*
 * CPU oracle for decode attention over a dynamic key/value range.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the GPU library must compute.  It is used by the tests, by the smoke check
 * and by the benchmark's CPU-baseline leg, and by nothing else.  It shares no
 * code, layout, table or helper with the HIP path: keys and values live in
 * flat [B][T][Hkv][D] arrays (no temporal blocks, no block table), every
 * floating-point operation is fp64, and the loops follow the defining
 * equation term by term.
 *
 * What it follows.  The paper's attention equation (Section 2, Eq. 1):
 *     a_t = softmax(q_t . k_phi(t)^T * s) . v_phi(t)
 * with the attention pattern phi(t) (same section):
 *     causal:  phi(t) = 0 : t+1              (step t sees keys 0..t, itself included)
 *     window:  phi(t) = max(t-w', 0) : t+1   (a backward window)
 * Here `window` counts the visible keys, so lo = max(0, t-window+1); the
 * paper's slice with window size w' is window = w'+1.  window = 0 selects the
 * causal pattern.  Static tiling (Section 4.3) is an exact reformulation of
 * the same result, so it does not appear in the attention routine; its integer
 * bookkeeping (tile count ceil((t+1)/Z), tile n = [nZ, min((n+1)Z, t+1)),
 * the padding of the last tile) is restated below with counting loops.
 *
 * Grouped-query attention is not described in the paper; query head h reads
 * key/value head h div (Hq/Hkv) (contiguous groups).
 *
 * Every function here is pinned by tests that do not call it to produce their
 * expected value (closed forms, a brute-force evaluator written differently,
 * the padded+masked formulation, the paper's tiled three-reduction form, the
 * paper's printed inverse-window example; for the rotary embedding: closed
 * forms at chosen angles, norm preservation, the relative-position identity and
 * composition of rotations; for releases and ring sizes: the paper's printed
 * inverse-window example read as "last reader of key j", and closed forms; for the
 * discounted sum: closed forms of constant and impulse rewards, the recurrence between
 * neighbouring steps, a differently written evaluator, the parameters Algorithm 1 prints).
 * Nothing is "parity unpinned".
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Is key j visible to the query of step t?  (Section 2: causal and window
 * patterns; window = number of visible keys, 0 = causal.) */
static int visible(int j, int t, int window) {
  if (j < 0 || j > t) return 0;
  if (window == 0) return 1;
  return (t - j) < window;
}

/*
 * Integer quantities of a step, by counting (Section 2 patterns; Section 4.3
 * tiles of static size Z).  Outputs:
 *   lo, hi            first and last visible key (hi == t)
 *   first_tile        tile holding key lo        (tile of key j is j div Z)
 *   last_tile         tile holding key t
 *   n_tiles           number of tiles that exist at step t = ceil((t+1)/Z)
 *   first_tile_skip   keys of first_tile that lie before lo (masked at the front)
 *   last_tile_valid   keys of last_tile that exist at step t (the rest is padding)
 * Returns 0, or -1 for t < 0, window < 0 or Z < 1.
 */
int tempo_oracle_visible_range(int t, int window, int Z, int* lo, int* hi,
                               int* first_tile, int* last_tile, int* n_tiles,
                               int* first_tile_skip, int* last_tile_valid) {
  if (t < 0 || window < 0 || Z < 1) return -1;
  int first = -1, last = -1;
  for (int j = 0; j <= t; ++j) {
    if (visible(j, t, window)) {
      if (first < 0) first = j;
      last = j;
    }
  }
  /* Walk the keys in order, opening a new tile every Z keys. */
  int tile = 0, slot = 0, tile_of_first = 0, tile_of_last = 0;
  int skipped_in_first = 0, existing_in_last = 0;
  for (int j = 0; j <= t; ++j) {
    if (j == first) tile_of_first = tile;
    if (j == last) tile_of_last = tile;
    if (++slot == Z) { slot = 0; ++tile; }
  }
  tile = 0; slot = 0;
  for (int j = 0; j <= t; ++j) {
    if (tile == tile_of_first && j < first) ++skipped_in_first;
    if (tile == tile_of_last) ++existing_in_last;
    if (++slot == Z) { slot = 0; ++tile; }
  }
  int tiles = 0;
  for (int j = 0; j <= t; j += Z) ++tiles;
  *lo = first; *hi = last;
  *first_tile = tile_of_first; *last_tile = tile_of_last; *n_tiles = tiles;
  *first_tile_skip = skipped_in_first; *last_tile_valid = existing_in_last;
  return 0;
}

/* Number of visible keys of step t that fall in tile n (Section 4.3: tile n
 * spans keys [nZ, min((n+1)Z, t+1)); the window pattern further cuts its front). */
int tempo_oracle_tile_visible_count(int t, int window, int Z, int n) {
  if (t < 0 || window < 0 || Z < 1 || n < 0) return -1;
  int count = 0;
  for (int j = 0; j <= t; ++j) {
    int tile = 0;
    for (int k = Z; k <= j; k += Z) ++tile;
    if (tile == n && visible(j, t, window)) ++count;
  }
  return count;
}

/* Where step t's key/value is written (block store, Section 6: one write per
 * timestep into a pre-allocated block): tile t div Z, slot t mod Z, found by
 * walking. */
int tempo_oracle_append_slot(int t, int Z, int* tile, int* slot) {
  if (t < 0 || Z < 1) return -1;
  int n = 0, s = 0;
  for (int j = 0; j < t; ++j) {
    if (++s == Z) { s = 0; ++n; }
  }
  *tile = n; *slot = s;
  return 0;
}

/*
 * Which stored keys are dead once step t has been answered?  (Section 5.2,
 * scheduling deallocations: what step j produced may be released only after the
 * last step that reads it, which follows from the inverse of the consumer's
 * dependence.)  Key j is dead after step t if none of the later steps sees it;
 * later steps are tried one by one up to the first that cannot see any key <= t.
 *   dead_keys    number of leading dead keys 0 .. dead_keys-1
 *   dead_tiles   number of leading tiles (of Z keys) all of whose keys are dead
 * Causal (window 0): every later step sees every key, nothing is ever dead.
 * Returns 0, or -1 for t < 0, window < 0 or Z < 1.
 */
int tempo_oracle_release(int t, int window, int Z, int* dead_keys, int* dead_tiles) {
  if (t < 0 || window < 0 || Z < 1) return -1;
  int dead = 0;
  for (int j = 0; j <= t; ++j) {
    int seen_later = 0;
    if (window == 0) seen_later = 1;
    for (int later = t + 1; !seen_later && later <= t + window; ++later) {
      if (visible(j, later, window)) seen_later = 1;
    }
    if (seen_later) break;
    ++dead;
  }
  int tiles = 0;
  for (int first = 0; first + Z <= dead; first += Z) ++tiles;  /* whole tiles inside the dead prefix */
  *dead_keys = dead;
  *dead_tiles = tiles;
  return 0;
}

/*
 * How many blocks must a circular (window) store of tile size Z hold per sequence
 * so that a call answering `queries` consecutive steps with this window finds every
 * tile it reads still resident, wherever the steps fall relative to the tile
 * boundaries?  (Section 6, window store: a pre-allocated circular buffer sized by the
 * window.)  By trying every first step over several tile periods and counting the
 * tiles between the oldest visible key of the first step and the newest key of the
 * last.  The answer is that largest count itself: consecutive tiles n, n+1, ... land
 * in distinct blocks of a circular store of R blocks (tile n in block n mod R) exactly
 * when there are at most R of them.  Returns the count, or -1 for window < 1, Z < 1
 * or queries < 1.
 */
int tempo_oracle_ring_blocks(int window, int Z, int queries) {
  if (window < 1 || Z < 1 || queries < 1) return -1;
  int most = 0;
  for (int first = 0; first < window + 4 * Z; ++first) {
    const int last = first + queries - 1;
    int oldest = -1;
    for (int j = 0; j <= first; ++j) {
      if (visible(j, first, window)) { oldest = j; break; }
    }
    /* walk the keys in order, opening a new tile every Z keys; count the tiles that hold a key that matters */
    int tiles = 0, counted_tile = -1, tile = 0, slot = 0;
    for (int j = 0; j <= last; ++j) {
      if (j >= oldest && tile != counted_tile) { ++tiles; counted_tile = tile; }
      if (++slot == Z) { slot = 0; ++tile; }
    }
    if (tiles > most) most = tiles;
  }
  return most;
}

/*
 * Eq. 1 for every sequence b and query head h, at that sequence's own step
 * t[b].  All arrays are fp64, row-major:
 *   q   [B][Hq][D]        query of step t[b]
 *   K,V [B][T][Hkv][D]    keys/values of steps 0..T-1 (only 0..t[b] are read)
 *   out [B][Hq][D]
 * window: number of visible keys (0 = causal).  Returns 0, or -1 on a bad
 * argument (Hq not a multiple of Hkv, t[b] outside [0,T), ...).
 */
int tempo_oracle_attend(const double* q, const double* K, const double* V,
                        int B, int T, int Hq, int Hkv, int D,
                        const int* t, int window, double scale, double* out) {
  if (!q || !K || !V || !t || !out) return -1;
  if (B < 1 || T < 1 || Hq < 1 || Hkv < 1 || D < 1 || window < 0) return -1;
  if (Hq % Hkv != 0) return -1;
  for (int b = 0; b < B; ++b)
    if (t[b] < 0 || t[b] >= T) return -1;
  const int group = Hq / Hkv;

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int b = 0; b < B; ++b) {
    for (int h = 0; h < Hq; ++h) {
      const int g = h / group;                 /* key/value head of query head h */
      const int hi = t[b];
      const int lo = (window == 0) ? 0 : (hi - window + 1 > 0 ? hi - window + 1 : 0);
      const double* qv = q + ((size_t)b * Hq + h) * D;
      double* ov = out + ((size_t)b * Hq + h) * D;

      /* logits z_j = s * <q, k_j>, and their maximum */
      double zmax = -INFINITY;
      for (int j = lo; j <= hi; ++j) {
        const double* kv = K + (((size_t)b * T + j) * Hkv + g) * D;
        double z = 0.0;
        for (int d = 0; d < D; ++d) z += qv[d] * kv[d];
        z *= scale;
        if (z > zmax) zmax = z;
      }
      /* softmax weights p_j = exp(z_j - zmax) / sum, applied to v_j */
      double denom = 0.0;
      for (int d = 0; d < D; ++d) ov[d] = 0.0;
      for (int j = lo; j <= hi; ++j) {
        const double* kv = K + (((size_t)b * T + j) * Hkv + g) * D;
        const double* vv = V + (((size_t)b * T + j) * Hkv + g) * D;
        double z = 0.0;
        for (int d = 0; d < D; ++d) z += qv[d] * kv[d];
        z *= scale;
        const double p = exp(z - zmax);
        denom += p;
        for (int d = 0; d < D; ++d) ov[d] += p * vv[d];
      }
      for (int d = 0; d < D; ++d) ov[d] /= denom;
    }
  }
  return 0;
}

/*
 * Rotary position embedding of the producer step (the operation whose output the
 * block store receives in place, Section 6 "in-place writes").  The paper names
 * no position encoding; its decoding workload is a Llama-3.2 model, whose public
 * definition rotates each head vector x of dimension D at position t by
 *     angle_i = t * theta^(-2i/D),           i = 0 .. D/2-1
 *     y[i]       = x[i] * cos(angle_i) - x[i + D/2] * sin(angle_i)
 *     y[i + D/2] = x[i + D/2] * cos(angle_i) + x[i] * sin(angle_i)
 * (dimension i is paired with i + D/2; no frequency rescaling).
 *   x, y  [B][H][D] fp64;  t [B] positions;  theta > 0 the base.
 * Returns 0, or -1 on a bad argument (odd D, negative position, ...).
 */
int tempo_oracle_rope(const double* x, int B, int H, int D, const int* t, double theta, double* y) {
  if (!x || !t || !y || B < 1 || H < 1 || D < 2 || D % 2 != 0 || !(theta > 0.0)) return -1;
  for (int b = 0; b < B; ++b)
    if (t[b] < 0) return -1;
  const int half = D / 2;
  for (int b = 0; b < B; ++b) {
    for (int h = 0; h < H; ++h) {
      const double* xv = x + ((size_t)b * H + h) * D;
      double* yv = y + ((size_t)b * H + h) * D;
      for (int i = 0; i < half; ++i) {
        const double angle = (double)t[b] * pow(theta, -2.0 * (double)i / (double)D);
        const double c = cos(angle), sn = sin(angle);
        yv[i] = xv[i] * c - xv[i + half] * sn;
        yv[i + half] = xv[i + half] * c + xv[i] * sn;
      }
    }
  }
  return 0;
}

/* cos and sin of the same angles as a table [positions][D/2] (position t = row t),
 * the form in which inference stacks keep them.  Returns 0 or -1. */
int tempo_oracle_rope_table(int positions, int D, double theta, double* cos_out, double* sin_out) {
  if (!cos_out || !sin_out || positions < 1 || D < 2 || D % 2 != 0 || !(theta > 0.0)) return -1;
  const int half = D / 2;
  for (int t = 0; t < positions; ++t) {
    for (int i = 0; i < half; ++i) {
      const double angle = (double)t * pow(theta, -2.0 * (double)i / (double)D);
      cos_out[(size_t)t * half + i] = cos(angle);
      sin_out[(size_t)t * half + i] = sin(angle);
    }
  }
  return 0;
}

/*
 * Anti-causal window reduction of the paper's reinforcement-learning example (Section 3,
 * Algorithm 1): the return of step t is the discounted sum of the rewards of the steps
 * t .. min(t+n, T)-1 (an n-step return), or of all steps t .. T-1 (the whole future):
 *     g[b][t] = sum_{k = 0}^{m-1} gamma^k * r[b][t+k],   m = min(n, T-t),  or  m = T-t  if n == 0.
 * The paper names the operation ("discounted_sum") without a formula; this is the usual
 * meaning of a discounted return, the first reward undiscounted.  The range is the forward
 * (anti-causal) window whose inverse the paper prints next to the attention windows.
 *   r, g  [B][T] fp64, row-major.   Returns 0, or -1 on a bad argument.
 */
int tempo_oracle_discounted_sum(const double* r, int B, int T, int n, double gamma, double* g) {
  if (!r || !g || B < 1 || T < 1 || n < 0) return -1;
  for (int b = 0; b < B; ++b) {
    for (int t = 0; t < T; ++t) {
      const int stop = (n == 0 || t + n > T) ? T : t + n;   /* the slice t : min(t+n, T) */
      double sum = 0.0, weight = 1.0;                         /* gamma^0 */
      for (int j = t; j < stop; ++j) {
        sum += weight * r[(size_t)b * T + j];
        weight *= gamma;
      }
      g[(size_t)b * T + t] = sum;
    }
  }
  return 0;
}

/* Threads the attention routine will use (for reporting beside a timing). */
int tempo_oracle_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
