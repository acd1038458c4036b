// Static work partition of one decode step, shared by the partial kernel (which
// walks it) and the combine kernel (which enumerates the partial slots of a row).
//
// Keys are processed in tiles of TK rows.  A "prefix unit" is one (prompt, KV
// head) and owns ceil(Lp/TK) tiles; a "suffix unit" is one (sequence, KV head)
// and owns ceil(Ls/TK) tiles.  Prefix tiles form one line (prompt-major, then KV
// head, then tile), suffix tiles another (sequence-major, then KV head, then tile).
//
// The partial kernel runs 2 * n_launch workgroups, two per compute unit: workgroup
// c ("A") and workgroup n_cu + c ("B") form pair c.  n_launch is the largest power of
// two that is at most the device's compute-unit count and at most N_CU (256 on a
// whole MI355X; 128, 64 or 32 when the device is one partition of it), so that
// the share arithmetic is shifts, and n_cu = n_launch except for a small batch (fewer than
// SPARSE_BATCH_TILES tiles), which is cut among n_cu = n_launch / 2 pairs, the first 2 * n_cu
// workgroups, while the others stay idle: its wavefronts hold one or two tiles either way, but
// its rows are then cut into half as many partial results, which is what the combine step's
// time follows.  Every working pair gets the same
// share of each line (position N*c/n_cu .. N*(c+1)/n_cu), so that every compute
// unit carries the same mix of work and all finish together.  Inside a pair the
// two workgroups are evened out by tile weight (a prefix tile costs wP, a suffix
// tile SUFFIX_WEIGHT): in a batch whose suffix tiles outweigh its prefix tiles, A takes all
// prefix tiles plus the first few suffix tiles and B the other suffix tiles; in
// a prefix-heavy batch (short responses behind long multimodal prompts, the
// first steps of any rollout), A takes prefix tiles only and B the last few
// prefix tiles plus all suffix tiles.  A workgroup processes its
// prefix tiles together (one shared K/V tile in LDS, 16-row query blocks spread
// over the wavefronts) and then cuts its suffix tiles into WG_WAVES consecutive
// runs, one per wavefront.
//
// A KV group of more than 64 query rows ("dual" partition) is handled in row halves of 64
// by twin pairs: pairs c and c ^ 8 run on the same die (workgroup i goes to die i % 8) and
// walk the same share of the prefix line at the same time, one for the even half of the
// rows and one for the odd half, so that a tile is fetched from memory once and the second
// request finds it in the die's L2.  The line then has n_cu / 2 shares of twice the length;
// with more than 128 rows it holds every (prompt, KV head) twice, once per pair of halves.
// Everything else (the split inside a pair, the suffix line) is as above.
//
// Every maximal run of tiles of one unit inside one workgroup (prefix) or one
// wavefront (suffix) yields one partial (o, lse); its slot is unit + (2c + [B])
// (prefix) or unit + WG_WAVES*(2c + [B]) + wavefront (suffix), unique because
// both terms are monotone along the line (dual: 2 * (line unit + 2q + [B]) + side with q the
// share of the twins, for the same reason).  Nothing here depends on run-time timing, so
// the split and hence the rounding order is the same on every call.
#pragma once

#include <stdint.h>

namespace rlda {

constexpr int TK = 32;            // keys per tile
constexpr int WG_WAVES = 4;       // wavefronts per workgroup
constexpr int N_CU = 256;         // most workgroup pairs: one per compute unit of a whole MI355X
constexpr int N_WG = 2 * N_CU;    // most workgroups of the partial kernel (workspaces are sized for it)
constexpr int CU_PER_DIE = 32;    // compute units per die: workgroup i is dispatched to die i % (n_cu / 32)

// workgroup pairs the kernels use on a device with `compute_units` compute units (>= 1)
__host__ __device__ inline int pairs_for(int compute_units) {
  int n = 1;
  while (2 * n <= compute_units && 2 * n <= N_CU) n *= 2;
  return n;
}
constexpr int PREFIX_WEIGHT = 6;  // cost of a prefix tile ...
constexpr int SUFFIX_WEIGHT = 4;  // ... relative to a suffix tile, when the batch saturates the memory system
// A batch of fewer tiles than this (256 MB of K/V) does not: its suffix tiles then come back in half the
// time while a prefix tile still takes a workgroup one memory round trip per group of four plus the
// matrix work of all row blocks, so prefix tiles weigh more.
constexpr int SMALL_BATCH_TILES = 16384;
constexpr int PREFIX_WEIGHT_SMALL = 14;
// A batch of fewer tiles than this (2 per wavefront of half the grid) works with half the pairs, down to 32
// (not the dual partition of groups of more than 64 rows, which keeps the whole grid).
constexpr int SPARSE_BATCH_TILES = 2048;

struct Sched {
  int NPT;      // prefix tiles in total (all units)
  int NST;      // suffix tiles in total
  int wP;       // weight of a prefix tile (a suffix tile weighs SUFFIX_WEIGHT)
  int n_launch; // workgroup pairs launched, a power of two
  int n_cu;     // workgroup pairs that get work (n_launch, or half of it for a small batch), a power of two
  int cu_sh;    // its logarithm
  bool heavy;   // the prefix tiles outweigh the suffix tiles: B workgroups share them, A takes no suffix
  bool dual;    // twin pairs walk the same prefix tiles, for different row halves
  int tb;       // dual: pairs c and c ^ (1 << tb) are twins
  int psh;      // logarithm of the number of shares of the prefix line (cu_sh, dual: cu_sh - 1)
};

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// The R = G * Hq/Hkv query rows that share a prefix tile are handled in row parts ("halves") of at
// most 64 rows (one 16-row block per wavefront): 1, 2 or 4 parts.  With several parts and at least
// two pairs, twin pairs take one each (side_parts = 2) and the line holds line_parts units per
// (prompt, KV head).
constexpr int MAX_GROUP_ROWS = 256;
__host__ __device__ inline int row_parts(int R) { return R > 128 ? 4 : (R > 64 ? 2 : 1); }
__host__ __device__ inline int side_parts(int R, int n_cu) { return R > 64 && n_cu > 1 ? 2 : 1; }
__host__ __device__ inline int line_parts(int R, int n_cu) { return row_parts(R) / side_parts(R, n_cu); }
__host__ __device__ inline int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// The prefix weight is PREFIX_WEIGHT for a saturating batch; small suffix-heavy batches use PREFIX_WEIGHT_SMALL instead.
// NPT counts the tiles of the prefix line (in a dual partition every one is walked twice; n_cu > 1 then).
__host__ __device__ inline Sched make_sched(int NPT, int NST, int n_launch, bool dual = false) {
  Sched s;
  const int n_cu = !dual && NPT + NST < SPARSE_BATCH_TILES && n_launch >= 64 ? n_launch / 2 : n_launch;
  s.NPT = NPT; s.NST = NST; s.n_launch = n_launch; s.n_cu = n_cu; s.dual = dual;
  s.cu_sh = 31 - __builtin_clz((unsigned)n_cu);             // n_cu is a power of two >= 1
  s.tb = s.cu_sh > 3 ? 3 : (s.cu_sh > 0 ? s.cu_sh - 1 : 0);   // twins on one die: the die is c % 8 (fewer than 16 pairs: one die)
  s.psh = dual ? s.cu_sh - 1 : s.cu_sh;
  const int walked = dual ? 2 * NPT : NPT;     // lines are at most MAX_LINE tiles: no overflow
  s.heavy = PREFIX_WEIGHT * walked > SUFFIX_WEIGHT * NST;
  s.wP = !s.heavy && walked + NST < SMALL_BATCH_TILES ? PREFIX_WEIGHT_SMALL : PREFIX_WEIGHT;
  return s;
}

// Lines are limited to MAX_LINE tiles so that the share arithmetic (a line position times the pair count)
// stays in 32 bits.
constexpr int MAX_LINE = (1 << 30) / N_CU;

// pair c owns positions [share(N, c), share(N, c + 1)) of a line of N tiles (cu_sh = log2 of the pair count)
__host__ __device__ inline int share(int N, int c, int cu_sh) { return (int)(((unsigned)N * (unsigned)c) >> cu_sh); }
// the pair that owns position i (0 <= i < N): the largest c with share(N, c) <= i, that is
// ceil((i + 1) * 2^cu_sh / N) - 1.  A float quotient lands within one of it and two exact steps settle it
// (an integer division costs the combine kernels, which ask four times per row, several times as much).
__host__ __device__ inline int share_owner(int N, int i, int cu_sh) {
  const int last = (1 << cu_sh) - 1;
  int c = (int)((float)(i + 1) * ((float)(1 << cu_sh) / (float)N));
  c = c > last ? last : c;
  if (share(N, c, cu_sh) > i) --c;
  if (share(N, c, cu_sh) > i) --c;
  if (c < last && share(N, c + 1, cu_sh) <= i) ++c;
  if (c < last && share(N, c + 1, cu_sh) <= i) ++c;
  return c;
}

// share of the prefix line that pair c walks, the row half it walks it for (dual), and the pair of a share and side
__host__ __device__ inline int prefix_share(const Sched& s, int c) {
  return s.dual ? ((c >> (s.tb + 1)) << s.tb) | (c & ((1 << s.tb) - 1)) : c;
}
__host__ __device__ inline int prefix_side(const Sched& s, int c) { return s.dual ? (c >> s.tb) & 1 : 0; }
__host__ __device__ inline int share_pair(const Sched& s, int q, int side) {
  return s.dual ? ((q >> s.tb) << (s.tb + 1)) | (side << s.tb) | (q & ((1 << s.tb) - 1)) : q;
}

// prefix tiles of pair c: [lo, hi), of which A takes [lo, mid) and B [mid, hi).  B gets some only
// in a prefix-heavy batch, and then as many as even out the pair.
__host__ __device__ inline void pair_prefix_range(const Sched& s, int c, int& lo, int& mid, int& hi) {
  const int q = prefix_share(s, c);
  lo = share(s.NPT, q, s.psh);
  hi = share(s.NPT, q + 1, s.psh);
  mid = hi;
  if (s.heavy) {
    const int ns = share(s.NST, c + 1, s.cu_sh) - share(s.NST, c, s.cu_sh);
    mid = hi - clampi((PREFIX_WEIGHT * (hi - lo) - SUFFIX_WEIGHT * ns) / (2 * PREFIX_WEIGHT), 0, hi - lo);   // wP = PREFIX_WEIGHT here
  }
}
// Workgroups are named by w = c for the A and n_launch + c for the B of pair c; pairs from n_cu on are idle.
// The grid's workgroup x takes the name wg_name(x): the first 2 * n_cu of the grid work (A of pair c is x = c, its
// B is x = n_cu + c), the others take the name of an idle pair.
__host__ __device__ inline int wg_name(const Sched& s, int x) {
  if (x >= 2 * s.n_cu) return s.n_launch - 1;               // only when n_cu < n_launch: an idle pair
  return (x & s.n_cu) ? s.n_launch + (x & (s.n_cu - 1)) : x;
}
__host__ __device__ inline int wg_grid_index(const Sched& s, int c, bool is_b) { return is_b ? s.n_cu + c : c; }
__host__ __device__ inline int wg_pair(const Sched& s, int w) { return w & (s.n_launch - 1); }
__host__ __device__ inline bool wg_is_b(const Sched& s, int w) { return w >= s.n_launch; }
__host__ __device__ inline void wg_prefix_range(const Sched& s, int w, int& lo, int& hi) {
  int a, m, b;
  const int c = wg_pair(s, w);
  pair_prefix_range(s, c, a, m, b);
  if (!wg_is_b(s, w)) { lo = a; hi = m; } else { lo = m; hi = b; }
  if (c >= s.n_cu) lo = hi = 0;
}
__host__ __device__ inline int prefix_tile_share(const Sched& s, int i) { return share_owner(s.NPT, i, s.psh); }

// suffix tiles of pair c: [lo, hi), of which A takes [lo, mid) and B [mid, hi).  A gets some only
// in a suffix-heavy batch, and then as many as even out the pair.
__host__ __device__ inline void pair_suffix_range(const Sched& s, int c, int& lo, int& mid, int& hi) {
  lo = share(s.NST, c, s.cu_sh);
  hi = share(s.NST, c + 1, s.cu_sh);
  mid = lo;
  if (!s.heavy) {
    const int q = prefix_share(s, c);
    const int np = share(s.NPT, q + 1, s.psh) - share(s.NPT, q, s.psh);
    mid = lo + clampi((SUFFIX_WEIGHT * (hi - lo) - s.wP * np) / (2 * SUFFIX_WEIGHT), 0, hi - lo);
  }
}
__host__ __device__ inline void wg_suffix_range(const Sched& s, int w, int& lo, int& hi) {
  int a, m, b;
  const int c = wg_pair(s, w);
  pair_suffix_range(s, c, a, m, b);
  if (!wg_is_b(s, w)) { lo = a; hi = m; } else { lo = m; hi = b; }
  if (c >= s.n_cu) lo = hi = 0;
}
__host__ __device__ inline int suffix_tile_pair(const Sched& s, int k) { return share_owner(s.NST, k, s.cu_sh); }

// run of wavefront v inside the workgroup's suffix range
__host__ __device__ inline void wave_suffix_range(int lo, int hi, int v, int& a, int& b) {
  const int q = ceil_div(hi - lo, WG_WAVES);
  a = lo + v * q; if (a > hi) a = hi;
  b = a + q;      if (b > hi) b = hi;
}
__host__ __device__ inline int suffix_tile_wave(int lo, int hi, int k) {      // (k - lo) / q without the division
  const int q = ceil_div(hi - lo, WG_WAVES), d = k - lo;
  int v = 0;
  for (int u = 1; u < WG_WAVES; ++u) v += d >= u * q ? 1 : 0;
  return v;
}
// slot term of workgroup w on the suffix line (A and B of a pair are neighbours there, A first) and on the
// prefix line (the same, by share)
__host__ __device__ inline int wg_rank(const Sched& s, int w) { return 2 * wg_pair(s, w) + (wg_is_b(s, w) ? 1 : 0); }
__host__ __device__ inline int wg_prefix_rank(const Sched& s, int w) {
  return 2 * prefix_share(s, wg_pair(s, w)) + (wg_is_b(s, w) ? 1 : 0);
}

// ---- walking the line -------------------------------------------------------------------
// X is the exclusive scan of per-head tile counts over `n` prompts (or sequences); every
// prompt/sequence contributes Hkv units of X[i+1]-X[i] tiles each.  `tile` is an index into that
// family's part of the line (0 <= tile < X[n]*Hkv).

// Unit (major, j) and tile-within-unit t that hold line position `tile`.
__host__ __device__ inline void locate(const int* X, int n, int Hkv, int tile, int& major, int& j, int& t) {
  int lo = 0, hi = n - 1;                      // largest i with X[i]*Hkv <= tile (its unit count is > 0)
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (X[mid] * Hkv <= tile) lo = mid; else hi = mid - 1;
  }
  const int T = X[lo + 1] - X[lo], rem = tile - X[lo] * Hkv;
  major = lo; j = rem / T; t = rem % T;
}

// Calls body(major, j, t0, ntiles) for every maximal run of one unit inside line range [lo, hi),
// starting at the located position.  tiles_of(major) returns the per-head tile count.
template <class TilesOf, class Body>
__host__ __device__ inline void for_each_run(int lo, int hi, int n, int Hkv, int major, int j, int t,
                                             TilesOf tiles_of, Body body) {
  for (int i = lo; i < hi;) {
    const int T = tiles_of(major);
    const int run = (T - t) < (hi - i) ? (T - t) : (hi - i);
    body(major, j, t, run);
    i += run; t = 0;
    if (++j == Hkv) {
      j = 0;
      do { ++major; } while (major < n && tiles_of(major) == 0);
    }
  }
}

// Workgroups (by prefix rank) holding a partial of unit (p, j) of the prefix line for row half `side` (0 unless
// dual): fn(rank) in line order.  Xp = scan over prompts.
template <class Fn>
__host__ __device__ inline void for_each_prefix_part(const Sched& s, const int* Xp, int Hkv, int p, int j, int side,
                                                     Fn fn) {
  const int T = Xp[p + 1] - Xp[p];
  if (T <= 0) return;
  const int is = Xp[p] * Hkv + j * T, ie = is + T;
  for (int q = prefix_tile_share(s, is); q <= prefix_tile_share(s, ie - 1); ++q) {
    int lo, mid, hi;                             // with fewer tiles than shares some hold nothing
    pair_prefix_range(s, share_pair(s, q, side), lo, mid, hi);
    if ((lo > is ? lo : is) < (mid < ie ? mid : ie)) fn(2 * q);
    if (s.heavy && (mid > is ? mid : is) < (hi < ie ? hi : ie)) fn(2 * q + 1);
  }
}

// (suffix rank of the workgroup, wavefront) pairs holding a partial of suffix unit (b, j): fn(rank, v)
// in line order.  Xs = scan over sequences, xs0 = its value at sequence 0 (so Xs may continue Xp).
template <class Fn>
__host__ __device__ inline void for_each_suffix_part(const Sched& s, const int* Xs, int xs0, int Hkv, int b, int j,
                                                     Fn fn) {
  const int T = Xs[b + 1] - Xs[b];
  if (T <= 0) return;
  const int ks = (Xs[b] - xs0) * Hkv + j * T, ke = ks + T;
  for (int c = suffix_tile_pair(s, ks); c <= suffix_tile_pair(s, ke - 1); ++c) {
    int lo, mid, hi;
    pair_suffix_range(s, c, lo, mid, hi);
    for (int half = 0; half < 2; ++half) {
      const int a = half ? mid : lo, e = half ? hi : mid;
      const int k0 = ks > a ? ks : a, k1 = (ke < e ? ke : e) - 1;
      if (k0 > k1) continue;
      for (int v = suffix_tile_wave(a, e, k0); v <= suffix_tile_wave(a, e, k1); ++v) fn(2 * c + half, v);
    }
  }
}

}  // namespace rlda
