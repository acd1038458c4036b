// Static work partition of one decode step, shared by the partial kernel (which
// walks it) and the combine kernel (which enumerates the partial slots of a row).
//
// Keys are processed in tiles of TK rows.  A "prefix unit" is one (prompt, KV
// head) and owns ceil(Lp/TK) tiles; a "suffix unit" is one (sequence, KV head)
// and owns ceil(Ls/TK) tiles.  All tiles are laid on one line, prefix tiles
// first (prompt-major, then KV head, then tile), then suffix tiles (sequence-
// major, then KV head, then tile).  A prefix tile weighs wP, a suffix tile wS;
// workgroup w takes the tiles whose weighted position falls in [w*S, (w+1)*S).
// Its prefix tiles are processed by the whole workgroup (one shared K/V tile in
// LDS, one 16-row query block per wavefront); its suffix tiles are cut into four
// consecutive runs, one per wavefront.  Every maximal run of tiles of one unit
// inside one workgroup (prefix) or one wavefront (suffix) yields one partial
// (o, lse); its slot is unit + workgroup (prefix) or unit + 4*workgroup +
// wavefront (suffix), which is unique because both terms are monotone along
// the line.  Nothing here depends on run-time timing, so the split and hence
// the rounding order is the same on every call.
#pragma once

#include <stdint.h>

namespace rlda {

constexpr int TK = 32;            // keys per tile
constexpr int WG_WAVES = 4;       // wavefronts per workgroup
constexpr int N_WG = 512;         // workgroups of the partial kernel: 256 CUs x 2 resident
constexpr int PREFIX_WEIGHT = 4;  // weight of a prefix tile on the line
constexpr int SUFFIX_WEIGHT = 4;  // weight of a suffix tile on the line

struct Sched {
  int NPT;      // prefix tiles in total (all units)
  int NST;      // suffix tiles in total
  int wP;       // weight of a prefix tile
  int wS;       // weight of a suffix tile
  int S;        // weighted share of one workgroup (>= 1)
  int n_wg;     // workgroups
};

__host__ __device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ inline int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

__host__ __device__ inline Sched make_sched(int NPT, int NST, int wP, int wS, int n_wg) {
  Sched s;
  s.NPT = NPT; s.NST = NST; s.wP = wP; s.wS = wS; s.n_wg = n_wg;
  const int W = wP * NPT + wS * NST;
  s.S = W > 0 ? ceil_div(W, n_wg) : 1;
  return s;
}

// prefix tiles [lo, hi) of workgroup w: tile i belongs to workgroup floor(wP*i / S)
__host__ __device__ inline void wg_prefix_range(const Sched& s, int w, int& lo, int& hi) {
  lo = clampi(ceil_div(w * s.S, s.wP), 0, s.NPT);
  hi = clampi(ceil_div((w + 1) * s.S, s.wP), 0, s.NPT);
}
__host__ __device__ inline int prefix_tile_owner(const Sched& s, int i) { return (s.wP * i) / s.S; }

// suffix tiles [lo, hi) of workgroup w
__host__ __device__ inline void wg_suffix_range(const Sched& s, int w, int& lo, int& hi) {
  const int base = s.wP * s.NPT;
  lo = w * s.S <= base ? 0 : clampi(ceil_div(w * s.S - base, s.wS), 0, s.NST);
  hi = (w + 1) * s.S <= base ? 0 : clampi(ceil_div((w + 1) * s.S - base, s.wS), 0, s.NST);
}
__host__ __device__ inline int suffix_tile_owner(const Sched& s, int k) { return (s.wP * s.NPT + s.wS * k) / s.S; }

// run of wavefront v inside the workgroup's suffix range
__host__ __device__ inline void wave_suffix_range(int lo, int hi, int v, int& a, int& b) {
  const int q = ceil_div(hi - lo, WG_WAVES);
  a = lo + v * q; if (a > hi) a = hi;
  b = a + q;      if (b > hi) b = hi;
}
__host__ __device__ inline int suffix_tile_wave(int lo, int hi, int k) {
  const int q = ceil_div(hi - lo, WG_WAVES);
  return (k - lo) / q;
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

// Workgroups holding a partial of prefix unit (p, j): fn(w) in increasing w.  Xp = scan over prompts.
template <class Fn>
__host__ __device__ inline void for_each_prefix_part(const Sched& s, const int* Xp, int Hkv, int p, int j, Fn fn) {
  const int T = Xp[p + 1] - Xp[p];
  if (T <= 0) return;
  const int is = Xp[p] * Hkv + j * T, ie = is + T;
  for (int w = prefix_tile_owner(s, is); w <= prefix_tile_owner(s, ie - 1); ++w) {
    int lo, hi;                                  // with a share below one tile weight some workgroups own nothing
    wg_prefix_range(s, w, lo, hi);
    if ((lo > is ? lo : is) < (hi < ie ? hi : ie)) fn(w);
  }
}

// (workgroup, wavefront) pairs holding a partial of suffix unit (b, j): fn(w, v) in line order.
// Xs = scan over sequences, xs0 = its value at sequence 0 (subtracted, so Xs may continue Xp).
template <class Fn>
__host__ __device__ inline void for_each_suffix_part(const Sched& s, const int* Xs, int xs0, int Hkv, int b, int j,
                                                     Fn fn) {
  const int T = Xs[b + 1] - Xs[b];
  if (T <= 0) return;
  const int ks = (Xs[b] - xs0) * Hkv + j * T, ke = ks + T;
  for (int w = suffix_tile_owner(s, ks); w <= suffix_tile_owner(s, ke - 1); ++w) {
    int lo, hi;
    wg_suffix_range(s, w, lo, hi);
    const int k0 = ks > lo ? ks : lo, k1 = (ke < hi ? ke : hi) - 1;
    if (k0 > k1) continue;
    for (int v = suffix_tile_wave(lo, hi, k0); v <= suffix_tile_wave(lo, hi, k1); ++v) fn(w, v);
  }
}

}  // namespace rlda
