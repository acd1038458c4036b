// Shared-prefix decode attention on gfx950 matrix cores (bf16 in, fp32 accumulate, d = 128).
// K/V stores hold bf16, or e4m3 bytes that are widened to bf16 (exactly) on their way into LDS.
//
// Two kernels per call:
//   partial_kernel  walks the static tile partition of rlda_sched.h with two workgroups of four
//                   wavefronts per compute unit.  Prefix tiles (the prompt s_0 shared by the K
//                   sampled trajectories of a group, Algorithm 1 / Sec. 3.2.2 of the paper) are
//                   staged once in LDS per workgroup and used by all G * Hq/Hkv query rows of
//                   the KV group (by each half of them when there are more than 64: a wavefront
//                   carries one 16-row block); suffix tiles (each trajectory's own generated tokens, Sec. 3.1
//                   transition s' = (s, a)) are streamed by single wavefronts.  Every maximal
//                   run of tiles of one (prompt or sequence, KV head) yields a partial (o, lse).
//   combine_kernel  merges the partials of every (sequence, head) by log-sum-exp and writes
//                   out / lse (combine16_kernel: the same with half the lanes per row, for
//                   batches of many units).
//
// Tile math (one wavefront, 16 query rows, 32 keys): scores are produced
// transposed, S^T = K_tile * Q^T, with v_mfma_f32_16x16x32_bf16 (A = 16 keys x 32
// dims read from LDS, B = Q^T held in registers).  In that accumulator layout a
// lane owns one query row and 4 keys per 16-key half, which is exactly the
// B-operand layout of the second contraction O^T += V_tile^T * P^T, so the
// probabilities go from accumulator to operand with a bf16 convert and no
// cross-lane traffic.  V^T comes from LDS through ds_read_b64_tr_b16.  The online
// softmax needs one 4-lane max per tile (two lane swaps); row sums stay per
// lane until the partial is written.
//
// The same source holds the prefill pass (causal attention of every prompt over itself, once per
// prompt: prefill2_kernel, and the register-staged prefill_kernel it grew out of), which is built
// from the same tile layout and products.
#include "rlda_internal.h"
#include "rlda_sched.h"

#include <mutex>
#include <type_traits>

namespace rlda {
namespace {

constexpr int D = 128;
constexpr int ROWB = D * 2;                       // bytes per K/V row in LDS (and in a bf16 store; also a q row)
constexpr int TILE_B = TK * ROWB;                 // 8 KB: one K or V tile
constexpr int STAGE_B = 2 * TILE_B;               // K tile + V tile
constexpr int NTHREADS = 64 * WG_WAVES;
constexpr int LDS_BYTES = WG_WAVES * STAGE_B;     // 64 KB: one stage per wavefront, two workgroups per CU
constexpr int MAX_SCAN = LDS_BYTES / 4;           // ints of LDS available to the length scan

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One level of a tree of shared prefix segments (rl_decode_attn_tree): `n` segments, each shared by G
// consecutive sequences (R = G * Hq/Hkv query rows per KV head); the level's segments are entries
// first .. first + n - 1 of the prefix line.
struct TreeLevel { const char* k; const char* v; const int32_t* lens; int first, G, R, cap; };
constexpr int MAX_LEVELS = RLDA_MAX_TREE_LEVELS;   // 4

// n / d for 0 <= n < 2^31 as a multiplication: m = floor(2^k / d) + 1 with k = 31 + ceil(log2 d) (m fits 32 bits,
// and m * d - 2^k <= d <= 2^(k - 31) makes the quotient exact).  The combine kernels split every row index three
// times; a 32-bit integer division costs them about ten times this.
struct FastDiv { uint32_t m; int k; };
inline FastDiv make_fastdiv(int d) {
  if (d < 1) d = 1;                                          // an empty batch launches nothing; keep the host safe
  int l = 0;
  while ((1 << l) < d) ++l;
  FastDiv f;
  f.k = 31 + l;
  f.m = (uint32_t)(((uint64_t)1 << f.k) / (uint32_t)d + 1);
  return f;
}
__device__ __forceinline__ int fast_div(int n, FastDiv f) { return (int)(((uint64_t)(uint32_t)n * f.m) >> f.k); }

struct SharedParams {
  const char* q; const char* kp; const char* vp; const char* ks; const char* vs;
  const int32_t* plens; const int32_t* slens;
  float* out; float* lse;
  int32_t* cum;           // [P + B + 1] exclusive scan of tile counts (prompts, then sequences)
  // partials: o rows as fp16 [slot][rows][D] (columns permuted, see write_partial), and per row the
  // pair (lse, power-of-two scale of the stored row) as fp32 [slot][rows][2]
  _Float16* po; float* pl;   // prefix, RS rows per slot
  _Float16* so; float* sl;   // suffix, r rows per slot
  int P, G, B, Hq, Hkv, r, R, Lp_cap, Ls_cap;
  // The R = G * r query rows of a KV group are handled in NH = 1, 2 or 4 row parts of at most 64
  // rows (NH = 2^NHs, more than one when R > 64): a prefix unit is (prompt, KV head, part), numbered
  // jp = j * NH + part, so that a wavefront never carries more than one 16-row block.
  // The prefix line holds HkvP = Hkv * NH units per prompt (NH = 1 << NHs); with SM = 2 each is walked by twin
  // pairs, for row halves 2 * (unit % NH) and 2 * (unit % NH) + 1.  A prefix partial slot holds RS rows.
  int NH, NHs, HkvP, RS, SM;
  float c;                // scale * log2(e): scores are kept in base 2
  // extended form only (kernels instantiated with EXT = true):
  const int32_t* table;   // [B, max_pages] page ids when ks / vs are page pools [n_pages, Hkv, page, D], else null
  const uint8_t* active;  // [B] finished-sequence flags, or null
  int page_shift, max_pages, n_pages;
  // e4m3 K/V stores only (kernels instantiated with F8 = true): per-KV-head factors, or null
  const float* kscale; const float* vscale;
  // tree form only (kernels instantiated with TREE = true): the prefix line holds the segments of all levels,
  // level after level, P is their total number, G and R are the largest group's, kp / vp / plens are unused
  TreeLevel lev[MAX_LEVELS];
  int n_lev;
  int n_cu;               // workgroup pairs (pairs_for the device's compute units); the grid is 2 * n_cu workgroups
  FastDiv div_Hq, div_G, div_r;   // exact quotients by Hq, G and r for the combine kernels' row arithmetic
};

// the level that entry `e` of the prefix line belongs to (e is wavefront-uniform: scalar selects)
__device__ __forceinline__ TreeLevel level_of(const SharedParams& P, int e) {
  TreeLevel r = P.lev[0];
#pragma unroll
  for (int i = 1; i < MAX_LEVELS; ++i)
    if (i < P.n_lev && e >= P.lev[i].first) r = P.lev[i];
  return r;
}

// Effective lengths: clamped to the capacity; in the extended form a finished sequence has no
// suffix, and a prompt none of whose G sequences is live has no prefix.
template <bool EXT, bool TREE = false>
__device__ __forceinline__ int plen_of(const SharedParams& P, int p) {
  if constexpr (TREE) {
    const TreeLevel lv = level_of(P, p);
    return clampi(lv.lens[p - lv.first], 0, lv.cap);
  }
  int L = clampi(P.plens[p], 0, P.Lp_cap);
  if (EXT && P.active) {
    bool any = false;
    for (int g = 0; g < P.G; ++g) any |= P.active[p * P.G + g] != 0;
    if (!any) L = 0;
  }
  return L;
}
template <bool EXT>
__device__ __forceinline__ int slen_of(const SharedParams& P, int b) {
  int L = clampi(P.slens[b], 0, P.Ls_cap);
  if (EXT && P.active && P.active[b] == 0) L = 0;
  return L;
}

// NT: 16-row query blocks a wavefront carries.  The kernels instantiate NT = 1 (row halves keep
// it at one block, see SharedParams); the tile routines stay written for any NT.
template <int NT>
struct WaveState {
  f32x4 O[NT][8];         // O^T accumulators: [row tile][16-column tile], lane (row, g) holds cols 16ct+4g..+3
  float m[NT];            // running max (base-2 scores), equal in the 4 lanes of a row
  float l[NT];            // this lane's share of the row sum, exact fp32 weights (for lse)
  float lr[NT];           // same with the bf16-rounded weights (normalises O)
};

__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }

// 16-byte chunk `chunk` of tile row `row` lives at this byte offset inside a K / V tile in LDS.
// K is read 16 rows x one chunk per wavefront instruction, V 4 rows x two adjacent chunks per
// 16 lanes; the xor patterns spread either access over all banks.
__device__ __forceinline__ int k_off(int row, int chunk) { return row * ROWB + ((chunk ^ (row & 15)) << 4); }
__device__ __forceinline__ int v_off(int row, int chunk) { return row * ROWB + ((chunk ^ ((row & 7) << 1)) << 4); }

#define RLDA_LDS(T, p) ((__attribute__((address_space(3))) T*)(p))
__device__ __forceinline__ bf16x8 lds_ld128(const char* p) { return *RLDA_LDS(const bf16x8, p); }
__device__ __forceinline__ void lds_st128(char* p, u32x4 v) { *RLDA_LDS(u32x4, p) = v; }
__device__ __forceinline__ s16x4 lds_ld_tr16(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16(RLDA_LDS(s16x4, const_cast<char*>(p)));
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains the vector-memory
// counter, which would force the global loads just issued for the next tiles to land first.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Explicit "all vector-memory loads have landed".  Placed right before a tile's registers are
// copied to LDS (where that wait is due anyway), it also tells the compiler that the query
// fragments loaded earlier are resident, so that it does not drain the loads issued for the next
// tile when the fragments are first used inside the loop.
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

template <int NT>
__device__ __forceinline__ void init_state(WaveState<NT>& st) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    st.m[nt] = -INFINITY; st.l[nt] = 0.f; st.lr[nt] = 0.f;
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) st.O[nt][ct] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
}

// The softmax step on scores already in registers, in two halves (prefill2_kernel issues its V reads
// between them): the masked scores and the row maxima, then the weights, row sums and the rescaling.
// The same quotient sum(p v) / sum(p) as the plain form inside compute_tile, with less vector-ALU work
// per score.  The score factor c must be positive.
//   * the score factor c goes into the exponent's fma instead of a multiply of its own;
//   * maxima are taken as the median of (a, b, +inf): fmaxf has to return the other operand for a
//     signalling NaN, for which the compiler first passes every operand it cannot prove quiet (a
//     matrix-unit result, a cross-lane read) through an instruction of its own (the +inf comes
//     through an empty asm so that the median is not folded back into fmaxf; no score is NaN here:
//     keys past a row's limit are replaced by -inf before, and stores hold numbers);
//   * the two cross-lane steps of a row maximum are gfx950's lane-swap instructions (rows of 16
//     lanes, then halves of 32) instead of reads through the LDS queue;
//   * a row's reference maximum moves only when a tile's maximum exceeds it by more than
//     RESCALE_GAP powers of two (or on the row's first tile): until then the exponentials are taken
//     against the stale maximum, are at most 2^RESCALE_GAP, and the 32 accumulator registers of a
//     row block are left alone;
//   * the sum of the bf16-rounded weights is a two-element dot product per register pair.
constexpr float RESCALE_GAP = 8.f;
__device__ __forceinline__ float max_raw(float a, float b) {
  uint32_t inf = 0x7f800000u;
  asm("" : "+s"(inf));
  return __builtin_amdgcn_fmed3f(a, b, __uint_as_float(inf));
}
template <int NT, bool MASK>
__device__ __forceinline__ void softmax_max(const f32x4 (&s0)[NT], const f32x4 (&s1)[NT], const int (&nvalid)[NT],
                                            const WaveState<NT>& st, float c, int g, float (&sv)[NT][8], float (&m_new)[NT]) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      sv[nt][x] = (!MASK || 4 * g + x < nvalid[nt]) ? s0[nt][x] : -INFINITY;
      sv[nt][4 + x] = (!MASK || 16 + 4 * g + x < nvalid[nt]) ? s1[nt][x] : -INFINITY;
    }
    float tmax = max_raw(max_raw(max_raw(sv[nt][0], sv[nt][1]), max_raw(sv[nt][2], sv[nt][3])),
                         max_raw(max_raw(sv[nt][4], sv[nt][5]), max_raw(sv[nt][6], sv[nt][7])));
    {
      // swap(x, x) returns (x with its odd rows replaced by the even ones, x with its even rows replaced by
      // the odd ones), resp. the same for the two halves of 32 lanes: their maximum is max(x[l], x[l ^ 16 or 32])
      typedef unsigned int u32p __attribute__((ext_vector_type(2)));
      const u32p a = __builtin_amdgcn_permlane16_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false);
      tmax = max_raw(__uint_as_float(a[0]), __uint_as_float(a[1]));
      const u32p b = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false);
      tmax = max_raw(__uint_as_float(b[0]), __uint_as_float(b[1]));
    }
    m_new[nt] = max_raw(st.m[nt], tmax * c);
  }
}
template <int NT>
__device__ __forceinline__ void softmax_weights(const float (&sv)[NT][8], const float (&m_new)[NT], WaveState<NT>& st, bf16x8 (&pb)[NT], float c) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    if (__any(m_new[nt] > st.m[nt] + RESCALE_GAP)) {         // first tile: -inf + gap = -inf
      const float alpha = __builtin_amdgcn_exp2f(st.m[nt] - m_new[nt]);
      st.l[nt] *= alpha;
      st.lr[nt] *= alpha;
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) st.O[nt][ct] *= alpha;
      st.m[nt] = m_new[nt];
    }
    const float nm = -st.m[nt];
    float se = 0.f, sr = 0.f;
#pragma unroll
    for (int x = 0; x < 8; x += 2) {
      const float pe0 = __builtin_amdgcn_exp2f(fmaf(sv[nt][x], c, nm));
      const float pe1 = __builtin_amdgcn_exp2f(fmaf(sv[nt][x + 1], c, nm));
      const bf16x2 pr = __builtin_convertvector(f32x2{pe0, pe1}, bf16x2);
      pb[nt][x] = pr[0]; pb[nt][x + 1] = pr[1];
      se += pe0 + pe1;
      sr = __builtin_amdgcn_fdot2_f32_bf16(pr, bf16x2{static_cast<__bf16>(1.f), static_cast<__bf16>(1.f)}, sr, false);
    }
    st.l[nt] += se;
    st.lr[nt] += sr;
  }
}
// One 32-key tile (K at Kl, V at Vl in LDS, first `nvalid` keys real) against NT blocks of 16 query rows.
// nvalid may differ from lane to lane (a causal limit); MASK = false: every key is real for every row.
// LEAN: the softmax step in the form above (needs c > 0: the launchers send other scales elsewhere); the
// decode kernels use it (their e4m3 instantiations, which have the conversions on the vector ALU as well,
// run 3-4 % faster for it, the bf16 ones the same), the register-staged prefill kernel the plain form.
template <int NT, bool MASK = true, bool LEAN = false>
__device__ __forceinline__ void compute_tile(const char* Kl, const char* Vl, const int (&nvalid)[NT],
                                             const bf16x8 (&qf)[NT][4], WaveState<NT>& st, float c, int lane) {
  const int m16 = lane & 15, g = lane >> 4;
  f32x4 s0[NT], s1[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) { s0[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; s1[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int off = k_off(m16, 4 * ks + g);
    const bf16x8 a0 = lds_ld128(Kl + off);
    const bf16x8 a1 = lds_ld128(Kl + off + 16 * ROWB);
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      s0[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a0, qf[nt][ks], s0[nt], 0, 0, 0);
      s1[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a1, qf[nt][ks], s1[nt], 0, 0, 0);
    }
  }
  bf16x8 pb[NT];
  if constexpr (LEAN) {
    float sv[NT][8], m_new[NT];
    softmax_max<NT, MASK>(s0, s1, nvalid, st, c, g, sv, m_new);
    softmax_weights<NT>(sv, m_new, st, pb, c);
  } else {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    float sv[8];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      sv[x] = (!MASK || 4 * g + x < nvalid[nt]) ? s0[nt][x] * c : -INFINITY;
      sv[4 + x] = (!MASK || 16 + 4 * g + x < nvalid[nt]) ? s1[nt][x] * c : -INFINITY;
    }
    float tmax = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])), fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16, 64));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));          // finite: key 0 of the tile is always real
    const float m_new = fmaxf(st.m[nt], tmax);
    const float alpha = __builtin_amdgcn_exp2f(st.m[nt] - m_new);   // first tile: exp2(-inf) = 0
    float se = 0.f, sr = 0.f;
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const float pe = __builtin_amdgcn_exp2f(sv[x] - m_new);      // masked keys: 0
      const __bf16 pr = static_cast<__bf16>(pe);
      pb[nt][x] = pr;
      se += pe;
      sr += static_cast<float>(pr);
    }
    st.l[nt] = st.l[nt] * alpha + se;
    st.lr[nt] = st.lr[nt] * alpha + sr;
    st.m[nt] = m_new;
    if (__any(alpha != 1.f)) {
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) st.O[nt][ct] *= alpha;
    }
  }
  }
  // lane (m16, g) of a 16-lane block addresses row 4g + m16/4, columns 16ct + 4(m16%4)..+3 and
  // receives V[4g..4g+3][16ct + m16]: the A operand of O^T += V^T P^T for the keys its P holds.
  const int vrow = 4 * g + (m16 >> 2);
#pragma unroll
  for (int ct = 0; ct < 8; ++ct) {
    const int off = v_off(vrow, 2 * ct + ((m16 & 3) >> 1)) + ((m16 & 1) << 3);
    const s16x4 lo = lds_ld_tr16(Vl + off);
    const s16x4 hi = lds_ld_tr16(Vl + off + 16 * ROWB);
    union { s16x4 h[2]; bf16x8 v; } vt;
    vt.h[0] = lo; vt.h[1] = hi;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      st.O[nt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt.v, pb[nt], st.O[nt][ct], 0, 0, 0);
  }
}

// the same with one key count for all row blocks (the decode kernels: a tile's tail)
template <int NT, bool MASK = true, bool LEAN = false>
__device__ __forceinline__ void compute_tile(const char* Kl, const char* Vl, int nvalid, const bf16x8 (&qf)[NT][4],
                                             WaveState<NT>& st, float c, int lane) {
  int nv[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) nv[nt] = nvalid;
  compute_tile<NT, MASK, LEAN>(Kl, Vl, nv, qf, st, c, lane);
}

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

// Byte offset, inside a stored partial row of D halves, of the four columns 4 * q .. 4 * q + 3:
// a lane of the tile routine owns columns 16 ct + 4 g .. + 3 of every column tile ct and stores the
// eight values of two neighbouring tiles as one 16-byte chunk, chunk (ct / 2) * 4 + g.
__device__ __forceinline__ int part_col_off(int q) {
  const int ct = q >> 2, g = q & 3;
  return ((ct >> 1) * 4 + g) * 16 + (ct & 1) * 8;
}

// Normalise and store one partial: rows [rowbase, rowbase + 16) of a unit with `nrows` rows.
//
// What the stores of the partials cost this kernel follows their instruction count, not their
// bytes (37 k 16-byte stores cost 14 us of 115; half as many, half; 4-byte stores in their place,
// the same), so a row of o is stored as fp16 in four instructions instead of eight.  To keep
// fp16's range out of the picture every row is first scaled by a power of two that brings its
// largest magnitude into [0.5, 1); the inverse scale is stored next to the row's lse.  The
// rounding (2^-11 of the row's largest |o|, at most 2e-3 for |v| <= 4) stays inside the
// tolerance of the bf16 path, whose weights are already rounded to bf16.
template <int NT>
__device__ __forceinline__ void write_partial(const WaveState<NT>& st, _Float16* po, float* pl, int slot, int nrows,
                                              int rowbase, int lane, float vfac) {
  const int m16 = lane & 15, g = lane >> 4;
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    float l = st.l[nt], lr = st.lr[nt];
    l += __shfl_xor(l, 16, 64);   l += __shfl_xor(l, 32, 64);
    lr += __shfl_xor(lr, 16, 64); lr += __shfl_xor(lr, 32, 64);
    float mx = 0.f;
#pragma unroll
    for (int ct = 0; ct < 8; ++ct)
#pragma unroll
      for (int x = 0; x < 4; ++x) mx = fmaxf(mx, fabsf(st.O[nt][ct][x]));
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64)); mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const int row = rowbase + 16 * nt + m16;
    if (row < nrows) {
      const float inv = vfac / lr;                           // vfac: factor of the V store (1 unless e4m3)
      const int e = clampi((int)((__float_as_uint(mx * inv) >> 23) & 255u), 1, 252);   // max |o| in [2^(e-127), 2^(e-126))
      const float k = inv * __uint_as_float((uint32_t)(253 - e) << 23);                // o * 2^(126-e) in [0.5, 1)
      char* o = reinterpret_cast<char*>(po + ((size_t)slot * nrows + row) * D);
#pragma unroll
      for (int ct = 0; ct < 8; ct += 2) {
        const f32x4 a = st.O[nt][ct] * k, b = st.O[nt][ct + 1] * k;
        const f16x8 h = {(_Float16)a[0], (_Float16)a[1], (_Float16)a[2], (_Float16)a[3],
                         (_Float16)b[0], (_Float16)b[1], (_Float16)b[2], (_Float16)b[3]};
        *reinterpret_cast<f16x8*>(o + ((ct >> 1) * 4 + g) * 16) = h;
      }
      if (g == 0)
        *reinterpret_cast<float2*>(pl + 2 * ((size_t)slot * nrows + row)) =
            make_float2((st.m[nt] + __builtin_amdgcn_logf(l)) * 0.69314718055994531f,
                        __uint_as_float((uint32_t)(e + 1) << 23));                     // 2^(e-126)
    }
  }
}

__device__ __forceinline__ u32x4 ldg16(const char* p) { return *reinterpret_cast<const u32x4*>(p); }
// K/V rows that are read exactly once per call are streamed past the caches: all suffix tiles, and the prefix
// tiles of KV groups of at most 64 rows.  A larger group reads each prefix tile once per row part; with ordinary
// loads the second read is served by the memory-side cache (160 -> 150 us per step on the 128-row workload).
// (For single-part groups ordinary prefix loads only help a benchmark that returns to the same prefix within
// the 256 MB of that cache; with more K/V in rotation they cost 1 %.)
__device__ __forceinline__ u32x4 ldg16_stream(const char* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}

// ---- how a wavefront moves one 32-key K (or V) tile from the store to LDS.
// bf16 store: 8 instructions of 16 bytes per lane, instruction i covering tile rows 4i .. 4i+3
// (16 lanes per 256-byte row).  e4m3 store: 4 instructions, instruction i covering rows 8i .. 8i+7
// (8 lanes per 128-byte row); a lane's 16 bytes become two adjacent 16-byte bf16 chunks in LDS.
template <bool F8>
struct Stage {
  static constexpr int NL = F8 ? 4 : 8;                     // load instructions per tile
  static constexpr int GROWB = F8 ? D : 2 * D;              // bytes per row in the store
  static constexpr int RS = F8 ? 8 : 4;                     // tile rows per instruction
  // instruction i of lane `lane` fetches 16 bytes: chunk chunk(lane) of tile row RS * i + lrow(lane)
  __device__ static __forceinline__ int lrow(int lane) { return F8 ? lane >> 3 : lane >> 4; }
  __device__ static __forceinline__ int chunk(int lane) { return F8 ? lane & 7 : lane & 15; }
};

// four e4m3 bytes -> four bf16 (exact: 4 significant bits, exponents inside bf16's range), with
// gfx950's packed converter: two bytes of the source word per instruction, scaled by 2^0
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x2 e4m3x4_to_bf16(uint32_t w) {
  const bf16x2 lo = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, false);   // bytes 0, 1
  const bf16x2 hi = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(w, 1.0f, true);    // bytes 2, 3
  return u32x2{*reinterpret_cast<const uint32_t*>(&lo), *reinterpret_cast<const uint32_t*>(&hi)};
}
// 16 e4m3 bytes -> two 16-byte chunks of 8 bf16
__device__ __forceinline__ void e4m3x16_to_bf16(const u32x4& w, u32x4& lo, u32x4& hi) {
  const u32x2 a = e4m3x4_to_bf16(w[0]), b = e4m3x4_to_bf16(w[1]), c = e4m3x4_to_bf16(w[2]), d = e4m3x4_to_bf16(w[3]);
  lo = u32x4{a[0], a[1], b[0], b[1]};
  hi = u32x4{c[0], c[1], d[0], d[1]};
}

// registers of one tile -> LDS (K tile at Kl, V tile at Vl), in the swizzled layout compute_tile reads
template <bool F8>
__device__ __forceinline__ void stage_store(char* Kl, char* Vl, const u32x4 (&rk)[Stage<F8>::NL],
                                            const u32x4 (&rv)[Stage<F8>::NL], int lrow, int chunk) {
#pragma unroll
  for (int i = 0; i < Stage<F8>::NL; ++i) {
    const int row = Stage<F8>::RS * i + lrow;
    if (!F8) {
      lds_st128(Kl + k_off(row, chunk), rk[i]);
      lds_st128(Vl + v_off(row, chunk), rv[i]);
    } else {
      u32x4 a, b;
      e4m3x16_to_bf16(rk[i], a, b);
      lds_st128(Kl + k_off(row, 2 * chunk), a);
      lds_st128(Kl + k_off(row, 2 * chunk + 1), b);
      e4m3x16_to_bf16(rv[i], a, b);
      lds_st128(Vl + v_off(row, 2 * chunk), a);
      lds_st128(Vl + v_off(row, 2 * chunk + 1), b);
    }
  }
}

// locate() of the partition, evaluated by a whole wavefront at once (all lanes active, same
// arguments): ballots over every 64th entry find the block of 64 entries, a ballot inside the
// block finds the entry.  Two dependent LDS reads instead of one per bisection step.
__device__ __forceinline__ void locate_wave(const int* X, int n, int Hkv, int tile, int lane, int& major, int& j,
                                            int& t) {
  int cnt = 0;                                              // blocks whose first entry is at or before `tile`
  for (int b0 = 0; b0 * 64 < n; b0 += 64) {
    const int i = (b0 + lane) * 64;
    cnt += __popcll(__ballot(i < n && X[i] * Hkv <= tile));
  }
  const int base = (cnt - 1) * 64;                          // cnt >= 1 because X[0] = 0
  const int i = base + lane;
  const int lo = base + __popcll(__ballot(i < n && X[i] * Hkv <= tile)) - 1;
  const int T = X[lo + 1] - X[lo], rem = tile - X[lo] * Hkv;
  major = lo; j = rem / T; t = rem - j * T;
}

// ---- a position on the work line: unit (u, j), tile t inside it, and the unit's size
struct Cur { int u, j, t, T, L; };                          // T tiles, L keys

template <class LenOf>
__device__ __forceinline__ void cur_load(Cur& c, LenOf len_of) {   // values are wavefront-uniform
  c.u = uni(c.u);
  c.L = uni(len_of(c.u));
  c.T = ceil_div(c.L, TK);
}
// `by` tiles forward (by <= T - t); runs on into the next non-empty unit; n prompts or sequences
template <class LenOf>
__device__ __forceinline__ void cur_step(Cur& c, int by, LenOf len_of, int n, int Hkv) {
  c.t = uni(c.t + by);
  c.j = uni(c.j);
  if (c.t < c.T) return;
  c.t = 0;
  if (++c.j < Hkv) return;
  c.j = 0;
  do {
    if (++c.u >= n) { c.T = 0; c.L = 0; return; }
    cur_load(c, len_of);
  } while (c.T == 0);
}

// ---- prefix tiles of one workgroup: `n` tiles of the line starting at `cur`.
// Tiles are staged in groups of up to WG_WAVES tiles of one unit, one LDS stage each, wavefront v
// fetching tile v of the group (so the workgroup keeps as many bytes in flight as in the suffix
// phase).  The R query rows form NRB (a power of two <= 8) blocks of 16; wavefront v computes row
// block v % NRB on stages [(v / NRB) * NRB, +NRB).  The loads of the next group (also when it
// belongs to the next unit) are issued in NRB slices between those tile computations, so that the
// memory pipeline and the matrix pipeline of the CU overlap and no bubble opens at a unit
// boundary.  When a unit's run ends, the WG_WAVES / NRB wavefronts that share a row block are
// merged through LDS and the partial is written.
// TREE: the units are segments of several levels, each with its own store, capacity and group size.
struct PrefixUnit { const char* k; const char* v; int cap, R, b0; };   // stores of the segment (all KV heads), rows, first sequence
template <int NRB, int NT, bool EXT, bool F8, bool REREAD, bool TREE>
__device__ __forceinline__ void prefix_stream(const SharedParams& P, char* lds, Cur cur, int n, int rank, int side, int tid) {
  auto len_of = [&](int p) { return plen_of<EXT, TREE>(P, p); };
  const int lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  using St = Stage<F8>;
  constexpr int NL = St::NL, GROWB = St::GROWB;
  constexpr int LPS = NL / NRB;                             // loads (of K and of V) per slice
  const int rb = wv & (NRB - 1), part = wv / NRB, s_lo = part * NRB;
  const int rowbase = 16 * NT * rb;                         // inside the unit's row half
  const int lrow = St::lrow(lane), chunk = St::chunk(lane);
  auto half_of = [&](const Cur& c) {                        // row half of the unit that this workgroup computes
    if constexpr (REREAD) return (c.j & (P.NH - 1)) * P.SM + side;
    else return c.j & (P.NH - 1);
  };
  auto head_of = [&](const Cur& c) { return c.j >> P.NHs; };
  // where the K and V rows of unit c start in their store, its query rows and its first sequence
  auto unit_of = [&](const Cur& c) {
    if constexpr (TREE) {
      const TreeLevel lv = level_of(P, c.u);
      const size_t off = (size_t)((c.u - lv.first) * P.Hkv + head_of(c)) * lv.cap * GROWB;
      return PrefixUnit{lv.k + off, lv.v + off, lv.cap, lv.R, (c.u - lv.first) * lv.G};
    } else {
      const size_t off = (size_t)(c.u * P.Hkv + head_of(c)) * P.Lp_cap * GROWB;
      return PrefixUnit{P.kp + off, P.vp + off, P.Lp_cap, P.R, c.u * P.G};
    }
  };
  constexpr bool reread = REREAD;                           // the twin pair reads the same tile: keep it cached
  char* mine = lds + wv * STAGE_B;

  constexpr bool QPRE = NT == 1;                            // query rows of the next unit are prefetched (one block per wavefront)
  u32x4 rk[NL], rv[NL], qn[QPRE ? NT : 1][4];
  bf16x8 qf[NT][4];
  WaveState<NT> st;
  float cu = P.c;                                           // score factor of the current unit
  auto issue_q = [&](const Cur& c) {                        // row = sample * r + head-in-group
    int R = P.R, b0 = c.u * P.G;
    if constexpr (TREE) { const PrefixUnit pu = unit_of(c); R = pu.R; b0 = pu.b0; }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      const int row = 64 * half_of(c) + rowbase + 16 * nt + m16;
      const bool ok = row < R;
      const int b = b0 + (ok ? row / P.r : 0), h = head_of(c) * P.r + (ok ? row % P.r : 0);
      const char* qp = P.q + ((size_t)b * P.Hq + h) * ROWB + 16 * g;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const u32x4 v = ok ? ldg16(qp + 64 * ks) : u32x4{0, 0, 0, 0};
        if (QPRE) qn[nt][ks] = v; else qf[nt][ks] = *reinterpret_cast<const bf16x8*>(&v);
      }
    }
  };
  auto group_size = [&](const Cur& c, int rem) { return min(min(WG_WAVES, c.T - c.t), rem); };

  int rem = n, gs = group_size(cur, rem);
  if (QPRE) issue_q(cur);
  if (wv < gs) {
    const PrefixUnit pu = unit_of(cur);
    const char* kb = pu.k;
    const char* vb = pu.v;
    const int key0 = (cur.t + wv) * TK, last = min(TK, cur.L - key0) - 1;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const size_t off = (size_t)(key0 + min(St::RS * i + lrow, last)) * GROWB + 16 * chunk;
      if constexpr (reread) { rk[i] = ldg16(kb + off); rv[i] = ldg16(vb + off); }
      else                  { rk[i] = ldg16_stream(kb + off); rv[i] = ldg16_stream(vb + off); }
    }
  }
  bool fresh = true;
  while (rem > 0) {
    const bool active = 64 * half_of(cur) + rowbase < (TREE ? unit_of(cur).R : P.R);   // this wavefront's row block exists in the unit's half
    wait_vmem();
    if (wv < gs) stage_store<F8>(mine, mine + TILE_B, rk, rv, lrow, chunk);
    if (fresh) {
      if (F8 && P.kscale) cu = P.c * P.kscale[head_of(cur)];
      if (QPRE) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
          for (int ks = 0; ks < 4; ++ks) qf[nt][ks] = *reinterpret_cast<bf16x8*>(&qn[nt][ks]);
      } else {
        issue_q(cur);
        wait_vmem();
      }
      init_state(st);
    }
    Cur nxt = cur;
    const int rem2 = rem - gs;
    int ngs = 0;
    bool next_fresh = false;
    if (rem2 > 0) {
      cur_step(nxt, gs, len_of, P.P, P.HkvP);
      ngs = group_size(nxt, rem2);
      next_fresh = nxt.u != cur.u || nxt.j != cur.j;
    }
    lds_barrier();
    if (QPRE && next_fresh) issue_q(nxt);
    const bool more = wv < ngs;                             // this wavefront fetches a tile of the next group
    const PrefixUnit pn = unit_of(nxt);
    const char* kb = pn.k;
    const char* vb = pn.v;
    const int key0 = (nxt.t + wv) * TK, last = min(TK, nxt.L - key0) - 1;
    // the upper half of the wavefronts issues a slice before each tile computation, the lower half
    // after it, so that they alternate between the memory pipeline and the matrix pipeline
    const bool first = wv >= WG_WAVES / 2;
    auto slice = [&](int k) {
#pragma unroll
      for (int i = 0; i < NL; ++i) {                        // rows past the length re-read the last real row
        if (i >= k * LPS && i < (k + 1) * LPS) {
          const size_t off = (size_t)(key0 + min(St::RS * i + lrow, last)) * GROWB + 16 * chunk;
          if constexpr (reread) { rk[i] = ldg16(kb + off); rv[i] = ldg16(vb + off); }
          else                  { rk[i] = ldg16_stream(kb + off); rv[i] = ldg16_stream(vb + off); }
        }
      }
    };
#pragma unroll
    for (int k = 0; k < NRB; ++k) {
      const int s = s_lo + k;
      if (more && first) slice(k);
      if (active && s < gs)
        compute_tile<NT, true, true>(lds + s * STAGE_B, lds + s * STAGE_B + TILE_B, min(TK, cur.L - (cur.t + s) * TK), qf, st,
                        F8 ? cu : P.c, lane);
      if (more && !first) slice(k);
    }
    lds_barrier();                                          // stages are rewritten by the next group
    if (rem2 == 0 || next_fresh) {                          // the unit's run ends here
      // parts > 0 park their state in their own stage, lane-major (the part-0 wavefront reads with
      // the same lane index), then part 0 folds them in
      if (NRB < WG_WAVES) {
        float* park = reinterpret_cast<float*>(mine);
        constexpr int PW = 35 * 64;                         // floats parked per row block
        if (part > 0 && active) {
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
            for (int ct = 0; ct < 8; ++ct)
#pragma unroll
              for (int x = 0; x < 4; ++x) park[nt * PW + (ct * 4 + x) * 64 + lane] = st.O[nt][ct][x];
            park[nt * PW + 32 * 64 + lane] = st.m[nt];
            park[nt * PW + 33 * 64 + lane] = st.l[nt];
            park[nt * PW + 34 * 64 + lane] = st.lr[nt];
          }
        }
        lds_barrier();
        if (part == 0 && active) {
          for (int pp = 1; pp < WG_WAVES / NRB; ++pp) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
              const float* o = reinterpret_cast<const float*>(lds + (pp * NRB + rb) * STAGE_B) + nt * PW;
              const float m2 = o[32 * 64 + lane];
              if (__all(m2 == -INFINITY)) continue;         // that wavefront had no tile in this run
              const float mn = fmaxf(st.m[nt], m2);
              const float a1 = __builtin_amdgcn_exp2f(st.m[nt] - mn), a2 = __builtin_amdgcn_exp2f(m2 - mn);
#pragma unroll
              for (int ct = 0; ct < 8; ++ct)
#pragma unroll
                for (int x = 0; x < 4; ++x)
                  st.O[nt][ct][x] = st.O[nt][ct][x] * a1 + o[(ct * 4 + x) * 64 + lane] * a2;
              st.l[nt] = st.l[nt] * a1 + o[33 * 64 + lane] * a2;
              st.lr[nt] = st.lr[nt] * a1 + o[34 * 64 + lane] * a2;
              st.m[nt] = mn;
            }
          }
        }
        lds_barrier();                                      // parked state is dead before tiles are stored again
      }
      if (active && part == 0)
        write_partial<NT>(st, P.po, P.pl, REREAD ? (cur.u * P.HkvP + cur.j + rank) * P.SM + side : cur.u * P.HkvP + cur.j + rank,
                          P.RS, rowbase, lane,
                          F8 && P.vscale ? P.vscale[head_of(cur)] : 1.f);
    }
    fresh = next_fresh; cur = nxt; rem = rem2; gs = ngs;
  }
}

// ---- suffix tiles of one wavefront: `n` tiles of the line starting at `cur`, streamed through the
// wavefront's private 16 KB of LDS.  The loads of tile i + 1 (and the query rows of its unit when
// it starts a new one) are in flight while tile i is computed, across unit boundaries as well.
// `flush`: this wavefront writes its die's L2 back once its first tile has landed, see below.
template <bool EXT, bool F8>
__device__ __forceinline__ void suffix_stream(const SharedParams& P, char* wlds, Cur cur, int n, int slot_base,
                                              int lane, bool flush) {
  auto len_of = [&](int b) { return slen_of<EXT>(P, b); };
  using St = Stage<F8>;
  constexpr int NL = St::NL, GROWB = St::GROWB;
  const int m16 = lane & 15, g = lane >> 4, lrow = St::lrow(lane), chunk = St::chunk(lane);
  u32x4 rk[NL], rv[NL], qn[4];
  bf16x8 qf[1][4];
  WaveState<1> st;
  float cu = P.c;                                           // score factor of the current unit
  auto issue_q = [&](const Cur& c) {
    const bool ok = m16 < P.r;
    const char* qp = P.q + ((size_t)c.u * P.Hq + c.j * P.r + (ok ? m16 : 0)) * ROWB + 16 * g;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) qn[ks] = ok ? ldg16(qp + 64 * ks) : u32x4{0, 0, 0, 0};
  };
  auto issue_tile = [&](const Cur& c) {                     // every instruction fetches 1 KB of contiguous rows
    const int key0 = c.t * TK, last = min(TK, c.L - key0) - 1;
    size_t row0 = (size_t)(c.u * P.Hkv + c.j) * P.Ls_cap + key0;      // first row of the tile in the store
    if (EXT && P.table) {                                   // a tile never straddles pages: TK divides the page size
      const int pg = uni(clampi(P.table[(size_t)c.u * P.max_pages + (key0 >> P.page_shift)], 0, P.n_pages - 1));
      row0 = (((size_t)pg * P.Hkv + c.j) << P.page_shift) + (key0 & ((1 << P.page_shift) - 1));
    }
    const char* kb = P.ks + row0 * GROWB;
    const char* vb = P.vs + row0 * GROWB;
#pragma unroll
    for (int i = 0; i < NL; ++i) {                          // rows past the length re-read the last real row
      const size_t off = (size_t)min(St::RS * i + lrow, last) * GROWB + 16 * chunk;
      rk[i] = ldg16_stream(kb + off);
      rv[i] = ldg16_stream(vb + off);
    }
  };
  issue_q(cur);
  issue_tile(cur);
  // The partial rows stored so far sit in this die's L2 as dirty lines.  Left alone they trickle out one
  // by one under the read stream, and such lone write-backs cost the stream far more than their bytes
  // (measured at the 7B shape: the K/V stream runs at 6.2 TB/s for the rest of the kernel once the
  // workgroups have stored their prefix partials, against 7.0-7.5 TB/s when the lines are written back
  // in one go; stores that write through cost more than that single write-back).  An agent-scope
  // release is that write-back; one wavefront per die issues it (more than one per die only adds cost),
  // a tile's round trip after its own workgroup's prefix partial.
  if (flush) {
    wait_vmem();
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
  }
  bool fresh = true;
  for (int i = 0; i < n; ++i) {
    wait_vmem();
    stage_store<F8>(wlds, wlds + TILE_B, rk, rv, lrow, chunk);
    if (fresh) {
      if (F8 && P.kscale) cu = P.c * P.kscale[cur.j];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) qf[0][ks] = *reinterpret_cast<bf16x8*>(&qn[ks]);
      init_state(st);
    }
    Cur nxt = cur;
    const bool has_next = i + 1 < n;
    bool next_fresh = false;
    if (has_next) {
      cur_step(nxt, 1, len_of, P.B, P.Hkv);
      next_fresh = nxt.u != cur.u || nxt.j != cur.j;
      if (next_fresh) issue_q(nxt);
      issue_tile(nxt);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    compute_tile<1, true, true>(wlds, wlds + TILE_B, min(TK, cur.L - cur.t * TK), qf, st, F8 ? cu : P.c, lane);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    if (!has_next || next_fresh)
      write_partial<1>(st, P.so, P.sl, cur.u * P.Hkv + cur.j + slot_base, P.r, 0, lane,
                       F8 && P.vscale ? P.vscale[cur.j] : 1.f);
    fresh = next_fresh; cur = nxt;
  }
}

template <int NRB, int NT, bool EXT, bool F8, bool REREAD = false, bool TREE = false>   // REREAD: KV groups of several row halves (NRB = 4), dual partition
__global__ void __launch_bounds__(NTHREADS, 2) partial_kernel(const SharedParams P) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  __shared__ int wsum[WG_WAVES];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;

  // ---- tile counts of all prompts and sequences, exclusive scan in LDS: every thread takes a
  // run of consecutive entries, the runs are chained by a wavefront scan and the wavefront totals
  int* X = reinterpret_cast<int*>(lds);
  const int n = P.P + P.B + 1;
  {
    const int per = ceil_div(n, NTHREADS);
    const int c0 = min(tid * per, n), c1 = min(c0 + per, n);
    int sum = 0;
    for (int i = c0; i < c1; ++i) {
      int e = 0;
      if (i < P.P) e = ceil_div(plen_of<EXT, TREE>(P, i), TK);
      else if (i < P.P + P.B) e = ceil_div(slen_of<EXT>(P, i - P.P), TK);
      X[i] = e;                                             // read back below by this thread only
      sum += e;
    }
    int incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const int t = __shfl_up(incl, o, 64);
      if (lane >= o) incl += t;
    }
    if (lane == 63) wsum[wv] = incl;
    __syncthreads();
    int off = incl - sum;
    for (int k = 0; k < wv; ++k) off += wsum[k];
    for (int i = c0; i < c1; ++i) { const int e = X[i]; X[i] = off; off += e; }
  }
  __syncthreads();
  const int cumP = X[P.P];
  const Sched sc = make_sched(cumP * P.HkvP, (X[P.P + P.B] - cumP) * P.Hkv, P.n_cu, REREAD && P.SM == 2);
  if (blockIdx.x == 0) for (int i = tid; i < n; i += NTHREADS) P.cum[i] = X[i];
  // a small batch works with the first half of the grid (never in the dual partition)
  const int w = REREAD ? (int)blockIdx.x : wg_name(sc, blockIdx.x);

  // ---- where this workgroup's prefix tiles and this wavefront's suffix tiles start
  int ilo, ihi, klo, khi, ka, kb;
  wg_prefix_range(sc, w, ilo, ihi);
  wg_suffix_range(sc, w, klo, khi);
  wave_suffix_range(klo, khi, wv, ka, kb);
  int pp = 0, pj = 0, pt = 0, sb = 0, sj = 0, st0 = 0;
  if (ilo < ihi) locate_wave(X, P.P, P.HkvP, ilo, lane, pp, pj, pt);
  if (ka < kb) {
    locate_wave(X + P.P, P.B, P.Hkv, ka + cumP * P.Hkv, lane, sb, sj, st0);   // X + P continues the prompt scan: shift the line
  }
  pp = uni(pp); pj = uni(pj); pt = uni(pt); sb = uni(sb); sj = uni(sj); st0 = uni(st0);
  __syncthreads();                                          // the scan is dead; LDS becomes tile storage

  // ---- prefix tiles of this workgroup (ends with a workgroup barrier), then the suffix tiles of
  // each wavefront in its own stage of the LDS
  if (ilo < ihi) {
    Cur c{pp, pj, pt, 0, 0};
    cur_load(c, [&](int p) { return plen_of<EXT, TREE>(P, p); });
    prefix_stream<NRB, NT, EXT, F8, REREAD, TREE>(P, lds, c, ihi - ilo, wg_prefix_rank(sc, w),
                                                  REREAD ? prefix_side(sc, wg_pair(sc, w)) : 0, tid);
  }
  if (ka < kb) {
    Cur c{sb, sj, st0, 0, 0};
    cur_load(c, [&](int b) { return slen_of<EXT>(P, b); });
    // Workgroup i runs on die i % (n_cu / CU_PER_DIE).  The first wavefront of the first workgroup on each die writes that
    // die's L2 back when its first suffix tile has landed: the workgroups of the die have stored their prefix
    // partials by then (all carry the same number of prefix tiles).  A wrong guess about which die a workgroup
    // is on only makes the write-back less useful.
    suffix_stream<EXT, F8>(P, lds + wv * STAGE_B, c, kb - ka, WG_WAVES * wg_rank(sc, w) + wv, lane,
                           ilo < ihi && w * CU_PER_DIE < P.n_cu && wv == 0);
  }
}

// ---- combine: 32 lanes per (sequence, head) row.  Lane k of the row first owns part k: all lse
// values of the row and the first sixteen parts' values are requested in one round trip (rows of a
// small batch are cut into that many parts, and every further round trip shows in its step time); the lse
// values become weights with two 32-lane reductions; then every lane accumulates its 4 columns.  Parts are taken in line order, so the sum has one fixed order.
template <bool EXT, bool TREE = false>
__global__ void __launch_bounds__(256) combine_kernel(const SharedParams P) {
  const int row = blockIdx.x * 8 + (threadIdx.x >> 5);
  const int sub = threadIdx.x & 31, c4 = sub * 4;
  const int coff = part_col_off(sub);                       // where this lane's 4 columns sit in a stored partial row
  if (row >= P.B * P.Hq) return;
  const int b = fast_div(row, P.div_Hq), h = row - b * P.Hq;
  if (EXT && P.active && P.active[b] == 0) {               // finished sequence: its prefix rows were computed, not used
    *reinterpret_cast<float4*>(P.out + (size_t)row * D + c4) = make_float4(0.f, 0.f, 0.f, 0.f);
    if (P.lse && c4 == 0) P.lse[row] = -INFINITY;
    return;
  }
  const int p = fast_div(b, P.div_G), gs = b - p * P.G, j = fast_div(h, P.div_r), hi_ = h - j * P.r;
  const int* X = P.cum;
  const int cumP = X[P.P];
  const Sched sc = make_sched(cumP * P.HkvP, (X[P.P + P.B] - cumP) * P.Hkv, P.n_cu, P.SM == 2);
  const int grow = gs * P.r + hi_;                          // row inside the KV group: sample-major
  const int half = P.RS == 64 ? grow >> 6 : 0, prow = grow - 64 * half;   // row half, row inside it
  const int jp = j * P.NH + (half >> (P.SM - 1)), side = half & (P.SM - 1);  // its unit on the line, which twin computes it

  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float M = -INFINITY, Z = 0.f;                             // running max and sum over batches of 32 parts
  for (int base = 0;; base += 32) {
    // part `base + sub` of this row, as 2 * (row index in its partial array) + [suffix]
    int n = 0, mine = -1;
    if constexpr (TREE) {                                   // the row's segment on every level, in level order
#pragma unroll
      for (int l = 0; l < MAX_LEVELS; ++l) {
        if (l < P.n_lev) {
          const int e = P.lev[l].first + b / P.lev[l].G, erow = (b % P.lev[l].G) * P.r + hi_;
          for_each_prefix_part(sc, X, P.Hkv, e, j, 0, [&](int c) {
            if (n == base + sub) mine = 2 * ((e * P.Hkv + j + c) * P.RS + erow);
            ++n;
          });
        }
      }
    } else {
      for_each_prefix_part(sc, X, P.HkvP, p, jp, side, [&](int c) {
        if (n == base + sub) mine = 2 * (((p * P.HkvP + jp + c) * P.SM + side) * P.RS + prow);
        ++n;
      });
    }
    for_each_suffix_part(sc, X + P.P, cumP, P.Hkv, b, j, [&](int rank, int v) {
      if (n == base + sub) mine = 2 * ((b * P.Hkv + j + WG_WAVES * rank + v) * P.r + hi_) + 1;
      ++n;
    });
    const int cnt = min(n - base, 32);
    if (cnt <= 0) break;
    // the first FIRST parts' values are requested together with the lse values (one round trip)
    constexpr int FIRST = 16, NEXT = 8;
    f16x4 v8[FIRST];
#pragma unroll
    for (int u = 0; u < FIRST; ++u) {
      const int id = __shfl(mine, min(u, cnt - 1), 32);
      v8[u] = *reinterpret_cast<const f16x4*>(reinterpret_cast<const char*>((id & 1 ? P.so : P.po) + (size_t)(id >> 1) * D) + coff);
    }
    const float2 ls = mine < 0 ? make_float2(-INFINITY, 0.f)
                               : *reinterpret_cast<const float2*>((mine & 1 ? P.sl : P.pl) + 2 * (size_t)(mine >> 1));
    const float l = ls.x;
    float m = l;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 32));
    const float Mn = fmaxf(M, m);                           // finite: every part holds at least one key
    const float resc = __expf(M - Mn);
    const float wgt = __expf(l - Mn);                       // lanes without a part: 0
    const float wsc = wgt * ls.y;                           // weight times the stored row's scale
    float zs = wgt;
#pragma unroll
    for (int o = 16; o > 0; o >>= 1) zs += __shfl_xor(zs, o, 32);
    Z = Z * resc + zs;
    M = Mn;
    acc.x *= resc; acc.y *= resc; acc.z *= resc; acc.w *= resc;
#pragma unroll
    for (int u = 0; u < FIRST; ++u) {
      const float wk = u < cnt ? __shfl(wsc, min(u, cnt - 1), 32) : 0.f;
      acc.x = fmaf(wk, (float)v8[u][0], acc.x); acc.y = fmaf(wk, (float)v8[u][1], acc.y);
      acc.z = fmaf(wk, (float)v8[u][2], acc.z); acc.w = fmaf(wk, (float)v8[u][3], acc.w);
    }
    for (int k0 = FIRST; k0 < cnt; k0 += NEXT) {
      f16x4 v[NEXT];
      float wk[NEXT];
#pragma unroll
      for (int u = 0; u < NEXT; ++u) {
        const int k = min(k0 + u, cnt - 1);
        const int id = __shfl(mine, k, 32);
        wk[u] = k0 + u < cnt ? __shfl(wsc, k, 32) : 0.f;
        v[u] = *reinterpret_cast<const f16x4*>(reinterpret_cast<const char*>((id & 1 ? P.so : P.po) + (size_t)(id >> 1) * D) + coff);
      }
#pragma unroll
      for (int u = 0; u < NEXT; ++u) {
        acc.x = fmaf(wk[u], (float)v[u][0], acc.x); acc.y = fmaf(wk[u], (float)v[u][1], acc.y);
        acc.z = fmaf(wk[u], (float)v[u][2], acc.z); acc.w = fmaf(wk[u], (float)v[u][3], acc.w);
      }
    }
    if (n - base <= 32) break;
  }
  const float inv = Z > 0.f ? 1.f / Z : 0.f;
  *reinterpret_cast<float4*>(P.out + (size_t)row * D + c4) = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
  if (P.lse && c4 == 0) P.lse[row] = Z > 0.f ? M + __logf(Z) : -INFINITY;
}

// from this many prefix units (prompts x KV heads x row parts) on, rows have few enough parts for combine16_kernel
constexpr int COMBINE16_MIN_UNITS = 128;

// ---- the same with 16 lanes per row and 16 rows per workgroup, for batches of many units, whose rows
// have few parts (a prefix unit is cut into about 1 + N_WG / units parts): half the wavefronts, so that
// 2048 x 16 rows are one resident generation of workgroups instead of two, at the price of a shallower
// first request (four parts instead of sixteen), which rows of many parts would pay in round trips.  Lane k of the row first owns part k:
// all lse values of the row and the first four parts' values are requested in one round trip; the lse
// values become weights with two 16-lane reductions; then every lane accumulates its 8 columns, one
// 16-byte chunk of every stored partial row.  Parts are taken in line order, so the sum has one fixed order.
template <bool EXT>
__global__ void __launch_bounds__(256, 8) combine16_kernel(const SharedParams P) {
  const int row = blockIdx.x * 16 + (threadIdx.x >> 4);
  const int sub = threadIdx.x & 15;
  const int coff = 16 * sub;                                // chunk `sub` of a stored partial row holds columns
  const int ca = 32 * (sub >> 2) + 4 * (sub & 3), cb = ca + 16;   // ca .. ca+3 and cb .. cb+3 (see part_col_off)
  if (row >= P.B * P.Hq) return;
  const int b = fast_div(row, P.div_Hq), h = row - b * P.Hq;
  float* orow = P.out + (size_t)row * D;
  if (EXT && P.active && P.active[b] == 0) {               // finished sequence: its prefix rows were computed, not used
    *reinterpret_cast<float4*>(orow + ca) = make_float4(0.f, 0.f, 0.f, 0.f);
    *reinterpret_cast<float4*>(orow + cb) = make_float4(0.f, 0.f, 0.f, 0.f);
    if (P.lse && sub == 0) P.lse[row] = -INFINITY;
    return;
  }
  const int p = fast_div(b, P.div_G), gs = b - p * P.G, j = fast_div(h, P.div_r), hi_ = h - j * P.r;
  const int* X = P.cum;
  const int cumP = X[P.P];
  const Sched sc = make_sched(cumP * P.HkvP, (X[P.P + P.B] - cumP) * P.Hkv, P.n_cu, P.SM == 2);
  const int grow = gs * P.r + hi_;                          // row inside the KV group: sample-major
  const int half = P.RS == 64 ? grow >> 6 : 0, prow = grow - 64 * half;   // row half, row inside it
  const int jp = j * P.NH + (half >> (P.SM - 1)), side = half & (P.SM - 1);  // its unit on the line, which twin computes it

  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float M = -INFINITY, Z = 0.f;                             // running max and sum over batches of 16 parts
  auto part_values = [&](int id) {
    return *reinterpret_cast<const f16x8*>(reinterpret_cast<const char*>((id & 1 ? P.so : P.po) + (size_t)(id >> 1) * D) + coff);
  };
  for (int base = 0;; base += 16) {
    // part `base + sub` of this row, as 2 * (row index in its partial array) + [suffix]
    int n = 0, mine = -1;
    for_each_prefix_part(sc, X, P.HkvP, p, jp, side, [&](int c) {
      if (n == base + sub) mine = 2 * (((p * P.HkvP + jp + c) * P.SM + side) * P.RS + prow);
      ++n;
    });
    for_each_suffix_part(sc, X + P.P, cumP, P.Hkv, b, j, [&](int rank, int v) {
      if (n == base + sub) mine = 2 * ((b * P.Hkv + j + WG_WAVES * rank + v) * P.r + hi_) + 1;
      ++n;
    });
    const int cnt = min(n - base, 16);
    if (cnt <= 0) break;
    // the first 4 parts' values are requested together with the lse values (one round trip)
    f16x8 v4[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v4[u] = part_values(__shfl(mine, min(u, cnt - 1), 16));
    const float2 ls = mine < 0 ? make_float2(-INFINITY, 0.f)
                               : *reinterpret_cast<const float2*>((mine & 1 ? P.sl : P.pl) + 2 * (size_t)(mine >> 1));
    const float l = ls.x;
    float m = l;
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, 16));
    const float Mn = fmaxf(M, m);                           // finite: every part holds at least one key
    const float resc = __expf(M - Mn);
    const float wgt = __expf(l - Mn);                       // lanes without a part: 0
    const float wsc = wgt * ls.y;                           // weight times the stored row's scale
    float zs = wgt;
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) zs += __shfl_xor(zs, o, 16);
    Z = Z * resc + zs;
    M = Mn;
#pragma unroll
    for (int x = 0; x < 8; ++x) acc[x] *= resc;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const float wk = u < cnt ? __shfl(wsc, min(u, cnt - 1), 16) : 0.f;
#pragma unroll
      for (int x = 0; x < 8; ++x) acc[x] = fmaf(wk, (float)v4[u][x], acc[x]);
    }
    for (int k0 = 4; k0 < cnt; k0 += 4) {
      f16x8 v[4];
      float wk[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int k = min(k0 + u, cnt - 1);
        wk[u] = k0 + u < cnt ? __shfl(wsc, k, 16) : 0.f;
        v[u] = part_values(__shfl(mine, k, 16));
      }
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int x = 0; x < 8; ++x) acc[x] = fmaf(wk[u], (float)v[u][x], acc[x]);
    }
    if (n - base <= 16) break;
  }
  const float inv = Z > 0.f ? 1.f / Z : 0.f;
  *reinterpret_cast<float4*>(orow + ca) = make_float4(acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
  *reinterpret_cast<float4*>(orow + cb) = make_float4(acc[4] * inv, acc[5] * inv, acc[6] * inv, acc[7] * inv);
  if (P.lse && sub == 0) P.lse[row] = Z > 0.f ? M + __logf(Z) : -INFINITY;
}

// ---- prefill: causal attention of a prompt over itself, computed once per prompt (its K/V are the
// shared prefix store of the decode steps).  One workgroup per (prompt, KV head, block of QB query
// positions): the QB * r rows (position-major, then query head of the group) form up to four
// 16-row blocks, one per wavefront, and share every K/V tile through LDS exactly as the G * r rows
// of a decode group do in prefix_stream; a lane's row sees the keys below its own limit
// (position + 1).  No key split: a workgroup walks all tiles up to its last position, so rows are
// normalised and written directly.  All blocks of one (prompt, KV head) run on one XCD, one unit
// after the other, from the end of the prompt (most tiles) to its start: workgroups are dealt to
// the eight XCDs round-robin, so workgroup i belongs to XCD i % 8 and is the (i / 8)-th of its XCD;
// with the units of an XCD laid out one after the other along that sequence, the 64 or so
// workgroups an XCD runs at a time read the same K/V (a few hundred KB), which then stays in its
// L2.  (Measured: spreading them over many units at a time made the pass wait on the fabric.)
struct PrefillParams {
  const char* q; const char* k; const char* v; const int32_t* lens;
  float* out; float* lse;
  int P, Hq, Hkv, r, Lp_cap, QB, nqb;
  float c;
};

template <int NTP>                                          // 16-row blocks per wavefront: the workgroup holds 64 * NTP rows
__global__ void __launch_bounds__(NTHREADS, 2) prefill_kernel(const PrefillParams P) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  constexpr int N_XCD = 8, WROWS = 16 * NTP;                // rows per wavefront
  const int units = P.P * P.Hkv;
  const int xcd = blockIdx.x % N_XCD, seq = blockIdx.x / N_XCD;
  const int pj = (seq / P.nqb) * N_XCD + xcd, qb = P.nqb - 1 - seq % P.nqb;
  if (pj >= units) return;                                  // the last round of units may not fill all XCDs
  const int p = pj / P.Hkv, j = pj % P.Hkv;
  const int L = clampi(P.lens[p], 0, P.Lp_cap), a = qb * P.QB;
  if (a >= L) return;                                       // the whole block is padding (same decision in every thread)
  const int nq = min(P.QB, L - a), n_keys = a + nq, n_tiles = ceil_div(n_keys, TK), nrows = nq * P.r;
  // this lane's query rows, one per block
  bool ok[NTP];
  int pos[NTP], h[NTP], limit[NTP];
  bf16x8 qf[NTP][4];
#pragma unroll
  for (int nt = 0; nt < NTP; ++nt) {
    const int row = WROWS * wv + 16 * nt + m16;
    ok[nt] = row < nrows;
    pos[nt] = a + (ok[nt] ? row / P.r : 0);
    h[nt] = j * P.r + (ok[nt] ? row % P.r : 0);
    limit[nt] = pos[nt] + 1;                                // keys [0, limit) are visible; rows that do not exist see key 0 only
    const char* qp = P.q + (((size_t)p * P.Lp_cap + pos[nt]) * P.Hq + h[nt]) * ROWB + 16 * g;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const u32x4 v = ok[nt] ? ldg16(qp + 64 * ks) : u32x4{0, 0, 0, 0};
      qf[nt][ks] = *reinterpret_cast<const bf16x8*>(&v);
    }
  }
  const int wave_last = a + min(nrows - 1, WROWS * wv + WROWS - 1) / P.r;   // last position any row of this wavefront holds (uniform)
  const int wave_first = a + (WROWS * wv) / P.r;            // first position; rows that do not exist see less, but are not stored
  const bool wave_has_rows = WROWS * wv < nrows;
  const char* kb = P.k + (size_t)(p * P.Hkv + j) * P.Lp_cap * ROWB;
  const char* vb = P.v + (size_t)(p * P.Hkv + j) * P.Lp_cap * ROWB;
  const int lrow = lane >> 4, chunk = lane & 15;
  u32x4 rk[8], rv[8];
  const size_t lane_off = (size_t)lrow * ROWB + 16 * chunk; // this lane's 16 bytes inside a group of four rows
  auto issue = [&](int t) {                                 // tile t (if it exists) into this wavefront's registers
    if (t >= n_tiles) return;
    const int key0 = t * TK;
    if (key0 + TK <= n_keys) {                              // a whole tile: one base per store, constant offsets
      const char* kt = kb + (size_t)key0 * ROWB + lane_off;
      const char* vt = vb + (size_t)key0 * ROWB + lane_off;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        rk[i] = ldg16(kt + i * 4 * ROWB);                   // the prompt's K/V are read by all its blocks: keep them cached
        rv[i] = ldg16(vt + i * 4 * ROWB);
      }
    } else {                                                // the last, partial tile: rows past the end re-read the last real row
      const int last = n_keys - key0 - 1;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const size_t off = (size_t)(key0 + min(4 * i + lrow, last)) * ROWB + 16 * chunk;
        rk[i] = ldg16(kb + off);
        rv[i] = ldg16(vb + off);
      }
    }
  };
  WaveState<NTP> st;
  init_state(st);
  char* mine = lds + wv * STAGE_B;
  issue(wv);
  for (int g0 = 0; g0 < n_tiles; g0 += WG_WAVES) {
    wait_vmem();
    if (g0 + wv < n_tiles) stage_store<false>(mine, mine + TILE_B, rk, rv, lrow, chunk);
    lds_barrier();
    issue(g0 + WG_WAVES + wv);                              // next group in flight during the arithmetic
#pragma unroll
    for (int s2 = 0; s2 < WG_WAVES; ++s2) {
      const int key0 = (g0 + s2) * TK;
      if (g0 + s2 < n_tiles && wave_has_rows && key0 <= wave_last) {     // tiles wholly in this wavefront's future are skipped
        if (key0 + TK <= wave_first + 1) {                               // wholly in every row's past: no masks
          compute_tile<NTP, false>(lds + s2 * STAGE_B, lds + s2 * STAGE_B + TILE_B, TK, qf, st, P.c, lane);
        } else {
          int nv[NTP];
#pragma unroll
          for (int nt = 0; nt < NTP; ++nt) nv[nt] = limit[nt] - key0;
          compute_tile<NTP>(lds + s2 * STAGE_B, lds + s2 * STAGE_B + TILE_B, nv, qf, st, P.c, lane);
        }
      }
    }
    lds_barrier();                                          // stages are rewritten by the next group
  }
  // normalise and write the rows
#pragma unroll
  for (int nt = 0; nt < NTP; ++nt) {
    float l = st.l[nt], lr = st.lr[nt];
    l += __shfl_xor(l, 16, 64);   l += __shfl_xor(l, 32, 64);
    lr += __shfl_xor(lr, 16, 64); lr += __shfl_xor(lr, 32, 64);
    if (ok[nt]) {
      const float inv = 1.f / lr;
      const size_t orow = ((size_t)p * P.Lp_cap + pos[nt]) * P.Hq + h[nt];
      float* o = P.out + orow * D + 4 * g;
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const f32x4 v = st.O[nt][ct] * inv;
        *reinterpret_cast<float4*>(o + 16 * ct) = make_float4(v[0], v[1], v[2], v[3]);
      }
      if (P.lse && g == 0) P.lse[orow] = (st.m[nt] + __builtin_amdgcn_logf(l)) * 0.69314718055994531f;
    }
  }
}

// ---- prefill, 128 rows per workgroup, K/V tiles moved from the store straight into LDS.
//
// What bounds prefill_kernel is not one unit but the order of a wavefront's own work: LDS read
// latency, matrix products and vector ALU follow each other, and at 256 registers two wavefronts per
// SIMD is all there is to overlap them.  The 64 registers that stage a K/V tile are what stands in
// the way of issuing the LDS reads of the next phase a phase ahead, so here the tiles take the
// direct path: global_load_lds_dwordx4 writes a lane's 16 bytes to LDS at (uniform base) + 16 * lane,
// and the layout's xor pattern, being a permutation of the 16 chunks of a row, goes into the lane's
// global address instead.  The compiler cannot tell which LDS bytes such a load writes and would make
// every later LDS read wait for all of them; the fragment reads are therefore issued as asm, with
// explicit waits that carry the destination registers as operands so that no use is moved above them.
//
// Schedule of a wavefront (tile t in stage t % 4; rounds of two tiles; buffer = round % 2):
//     row maxima (t) | V(t) reads issued | weights and sums (t) | wait V(t) | [end of round: loads landed, barrier, issue the
//     loads of round + 2 into the buffer just finished] | K(t+1) reads issued | value products (t) |
//     wait K(t+1) | score products (t+1)
// so that LDS latency lies under the vector ALU (V) and the matrix unit (K), and the matrix work of
// one tile's second product and the next tile's first product is one uninterrupted run for the other
// wavefront of the SIMD to put its softmax under.  Wavefront w moves the K (even w) or V (odd w) half
// of tile w / 2 of a round.
template <int OFF>
__device__ __forceinline__ bf16x8 lds_rd128_asm(uint32_t addr) {
  bf16x8 v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
template <int OFF>
__device__ __forceinline__ s16x4 lds_rd_tr16_asm(uint32_t addr) {
  s16x4 v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
__device__ __forceinline__ void wait_k_frags(bf16x8 (&k)[4][2]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(k[0][0]), "+v"(k[0][1]), "+v"(k[1][0]), "+v"(k[1][1]), "+v"(k[2][0]), "+v"(k[2][1]), "+v"(k[3][0]), "+v"(k[3][1]));
}
__device__ __forceinline__ void wait_v_frags(s16x4 (&v)[8][2]) {
  asm volatile("s_waitcnt lgkmcnt(0)"
               : "+v"(v[0][0]), "+v"(v[0][1]), "+v"(v[1][0]), "+v"(v[1][1]), "+v"(v[2][0]), "+v"(v[2][1]), "+v"(v[3][0]), "+v"(v[3][1]),
                 "+v"(v[4][0]), "+v"(v[4][1]), "+v"(v[5][0]), "+v"(v[5][1]), "+v"(v[6][0]), "+v"(v[6][1]), "+v"(v[7][0]), "+v"(v[7][1]));
}
template <int STAGE>
__device__ __forceinline__ void read_k_frags(const uint32_t (&ka)[4], bf16x8 (&k)[4][2]) {
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    k[ks][0] = lds_rd128_asm<STAGE * STAGE_B>(ka[ks]);
    k[ks][1] = lds_rd128_asm<STAGE * STAGE_B + 16 * ROWB>(ka[ks]);
  }
}
template <int STAGE>
__device__ __forceinline__ void read_v_frags(const uint32_t (&va)[8], s16x4 (&v)[8][2]) {
#pragma unroll
  for (int ct = 0; ct < 8; ++ct) {
    v[ct][0] = lds_rd_tr16_asm<STAGE * STAGE_B + TILE_B>(va[ct]);
    v[ct][1] = lds_rd_tr16_asm<STAGE * STAGE_B + TILE_B + 16 * ROWB>(va[ct]);
  }
}
template <int NT>
__device__ __forceinline__ void score_products(const bf16x8 (&k)[4][2], const bf16x8 (&qf)[NT][4], f32x4 (&s0)[NT], f32x4 (&s1)[NT]) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) { s0[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; s1[nt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
      s0[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[ks][0], qf[nt][ks], s0[nt], 0, 0, 0);
      s1[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k[ks][1], qf[nt][ks], s1[nt], 0, 0, 0);
    }
}
template <int NT>
__device__ __forceinline__ void value_products(const s16x4 (&v)[8][2], const bf16x8 (&pb)[NT], WaveState<NT>& st) {
#pragma unroll
  for (int ct = 0; ct < 8; ++ct) {
    union { s16x4 h[2]; bf16x8 v; } vt;
    vt.h[0] = v[ct][0]; vt.h[1] = v[ct][1];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
      st.O[nt][ct] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vt.v, pb[nt], st.O[nt][ct], 0, 0, 0);
  }
}
#define RLDA_G2L(src, dst, off)                                                                                 \
  __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src),                        \
                                   (__attribute__((address_space(3))) void*)(dst), 16, (off), 0)

template <int NTP>
__global__ void __launch_bounds__(NTHREADS, 2) prefill2_kernel(const PrefillParams P) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6, m16 = lane & 15, g = lane >> 4;
  constexpr int N_XCD = 8, WROWS = 16 * NTP;
  const int units = P.P * P.Hkv;
  const int xcd = blockIdx.x % N_XCD, seq = blockIdx.x / N_XCD;
  const int pj = (seq / P.nqb) * N_XCD + xcd, qb = P.nqb - 1 - seq % P.nqb;
  if (pj >= units) return;
  const int p = pj / P.Hkv, j = pj % P.Hkv;
  const int L = clampi(P.lens[p], 0, P.Lp_cap), a = qb * P.QB;
  if (a >= L) return;
  const int nq = min(P.QB, L - a), n_keys = a + nq, n_tiles = ceil_div(n_keys, TK), nrows = nq * P.r;
  bool ok[NTP];
  int pos[NTP], h[NTP], limit[NTP];
  bf16x8 qf[NTP][4];
#pragma unroll
  for (int nt = 0; nt < NTP; ++nt) {
    const int row = WROWS * wv + 16 * nt + m16;
    ok[nt] = row < nrows;
    pos[nt] = a + (ok[nt] ? row / P.r : 0);
    h[nt] = j * P.r + (ok[nt] ? row % P.r : 0);
    limit[nt] = pos[nt] + 1;
    const char* qp = P.q + (((size_t)p * P.Lp_cap + pos[nt]) * P.Hq + h[nt]) * ROWB + 16 * g;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const u32x4 v = ok[nt] ? ldg16(qp + 64 * ks) : u32x4{0, 0, 0, 0};
      qf[nt][ks] = *reinterpret_cast<const bf16x8*>(&v);
    }
  }
  const int wave_first = a + (WROWS * wv) / P.r;            // first position any row of this wavefront holds
  const bool wave_has_rows = WROWS * wv < nrows;
  // LDS addresses of this lane's fragment reads inside stage 0 (the stage goes into the immediate offset)
  const uint32_t l0 = (uint32_t)(uintptr_t)RLDA_LDS(char, lds);
  uint32_t ka[4], va[8];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) ka[ks] = l0 + k_off(m16, 4 * ks + g);
  const int vrow = 4 * g + (m16 >> 2);
#pragma unroll
  for (int ct = 0; ct < 8; ++ct) va[ct] = l0 + v_off(vrow, 2 * ct + ((m16 & 3) >> 1)) + ((m16 & 1) << 3);
  // this wavefront's share of a round's loads: eight instructions of four rows.  Instruction i puts tile row
  // 4 i + lane / 16 into LDS; the store's row is clamped to the last real key (a partial last tile re-reads it;
  // those keys are masked), and the 16-byte chunk a lane fetches is its LDS chunk xor the row's pattern.
  const int kind = uni(wv & 1), sub = uni(wv >> 1), lrow = lane >> 4, chunk = lane & 15;
  const char* gb = (kind ? P.v : P.k) + (size_t)(p * P.Hkv + j) * P.Lp_cap * ROWB;      // uniform
  const int cx = kind ? chunk ^ (lrow << 1) : chunk ^ lrow;                              // V: (row & 7) << 1, K: row & 15
  auto issue = [&](int round) {
    const int t = 2 * round + sub;
    if (t >= n_tiles) return;
    const int key0 = t * TK;
    char* dst = lds + uni((2 * (round & 1) + sub) * STAGE_B + kind * TILE_B);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int ci = kind ? ((4 * i) & 4) << 1 : (4 * i) & 12;
      const uint32_t off = (uint32_t)min(key0 + 4 * i + lrow, n_keys - 1) * ROWB + ((cx ^ ci) << 4);
      RLDA_G2L(gb + off, dst + i * 1024, 0);
    }
  };
  WaveState<NTP> st;
  init_state(st);
  f32x4 s0[NTP], s1[NTP];
  bf16x8 pb[NTP], kf[4][2];
  s16x4 vf[8][2];
  issue(0);
  issue(1);
  wait_vmem();
  __builtin_amdgcn_s_barrier();
  if (wave_has_rows) {
    read_k_frags<0>(ka, kf);
    wait_k_frags(kf);
    score_products<NTP>(kf, qf, s0, s1);
  }
  // one tile; STAGE = t % 4 is a compile-time constant of the unrolled body
  auto tile = [&](auto stage_c, int t) {
    constexpr int STAGE = decltype(stage_c)::value;
    const int key0 = t * TK;
    if (wave_has_rows) {
      float sv[NTP][8], m_new[NTP];
      int nv[NTP];
#pragma unroll
      for (int nt = 0; nt < NTP; ++nt) nv[nt] = limit[nt] - key0;
      if (key0 + TK <= wave_first + 1) softmax_max<NTP, false>(s0, s1, nv, st, P.c, g, sv, m_new);   // wholly in every row's past
      else                             softmax_max<NTP, true>(s0, s1, nv, st, P.c, g, sv, m_new);
      read_v_frags<STAGE>(va, vf);
      softmax_weights<NTP>(sv, m_new, st, pb, P.c);
      wait_v_frags(vf);
    }
    if ((STAGE & 1) || t == n_tiles - 1) {                  // the round's last tile: every fragment of the round is in registers
      wait_vmem();                                          // this wavefront's loads of the next round have landed
      __builtin_amdgcn_s_barrier();
      issue((t >> 1) + 2);                                  // into the buffer the round just left
    }
    if (wave_has_rows) {
      if (t + 1 < n_tiles) read_k_frags<(STAGE + 1) & 3>(ka, kf);
      value_products<NTP>(vf, pb, st);
      if (t + 1 < n_tiles) {
        wait_k_frags(kf);
        score_products<NTP>(kf, qf, s0, s1);
      }
    }
  };
  for (int t0 = 0; t0 < n_tiles; t0 += 4) {
    tile(std::integral_constant<int, 0>{}, t0);
    if (t0 + 1 < n_tiles) tile(std::integral_constant<int, 1>{}, t0 + 1);
    if (t0 + 2 < n_tiles) tile(std::integral_constant<int, 2>{}, t0 + 2);
    if (t0 + 3 < n_tiles) tile(std::integral_constant<int, 3>{}, t0 + 3);
  }
  // normalise and write the rows
#pragma unroll
  for (int nt = 0; nt < NTP; ++nt) {
    float l = st.l[nt], lr = st.lr[nt];
    l += __shfl_xor(l, 16, 64);   l += __shfl_xor(l, 32, 64);
    lr += __shfl_xor(lr, 16, 64); lr += __shfl_xor(lr, 32, 64);
    if (ok[nt]) {
      const float inv = 1.f / lr;
      const size_t orow = ((size_t)p * P.Lp_cap + pos[nt]) * P.Hq + h[nt];
      float* o = P.out + orow * D + 4 * g;
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) {
        const f32x4 v = st.O[nt][ct] * inv;
        *reinterpret_cast<float4*>(o + 16 * ct) = make_float4(v[0], v[1], v[2], v[3]);
      }
      if (P.lse && g == 0) P.lse[orow] = (st.m[nt] + __builtin_amdgcn_logf(l)) * 0.69314718055994531f;
    }
  }
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Layout { size_t cum, pl, po, sl, so, total; };

Layout layout(const Problem& ds) {
  const size_t B = (size_t)n_sequences(ds), E = (size_t)n_prefix_entries(ds), r = ds.Hq / ds.Hkv, Rg = r * max_group(ds);
  const size_t NH = row_parts((int)Rg), R = NH > 1 ? 64 : Rg;   // rows per prefix partial slot
  const size_t nps = E * ds.Hkv * NH + N_WG, nss = B * ds.Hkv + (size_t)WG_WAVES * N_WG;
  Layout L;
  size_t o = 0;
  L.cum = o; o = align256(o + (E + B + 1) * 4);
  L.pl = o;  o = align256(o + nps * R * 2 * 4);
  L.po = o;  o = align256(o + nps * R * D * 2);
  L.sl = o;  o = align256(o + nss * r * 2 * 4);
  L.so = o;  o = align256(o + nss * r * D * 2);
  L.total = o;
  return L;
}

}  // namespace

bool shared_supported(const Problem& ds) {
  if ((ds.dtype != RLDA_BF16 && ds.dtype != RLDA_BF16_KV8) || ds.d != D) return false;
  if (!(ds.scale > 0.f)) return false;                                  // the tile routine's softmax takes maxima before scaling
  const int64_t B = n_sequences(ds), E = n_prefix_entries(ds);
  const int r = ds.Hq / ds.Hkv;
  if (r > 16 || (int64_t)r * max_group(ds) > MAX_GROUP_ROWS) return false;   // rows of one KV group: <= 4 parts of 64
  // The scan of tile counts lives in LDS.  A batch with more prompts and sequences than it holds is run as
  // several launches over whole prompts (max_prompts_per_launch); the tree form has to fit as it is.
  if (ds.n_levels > 0 ? E + B + 1 > MAX_SCAN : ds.G + 2 > MAX_SCAN) return false;
  if (ds.paged && ds.page_shift < 5) return false;                      // a 32-key tile must not straddle pages
  const int NHp = row_parts(r * max_group(ds));                         // prefix units per (prompt, KV head)
  int64_t ptiles = (int64_t)ds.P * ds.Hkv * NHp * ceil_div(ds.Lp_cap, TK);
  int64_t pcap = ds.Lp_cap;
  if (ds.n_levels > 0) {
    // the tree form: bf16 stores, contiguous suffix, one row part (the largest group has at most 64 query rows per KV head)
    if (ds.dtype != RLDA_BF16 || ds.block_table || ds.seq_active || (int64_t)r * max_group(ds) > 64) return false;
    ptiles = 0; pcap = 0;
    for (int l = 0; l < ds.n_levels; ++l) {
      ptiles += (int64_t)ds.levels[l].n_seg * ds.Hkv * ceil_div(ds.levels[l].cap, TK);
      pcap = ds.levels[l].cap > pcap ? ds.levels[l].cap : pcap;
    }
  }
  if (ptiles > MAX_LINE || B * ds.Hkv * ceil_div(ds.Ls_cap, TK) > MAX_LINE) return false;       // 32-bit tile arithmetic
  // partial slots are indexed in 32 bits, also times two in the combine kernels
  const int64_t slot_rows = NHp > 1 ? 64 : (int64_t)r * max_group(ds);
  if ((E * ds.Hkv * NHp + N_WG) * slot_rows * 2 >= (int64_t)1 << 31 ||
      (B * ds.Hkv + (int64_t)WG_WAVES * N_WG) * r * 2 >= (int64_t)1 << 31) return false;
  if (pcap * ROWB >= (int64_t)1 << 31 || (int64_t)ds.Ls_cap * ROWB >= (int64_t)1 << 31) return false;
  return true;
}

// prompts one launch can take: their count, their sequences and one more entry fit the LDS scan
int max_prompts_per_launch(const Problem& ds) {
  if (ds.n_levels > 0) return ds.P;
  const int64_t fit = (MAX_SCAN - 1) / ((int64_t)ds.G + 1);
  return (int)(fit < ds.P ? fit : ds.P);
}

// prompts [p0, p0 + np) of a batch as a batch of its own
Problem prompt_range(const Problem& ds, int p0, int np) {
  Problem s = ds;
  const size_t kvb = kv_elem_bytes(ds.dtype), qb = ds.dtype == RLDA_F32 ? 4 : 2;
  const size_t b0 = (size_t)p0 * ds.G;
  auto adv = [](const void* p, size_t bytes) { return p ? static_cast<const void*>(static_cast<const char*>(p) + bytes) : p; };
  s.P = np;
  s.q = adv(ds.q, b0 * ds.Hq * ds.d * qb);
  s.k_prefix = adv(ds.k_prefix, (size_t)p0 * ds.Hkv * ds.Lp_cap * ds.d * kvb);
  s.v_prefix = adv(ds.v_prefix, (size_t)p0 * ds.Hkv * ds.Lp_cap * ds.d * kvb);
  s.prefix_lens = ds.prefix_lens + p0;
  if (ds.block_table) {                                     // the page pools are shared; the table rows move
    s.block_table = ds.block_table + b0 * ds.max_pages;
  } else {
    s.k_suffix = adv(ds.k_suffix, b0 * ds.Hkv * ds.Ls_cap * ds.d * kvb);
    s.v_suffix = adv(ds.v_suffix, b0 * ds.Hkv * ds.Ls_cap * ds.d * kvb);
  }
  s.suffix_lens = ds.suffix_lens + b0;
  if (ds.seq_active) s.seq_active = ds.seq_active + b0;
  s.out = ds.out + b0 * ds.Hq * ds.d;
  if (ds.lse) s.lse = ds.lse + b0 * ds.Hq;
  return s;
}

size_t shared_workspace_bytes(const Problem& ds) {
  const int np = max_prompts_per_launch(ds);
  return layout(np < ds.P ? prompt_range(ds, 0, np) : ds).total;
}

hipError_t launch_shared(const Problem& whole, hipStream_t stream, hipEvent_t mid) {
  // more prompts and sequences than one launch takes: whole prompts at a time, one after the other on the stream
  // (they share the workspace)
  const int np_max = max_prompts_per_launch(whole);
  if (np_max < whole.P) {
    for (int p0 = 0; p0 < whole.P; p0 += np_max) {
      const int np = whole.P - p0 < np_max ? whole.P - p0 : np_max;
      const hipError_t e = launch_shared(prompt_range(whole, p0, np), stream, p0 + np == whole.P ? mid : nullptr);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  const Problem& ds = whole;
  const Layout L = layout(ds);
  char* ws = static_cast<char*>(ds.workspace);
  SharedParams P;
  P.q = static_cast<const char*>(ds.q);
  P.kp = static_cast<const char*>(ds.k_prefix); P.vp = static_cast<const char*>(ds.v_prefix);
  P.ks = static_cast<const char*>(ds.k_suffix); P.vs = static_cast<const char*>(ds.v_suffix);
  P.plens = ds.prefix_lens; P.slens = ds.suffix_lens;
  P.out = ds.out; P.lse = ds.lse;
  P.cum = reinterpret_cast<int32_t*>(ws + L.cum);
  P.pl = reinterpret_cast<float*>(ws + L.pl); P.po = reinterpret_cast<_Float16*>(ws + L.po);
  P.sl = reinterpret_cast<float*>(ws + L.sl); P.so = reinterpret_cast<_Float16*>(ws + L.so);
  P.P = (int)n_prefix_entries(ds); P.G = max_group(ds); P.B = (int)n_sequences(ds); P.Hq = ds.Hq; P.Hkv = ds.Hkv;
  P.r = ds.Hq / ds.Hkv; P.R = P.r * P.G; P.Lp_cap = ds.Lp_cap; P.Ls_cap = ds.Ls_cap;
  P.div_Hq = make_fastdiv(P.Hq); P.div_G = make_fastdiv(P.G); P.div_r = make_fastdiv(P.r);
  P.c = ds.scale * 1.4426950408889634f;
  const bool tree = ds.n_levels > 0;
  P.n_lev = ds.n_levels;
  for (int l = 0, first = 0; l < MAX_LEVELS; ++l) {
    if (l < ds.n_levels) {
      const Problem::Level& lv = ds.levels[l];
      P.lev[l] = TreeLevel{static_cast<const char*>(lv.k), static_cast<const char*>(lv.v), lv.lens, first, lv.group,
                           P.r * lv.group, lv.cap};
      first += lv.n_seg;
    } else {
      P.lev[l] = TreeLevel{nullptr, nullptr, nullptr, 0x7fffffff, 1, 0, 0};
    }
  }

  // workgroup pairs: by the compute-unit count of the device, looked up once
  {
    static std::mutex mu;
    static int pairs[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (dev < 0 || dev >= 64 || pairs[dev] == 0) {
      int cus = 0;
      e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
      if (e != hipSuccess) return e;
      if (cus < 1) return hipErrorInvalidDevice;
      P.n_cu = pairs_for(cus);
      if (dev >= 0 && dev < 64) pairs[dev] = P.n_cu;
    } else {
      P.n_cu = pairs[dev];
    }
  }
  // row halves of the KV group, and wavefronts per prefix tile (NRB 16-row blocks, a power of two)
  P.SM = side_parts(P.R, P.n_cu);
  P.NH = line_parts(P.R, P.n_cu);
  P.NHs = P.NH == 4 ? 2 : P.NH - 1;
  P.HkvP = P.Hkv * P.NH;
  P.RS = P.R > 64 ? 16 * WG_WAVES : P.R;
  int nrb = 1;
  while (16 * nrb < P.RS) nrb *= 2;
  P.table = ds.block_table; P.active = ds.seq_active;
  P.page_shift = ds.page_shift; P.max_pages = ds.max_pages; P.n_pages = ds.n_pages;
  const bool ext = ds.block_table != nullptr || ds.seq_active != nullptr;
  const bool f8 = ds.dtype == RLDA_BF16_KV8;
  P.kscale = f8 ? ds.k_scale : nullptr; P.vscale = f8 ? ds.v_scale : nullptr;
  typedef void (*kern_t)(const SharedParams);
  static const kern_t kerns[16] = {       // [e4m3 store][extended form][row blocks 1, 2, 4], then the
                                          // four-block kernels of groups with several row parts: [e4m3][extended]
      partial_kernel<1, 1, false, false>, partial_kernel<2, 1, false, false>, partial_kernel<4, 1, false, false>,
      partial_kernel<1, 1, true, false>,  partial_kernel<2, 1, true, false>,  partial_kernel<4, 1, true, false>,
      partial_kernel<1, 1, false, true>,  partial_kernel<2, 1, false, true>,  partial_kernel<4, 1, false, true>,
      partial_kernel<1, 1, true, true>,   partial_kernel<2, 1, true, true>,   partial_kernel<4, 1, true, true>,
      partial_kernel<4, 1, false, false, true>, partial_kernel<4, 1, true, false, true>,
      partial_kernel<4, 1, false, true, true>,  partial_kernel<4, 1, true, true, true>};
  static const kern_t tree_kerns[3] = {partial_kernel<1, 1, false, false, false, true>, partial_kernel<2, 1, false, false, false, true>,
                                       partial_kernel<4, 1, false, false, false, true>};
  const kern_t kern = tree ? tree_kerns[nrb == 1 ? 0 : nrb == 2 ? 1 : 2]
                    : P.R > 64 ? kerns[12 + (f8 ? 2 : 0) + (ext ? 1 : 0)]
                               : kerns[(f8 ? 6 : 0) + (ext ? 3 : 0) + (nrb == 1 ? 0 : nrb == 2 ? 1 : 2)];
  // once per device: a kernel that uses more than 64 KB of LDS in total needs an opt-in
  {
    static std::mutex mu;
    static bool done[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (dev < 0 || dev >= 64 || !done[dev]) {
      for (int i = 0; i < 16 + 3; ++i) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(i < 16 ? kerns[i] : tree_kerns[i - 16]),
                                hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
      }
      if (dev >= 0 && dev < 64) done[dev] = true;
    }
  }
  hipLaunchKernelGGL(kern, dim3(2 * P.n_cu), dim3(NTHREADS), LDS_BYTES, stream, P);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (mid) {
    e = hipEventRecord(mid, stream);
    if (e != hipSuccess) return e;
  }
  const int rows = P.B * P.Hq;
  if (tree) {
    hipLaunchKernelGGL((combine_kernel<false, true>), dim3((rows + 7) / 8), dim3(256), 0, stream, P);
  } else if ((int64_t)ds.P * P.HkvP * P.SM >= COMBINE16_MIN_UNITS) {
    if (ext) hipLaunchKernelGGL(combine16_kernel<true>, dim3((rows + 15) / 16), dim3(256), 0, stream, P);
    else     hipLaunchKernelGGL(combine16_kernel<false>, dim3((rows + 15) / 16), dim3(256), 0, stream, P);
  } else {
    if (ext) hipLaunchKernelGGL(combine_kernel<true>, dim3((rows + 7) / 8), dim3(256), 0, stream, P);
    else     hipLaunchKernelGGL(combine_kernel<false>, dim3((rows + 7) / 8), dim3(256), 0, stream, P);
  }
  return hipGetLastError();
}

bool prefill_supported(int dtype, int Hq, int Hkv, int d) {
  return dtype == RLDA_BF16 && d == D && Hkv > 0 && Hq % Hkv == 0 && Hq / Hkv <= 16;
}

hipError_t launch_prefill(const void* q, const void* k, const void* v, const int32_t* lens, float* out, float* lse,
                          int P_, int Hq, int Hkv, int Lp_cap, float scale, hipStream_t stream) {
  PrefillParams P;
  P.q = static_cast<const char*>(q); P.k = static_cast<const char*>(k); P.v = static_cast<const char*>(v);
  P.lens = lens; P.out = out; P.lse = lse;
  P.P = P_; P.Hq = Hq; P.Hkv = Hkv; P.r = Hq / Hkv; P.Lp_cap = Lp_cap;
  P.c = scale * 1.4426950408889634f;
  // Two 16-row blocks per wavefront (128 rows per workgroup) amortise every LDS read, barrier and
  // tile over twice the matrix work (measured with the register-staged kernel: 440 -> 514 Tflop/s on
  // 32 prompts of 1280 tokens; prefill2_kernel, which they run on: 592, then 688 with its leaner softmax);
  // small problems keep one block so that there are enough workgroups for 256 compute units.  The
  // register-staged kernel is what scales that are not positive run on.
  const int rows1 = 16 * WG_WAVES;
  const int64_t units8 = (int64_t)8 * ceil_div(P_ * Hkv, 8);              // eight XCDs, whole rounds of units
  const bool two = units8 * ceil_div(Lp_cap, (2 * rows1) / P.r) >= 4 * N_WG && scale > 0.f;   // its softmax needs scale > 0
  P.QB = ((two ? 2 : 1) * rows1) / P.r;                     // query positions per workgroup
  P.nqb = ceil_div(Lp_cap, P.QB);
  typedef void (*kern_t)(const PrefillParams);
  const kern_t kern = two ? prefill2_kernel<2> : (scale > 0.f ? prefill2_kernel<1> : prefill_kernel<1>);
  {
    static std::mutex mu;
    static bool done[64] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (dev < 0 || dev >= 64 || !done[dev]) {
      for (const kern_t kf : {static_cast<kern_t>(prefill_kernel<1>), static_cast<kern_t>(prefill2_kernel<2>), static_cast<kern_t>(prefill2_kernel<1>)}) {
        e = hipFuncSetAttribute(reinterpret_cast<const void*>(kf), hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess) return e;
      }
      if (dev >= 0 && dev < 64) done[dev] = true;
    }
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(units8 * P.nqb)), dim3(NTHREADS), LDS_BYTES, stream, P);
  return hipGetLastError();
}

}  // namespace rlda
