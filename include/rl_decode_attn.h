/*
 * rl_decode_attn -- shared-prefix grouped-query decode attention for
 * GRPO-style rollouts, for AMD MI355X (gfx950).  C ABI, no C++ or framework
 * types in any signature.
 *
 * What one call computes.  The paper casts generation as an MDP whose state is
 * the whole sequence so far, whose action is one token and whose transition
 * appends it (Sec. 2.2; Sec. 3.1 "The MDP of RLLaVA", items (1)-(4)); the
 * initial state s_0 = (x_0, y_0) is an image part plus a text part (text under
 * Eq. 6), and for every prompt the old policy samples a group of K
 * trajectories from that same s_0 (Algorithm 1, rollout steps; Sec. 3.2.2
 * "Sampling stage"; Sec. 5.1: 4-8 responses per prompt).  One call is one
 * decode action of all B = P*G live trajectories for one attention layer:
 * sequence b = p*G + g has one query token, and its keys are the P-shared
 * prompt prefix of prompt p followed by its own generated suffix.  The paper
 * prints no attention formula; the call evaluates the scaled dot-product
 * softmax attention with grouped-query heads of the policy models it names
 * (Sec. 5.1 "Models"):
 *
 *   j = h / (Hq/Hkv)
 *   s_n = scale * <q[b,h,:], K_n>,   K_n/V_n = prefix[p,j,n,:]        n <  Lp[p]
 *                                             suffix[b,j,n-Lp[p],:]   n >= Lp[p]
 *   lse[b,h] = ln sum_n exp(s_n)            (natural log; -inf if no key)
 *   out[b,h,:] = sum_n exp(s_n - lse) V_n   (0 if no key)
 *
 * No causal mask is applied (the single query sees every resident key; the
 * caller has already appended the current token's K/V and counted it in
 * suffix_lens).  Positional rotation of q and K happens before the call.
 *
 * How it is computed: the prefix K/V of a prompt is read from HBM once and
 * reused by all G samples and all Hq/Hkv query heads of a KV group; each
 * sequence's suffix is streamed once; partial (o, lse) results of key ranges
 * are merged by a log-sum-exp combine.  The method is exact; what the result
 * carries is rounding.  fp32 inputs: fp32 rounding order only.  bf16 inputs:
 * scores and sums accumulate in fp32, the softmax weights are rounded to bf16
 * before the value contraction, and a partial result passes between the two
 * kernels as fp16 after a per-row power-of-two scaling that puts its largest
 * magnitude into [0.5, 1) (an error of at most 2^-12 of that magnitude per
 * element).  Observed against the fp64 definition on the benchmark shapes:
 * 1e-3 on out, 1e-6 on lse.
 */
#ifndef RL_DECODE_ATTN_H
#define RL_DECODE_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Element types.  out and lse are always fp32.
 *   RLDA_F32, RLDA_BF16   q and the K/V stores all hold this type.
 *   RLDA_BF16_KV8         q is bf16; the K/V stores (prefix, suffix or pages) hold one byte per
 *                         element, the e4m3 encoding of the OCP 8-bit floating point format (1 sign,
 *                         4 exponent bits with bias 7, 3 mantissa bits, subnormals, no infinity,
 *                         S.1111.111 = NaN, largest finite value 448), with one dequantisation factor
 *                         per KV head:  K_n[c] = k_scale[j] * e4m3(byte),  V_n[c] = v_scale[j] * e4m3(byte).
 *                         The rollout of Algorithm 1 is bound by reading the K/V of every live
 *                         trajectory once per generated token (Sec. 3.2.2 "Sampling stage"); a one-byte
 *                         store halves those bytes.  The call computes the attention of the header
 *                         comment on exactly these dequantised values (every e4m3 value is exact in
 *                         bf16, so nothing is rounded on the way in); how the bytes were produced is
 *                         the caller's business.  Both kernel families take it (d = 64 or 128; the
 *                         usual limits of RLDA_ALGO_SHARED decide which one AUTO picks).  NaN bytes
 *                         may sit in rows at or beyond a length like any other garbage.
 */
typedef enum { RLDA_F32 = 0, RLDA_BF16 = 1, RLDA_BF16_KV8 = 2 } rlda_dtype;

/* Kernel selection. */
typedef enum {
  RLDA_ALGO_AUTO = 0,      /* shared-prefix MFMA path when the shape allows it, else SIMPLE.  The fast path
                              takes bf16 q (bf16 or e4m3 K/V), d = 128, Hq/Hkv <= 16, G * Hq/Hkv <= 256,
                              scale > 0 and, for a paged store, pages of at least 32 rows.  Everything
                              else -- fp32, d = 64, other head ratios or scales, smaller pages -- runs on
                              SIMPLE, which is an order of magnitude slower on large batches (1.04 ms
                              against 0.11 ms on the 7B-shaped benchmark): rl_decode_attn_plan tells which
                              one a descriptor gets. */
  RLDA_ALGO_SIMPLE = 1,    /* one wavefront per (sequence, query head), no sharing, no split */
  RLDA_ALGO_SHARED = 2     /* force the shared-prefix path; RLDA_ERR_UNSUPPORTED if not possible */
} rlda_algo;

/* Return codes. */
enum {
  RLDA_OK = 0,
  RLDA_ERR_INVALID = -1,      /* NULL descriptor / required pointer NULL / negative size        */
  RLDA_ERR_UNSUPPORTED = -2,  /* d not in {64,128}, Hq % Hkv != 0, unknown dtype or algo, ...   */
  RLDA_ERR_WORKSPACE = -3,    /* workspace NULL or smaller than rl_decode_attn_workspace_bytes  */
  RLDA_ERR_STRUCT_SIZE = -4,  /* struct_size != sizeof(rlda_desc) of this library version       */
  RLDA_ERR_LAUNCH = -5        /* the HIP runtime reported an error when enqueuing               */
};

/*
 * Problem descriptor.  All tensors are contiguous, row-major, DEVICE memory
 * unless noted.  The library owns nothing: every pointer is borrowed until the
 * enqueued work has run on `stream`; inputs are never written; the contents of
 * `workspace` are undefined afterwards.
 */
typedef struct {
  uint32_t struct_size;        /* = sizeof(rlda_desc)                                            */
  int32_t  dtype;              /* rlda_dtype                                                     */
  int32_t  algo;               /* rlda_algo                                                      */
  int32_t  P, G;               /* prompts, samples per prompt; sequence b = p*G + g              */
  int32_t  Hq, Hkv, d;         /* query heads, KV heads (Hq % Hkv == 0), head dim (64 or 128)    */
  int32_t  Lp_cap, Ls_cap;     /* row capacity of the prefix / suffix KV buffers (>= 0)          */
  float    scale;              /* multiplies <q,k> before the softmax; any finite value (the shared-prefix
                                  path takes scale > 0 only, other values run on RLDA_ALGO_SIMPLE)    */
  const void*    q;            /* [B, Hq, d]                                                     */
  const void*    k_prefix;     /* [P, Hkv, Lp_cap, d]   (may be NULL if Lp_cap == 0)             */
  const void*    v_prefix;     /* [P, Hkv, Lp_cap, d]                                            */
  const int32_t* prefix_lens;  /* [P]  valid prefix rows per prompt; clamped to [0, Lp_cap]      */
  const void*    k_suffix;     /* [B, Hkv, Ls_cap, d]   (may be NULL if Ls_cap == 0)             */
  const void*    v_suffix;     /* [B, Hkv, Ls_cap, d]                                            */
  const int32_t* suffix_lens;  /* [B]  valid suffix rows per sequence; clamped to [0, Ls_cap]    */
  float*   out;                /* [B, Hq, d] fp32                                                */
  float*   lse;                /* [B, Hq]    fp32, natural log; may be NULL                      */
  void*    workspace;          /* device scratch, 256-byte aligned, may be NULL if 0 bytes needed */
  size_t   workspace_bytes;
  const float* k_scale;        /* [Hkv] fp32 > 0, RLDA_BF16_KV8 only (else ignored); NULL = all 1 */
  const float* v_scale;        /* [Hkv] fp32, likewise                                           */
} rlda_desc;

/*
 * Enqueue one decode-attention step on `hip_stream` (a hipStream_t passed as
 * void*; NULL = the default stream).  Asynchronous: never synchronises, never
 * reads device memory from the host, never allocates.  Lengths live on the
 * device, so out-of-range values cannot be rejected here; the kernels clamp
 * them to [0, cap].  Rows at or beyond a length are never used and may hold
 * anything (including NaN).  Returns RLDA_OK or a negative RLDA_ERR_* code; on
 * a validation error (-1 .. -4) nothing has been enqueued; after RLDA_ERR_LAUNCH
 * part of the work may have been, and out / lse are then undefined.  Results
 * are bit-reproducible from call to call for identical inputs.
 */
int rl_decode_attn(const rlda_desc* desc, void* hip_stream);

/*
 * rl_decode_attn for profiling: additionally records `mid_event` (a hipEvent_t
 * passed as void*, created by the caller with timing enabled; may be NULL) on
 * the stream right after the kernel that streams the K/V tensors, i.e. before
 * the log-sum-exp combine kernel where the path has one.  With events recorded
 * by the caller before and after the call this gives the duration of that
 * kernel alone.  Same arguments, return codes and effects otherwise.
 */
int rl_decode_attn_profiled(const rlda_desc* desc, void* hip_stream, void* mid_event);

/*
 * Bytes of device workspace rl_decode_attn needs for this descriptor (only the
 * shape fields, dtype and algo are read; no pointer is dereferenced, no device
 * is touched).  Returns 0 if none is needed or if the descriptor is invalid
 * (rl_decode_attn reports the reason).
 */
size_t rl_decode_attn_workspace_bytes(const rlda_desc* desc);

/*
 * The kernel family rl_decode_attn would run for this descriptor:
 * RLDA_ALGO_SIMPLE or RLDA_ALGO_SHARED, or a negative RLDA_ERR_* code.
 * Pure host function.
 */
int rl_decode_attn_plan(const rlda_desc* desc);

/*
 * rl_decode_attn for callers that cannot allocate or carry device memory of
 * their own for the library's scratch: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Same arguments, result
 * (bit for bit), stream and error behaviour as rl_decode_attn, except that
 * desc->workspace and desc->workspace_bytes are ignored: the scan of tile
 * counts and the partial results go to an array of
 * RLDA_STATIC_WORKSPACE_BYTES that is part of the library's device image
 * (every GPU the process uses holds one copy until the process ends).  The
 * call allocates and frees nothing, on the host or on the device.  A problem
 * whose rl_decode_attn_workspace_bytes exceeds the array returns
 * RLDA_ERR_WORKSPACE and enqueues nothing.  All calls on one GPU share that
 * GPU's array: calls that may overlap in time there (different streams, or
 * graphs replayed concurrently) race on it and must be ordered by the caller;
 * nothing needs to be cleared between calls (the kernels write every entry
 * they later read).
 */
#define RLDA_STATIC_WORKSPACE_BYTES (64u << 20)
int    rl_decode_attn_static(const rlda_desc* desc, void* hip_stream);
size_t rl_decode_attn_static_workspace_limit(void);          /* = RLDA_STATIC_WORKSPACE_BYTES; pure host */

/* Static, NUL-terminated description of a return code. */
const char* rl_decode_attn_strerror(int code);

/*
 * Text of the HIP runtime status of the calling thread's most recent
 * rl_decode_attn / rl_lse_combine enqueue (for diagnosing RLDA_ERR_LAUNCH).
 */
const char* rl_decode_attn_last_hip_error(void);

/* Library version: major*10000 + minor*100 + patch. */
int rl_decode_attn_version(void);

/*
 * ---- Paged suffix store, finished trajectories ------------------------------
 *
 * A rollout is T consecutive decode actions (Sec. 2.2, Sec. 3.1 transition
 * s' = (s, a)): every suffix grows by one token per step and trajectories stop
 * at different steps (Algorithm 1 samples y_{1:T} per trajectory).  A padded
 * [B, Hkv, Ls_cap, d] suffix store reserves the maximum length for every
 * sequence; here the suffix K/V live in fixed-size pages drawn from one pool
 * and a block table names the pages of each sequence in order, so capacity
 * follows the live tokens (the decode-side counterpart of the padding-free,
 * dynamically batched training the paper lists in Sec. 4.4, "Resource-Efficient
 * Training").  Same result as
 * rl_decode_attn on the gathered suffix.
 *
 * Key n of sequence b's suffix is row n % page_size of page
 * block_table[b, n / page_size].  A page holds all KV heads:
 * k_pages / v_pages are [n_pages, Hkv, page_size, d].  page_size is a power of
 * two (below 32 rows the call runs on RLDA_ALGO_SIMPLE).  Table entries at or beyond ceil(suffix_lens[b] / page_size) are
 * never read as page ids of live keys and may hold anything; entries that are
 * used are clamped to [0, n_pages) (a wrong id gives a wrong result, never an
 * out-of-pool access).  suffix_lens are clamped to [0, max_pages * page_size].
 *
 * seq_active (may be NULL = all active): one byte per sequence; 0 marks a
 * finished trajectory.  Its suffix is not read, out[b] = 0 and lse[b] = -inf
 * are written for it, and a prompt whose G sequences are all finished has its
 * prefix skipped as well.
 *
 * Other fields, ownership, stream and error behaviour are those of rlda_desc /
 * rl_decode_attn.  mid_event as in rl_decode_attn_profiled (may be NULL).
 */
typedef struct {
  uint32_t struct_size;        /* = sizeof(rlda_paged_desc)                                       */
  int32_t  dtype;              /* rlda_dtype                                                     */
  int32_t  algo;               /* rlda_algo                                                      */
  int32_t  P, G;
  int32_t  Hq, Hkv, d;
  int32_t  Lp_cap;             /* row capacity of the prefix buffers                             */
  int32_t  page_size;          /* rows per page, a power of two (>= 32 for the shared-prefix path) */
  int32_t  max_pages;          /* columns of block_table (>= 0)                                  */
  int32_t  n_pages;            /* pages in the pool (>= 1 if max_pages > 0)                      */
  float    scale;
  const void*    q;            /* [B, Hq, d]                                                     */
  const void*    k_prefix;     /* [P, Hkv, Lp_cap, d]                                            */
  const void*    v_prefix;
  const int32_t* prefix_lens;  /* [P]                                                            */
  const void*    k_pages;      /* [n_pages, Hkv, page_size, d]                                   */
  const void*    v_pages;
  const int32_t* block_table;  /* [B, max_pages] page ids                                        */
  const int32_t* suffix_lens;  /* [B]                                                            */
  const uint8_t* seq_active;   /* [B] or NULL                                                    */
  float*   out;                /* [B, Hq, d] fp32                                                */
  float*   lse;                /* [B, Hq] fp32; may be NULL                                      */
  void*    workspace;
  size_t   workspace_bytes;    /* >= rl_decode_attn_paged_workspace_bytes                        */
  const float* k_scale;        /* [Hkv] fp32 > 0, RLDA_BF16_KV8 only; NULL = all 1               */
  const float* v_scale;        /* [Hkv] fp32, likewise                                           */
} rlda_paged_desc;

int    rl_decode_attn_paged(const rlda_paged_desc* desc, void* hip_stream, void* mid_event);
size_t rl_decode_attn_paged_workspace_bytes(const rlda_paged_desc* desc);
int    rl_decode_attn_paged_plan(const rlda_paged_desc* desc);

/*
 * ---- A tree of shared prefixes ---------------------------------------------------
 *
 * The trajectories of a group share more than the prompt when the rollout has
 * several turns: in the paper's agentic tasks (Sec. 5.1, tasks (4) and (5), and
 * the multi-turn direction named as future work) a state is the prompt s_0
 * followed by turns that themselves hold observations, and sub-groups of the K
 * trajectories sampled from s_0 (Algorithm 1) may have a first turn in common.
 * The keys of sequence b are then, level by level, the segment it shares with
 * group_0 - 1 others, the segment it shares with group_1 - 1 others, ..., and
 * finally its own suffix.  This call takes that list:
 *
 *   level l:  k, v   [B / group_l, Hkv, cap_l, d]   one segment per `group_l`
 *                                                    consecutive sequences
 *             lens   [B / group_l]                   valid rows, clamped to [0, cap_l]
 *   sequence b attends to segment b / group_l of every level and to its suffix.
 *
 * The result is the attention of the header comment over the union of these
 * keys (rl_decode_attn is the case of one level with group_0 = G).  Every
 * segment is read from HBM once for all the sequences and query heads that
 * share it; one launch of the K/V-streaming kernel walks all levels and the
 * suffixes, one combine launch merges the partial results; q is read once.
 *
 * group_l >= 1 must divide B; levels need not nest.  0 <= n_levels <=
 * RLDA_MAX_TREE_LEVELS.  Supported: RLDA_BF16, d = 128, Hq/Hkv <= 16,
 * max_l(group_l) * Hq/Hkv <= 64, scale > 0, contiguous stores; anything else
 * returns RLDA_ERR_UNSUPPORTED (compose rl_decode_attn calls and rl_lse_combine
 * instead).  Other fields, ownership, stream, clamping and error behaviour as
 * for rlda_desc / rl_decode_attn.
 */
#define RLDA_MAX_TREE_LEVELS 4
typedef struct {
  const void*    k;            /* [B / group, Hkv, cap, d]  (may be NULL if cap == 0)            */
  const void*    v;            /* same shape                                                     */
  const int32_t* lens;         /* [B / group]                                                    */
  int32_t        group;        /* consecutive sequences that share one segment                   */
  int32_t        cap;          /* row capacity of the level's segments (>= 0)                    */
} rlda_tree_level;

typedef struct {
  uint32_t struct_size;        /* = sizeof(rlda_tree_desc)                                       */
  int32_t  dtype;              /* RLDA_BF16                                                      */
  int32_t  B;                  /* sequences                                                      */
  int32_t  Hq, Hkv, d;
  int32_t  n_levels;           /* shared levels in use                                           */
  int32_t  Ls_cap;             /* row capacity of the suffix buffers                             */
  float    scale;
  rlda_tree_level levels[RLDA_MAX_TREE_LEVELS];
  const void*    q;            /* [B, Hq, d]                                                     */
  const void*    k_suffix;     /* [B, Hkv, Ls_cap, d]                                            */
  const void*    v_suffix;
  const int32_t* suffix_lens;  /* [B]                                                            */
  float*   out;                /* [B, Hq, d] fp32                                                */
  float*   lse;                /* [B, Hq] fp32; may be NULL                                      */
  void*    workspace;
  size_t   workspace_bytes;    /* >= rl_decode_attn_tree_workspace_bytes                         */
} rlda_tree_desc;

int    rl_decode_attn_tree(const rlda_tree_desc* desc, void* hip_stream);
size_t rl_decode_attn_tree_workspace_bytes(const rlda_tree_desc* desc);   /* 0 if invalid or unsupported */

/*
 * The log-sum-exp combine step on its own (merge of split-softmax partials):
 * for each of n_rows rows, given n_parts partial results over disjoint key
 * sets, o_parts [n_parts, n_rows, d] fp32 (each already normalised) and
 * lse_parts [n_parts, n_rows] fp32 (-inf marks an empty part),
 *   lse = ln sum_i exp(lse_i),  out = sum_i exp(lse_i - lse) * o_i,
 * with out = 0, lse = -inf when every part is empty.  All pointers are device
 * memory; lse may be NULL.  d must be 64 or 128.  Asynchronous on `hip_stream`.
 */
int rl_lse_combine(const float* o_parts, const float* lse_parts, int32_t n_parts,
                   int64_t n_rows, int32_t d, float* out, float* lse, void* hip_stream);

/*
 * Testing hook, pure host code: the static work partition the shared-prefix
 * path uses for the given lengths (HOST arrays prefix_lens [P], suffix_lens
 * [P*G]; rows_per_kv_group = G * Hq / Hkv, at most 256).  A KV group with more
 * than 64 query rows is handled in n = 2 (or, above 128 rows, 4) row parts: its
 * prefix units are (prompt, KV head, part) and the "KV head" column of a prefix
 * row holds n * head + part.  `runs` receives one row of 8 int32 per run of tiles a workgroup
 * (prefix) or wavefront (suffix) processes: kind (0 prefix, 1 suffix), prompt
 * or sequence, KV head, first tile, tile count, workgroup, wavefront (-1 for
 * prefix), partial slot.  `parts` receives one row of 6 int32 per partial the
 * combine step reads: kind, prompt or sequence, KV head, workgroup, wavefront,
 * slot.  Rows beyond the capacities are counted but not stored.  Returns the
 * number of runs (or RLDA_ERR_INVALID) and stores the number of parts in
 * *n_parts.  Tiles are 32 keys.
 */
int64_t rl_decode_attn_debug_partition(int32_t P, int32_t G, int32_t Hkv, int32_t rows_per_kv_group,
                                       int32_t Lp_cap, int32_t Ls_cap,
                                       const int32_t* prefix_lens, const int32_t* suffix_lens,
                                       int32_t* runs, int64_t runs_cap, int32_t* parts, int64_t parts_cap,
                                       int64_t* n_parts);

/*
 * The same for a device with `compute_units` compute units (rl_decode_attn_debug_partition is the case
 * of 256, a whole MI355X).  The shared-prefix path asks the device for its compute-unit count at the
 * first call and runs two workgroups on each of n pairs, n = rl_decode_attn_debug_pairs(compute_units):
 * the largest power of two that is at most the count and at most 256 (128, 64 or 32 on the
 * partitions of an MI355X), so the work is split for the device at hand; on other counts the split
 * is still exact, only less even.  Workgroup numbers in `runs` / `parts` are then below 2 n, and the
 * second workgroup of pair c is n + c.  Pure host functions.
 */
int32_t rl_decode_attn_debug_pairs(int32_t compute_units);   /* RLDA_ERR_INVALID below 1 */
int64_t rl_decode_attn_debug_partition_on(int32_t compute_units, int32_t P, int32_t G, int32_t Hkv,
                                          int32_t rows_per_kv_group, int32_t Lp_cap, int32_t Ls_cap,
                                          const int32_t* prefix_lens, const int32_t* suffix_lens,
                                          int32_t* runs, int64_t runs_cap, int32_t* parts, int64_t parts_cap,
                                          int64_t* n_parts);

#ifdef __cplusplus
}
#endif
#endif
