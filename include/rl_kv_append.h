/*
 * rl_kv_append_rope -- the state transition of one decode step for one
 * attention layer, for AMD MI355X (gfx950).  C ABI.
 *
 * The transition of the paper's MDP appends the chosen token to the state
 * (Sec. 2.2; Sec. 3.1 "The MDP of RLLaVA", item (3): s' = (s, a)).  For the
 * key/value store of a layer this means: rotate the new token's query and key
 * by its position, write the rotated key and the value into the next free row
 * of every live sequence's suffix store, and count it, so that the attention
 * call that follows (rl_decode_attn / rl_decode_attn_paged) sees it.  One
 * launch does all four.
 *
 * Rotary embedding.  The paper names the policy models (Sec. 5.1) but prints
 * no formula; this is the rotary position embedding of RoFormer (Su et al.,
 * 2021) in the "rotate-half" pairing, with the three-component positions of
 * the multimodal variant those models use: for frequency index i in [0, d/2)
 * and the position component c(i) of the section i falls in,
 *     angle = positions[c(i)][b] * inv_freq[i]
 *     y[i]       = x[i] * cos(angle) - x[i + d/2] * sin(angle)
 *     y[i + d/2] = x[i + d/2] * cos(angle) + x[i] * sin(angle)
 * applied to every head of q and k_new of sequence b.  sections[0..2] are the
 * numbers of consecutive frequency indices that use the temporal, height and
 * width component (sum = d/2); for text tokens the three components are equal
 * and the scheme is the ordinary one-dimensional embedding.  Angles, cosines
 * and sines are evaluated in fp64 from the fp32 inv_freq table and rounded to
 * fp32; the rotation itself is fp32, rounded to the element type on store.
 *
 * Destination.  Row n = suffix_lens[b] (before the call) of sequence b's
 * suffix: contiguous store [B, Hkv, Ls_cap, d] when block_table is NULL, else
 * the page pools of rlda_paged_desc (row n % page_size of page
 * block_table[b, n / page_size], id clamped to the pool).  If n is outside
 * [0, capacity) nothing is written for that sequence and its length stays.
 * Otherwise suffix_lens[b] becomes n + 1.  Sequences with seq_active[b] == 0
 * are left alone entirely (q is still rotated: it is not used).
 */
#ifndef RL_KV_APPEND_H
#define RL_KV_APPEND_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* All pointers are DEVICE memory, borrowed until the enqueued work has run. */
typedef struct {
  uint32_t struct_size;         /* = sizeof(rl_kv_append_desc)                                   */
  int32_t  dtype;               /* element type of q, k_new, v_new and the stores: 0 fp32, 1 bf16;
                                   2: q, k_new, v_new bf16 and the stores e4m3 bytes (see below)  */
  int32_t  B, Hq, Hkv, d;       /* sequences, query heads, KV heads, head dim (64 or 128)        */
  int32_t  Ls_cap;              /* contiguous store: rows per sequence                           */
  int32_t  page_size, max_pages, n_pages;   /* paged store (block_table != NULL); else ignored   */
  int32_t  sections[3];         /* frequency indices per position component, sum = d/2           */
  void*          q;             /* [B, Hq, d]   rotated in place                                 */
  const void*    k_new;         /* [B, Hkv, d]  before rotation                                  */
  const void*    v_new;         /* [B, Hkv, d]                                                   */
  const int32_t* positions;     /* [3, B]       temporal, height, width position of the token    */
  const float*   inv_freq;      /* [d/2]                                                         */
  void*          k_store;       /* [B, Hkv, Ls_cap, d] or [n_pages, Hkv, page_size, d]           */
  void*          v_store;
  const int32_t* block_table;   /* [B, max_pages] or NULL                                        */
  int32_t*       suffix_lens;   /* [B]  in: row to write; out: incremented where a row was written */
  const uint8_t* seq_active;    /* [B] or NULL                                                   */
  const float*   k_scale;       /* [Hkv] dtype 2 only (else ignored): factors of the e4m3 stores, > 0; NULL = 1 */
  const float*   v_scale;       /* [Hkv] likewise                                                */
} rl_kv_append_desc;

/*
 * dtype 2 (the stores of RLDA_BF16_KV8 in rl_decode_attn.h): the appended rows are quantised,
 *   byte = the e4m3 value nearest to x / factor[j]  (x and the quotient in fp32; ties to the even
 *          code; magnitudes above 448, infinities included, become 448; NaN becomes 0x7f)
 * where x is the rotated key as computed in fp32 (not rounded to bf16 first) or the value as
 * given.  Reading the row back through rl_decode_attn with the same factors gives x to within
 * half an e4m3 step (relative 2^-4).
 */

/*
 * Enqueue on `hip_stream` (hipStream_t as void*).  Asynchronous, allocates
 * nothing, needs no workspace.  Returns 0 or a negative code with the meaning
 * of the RLDA_ERR_* values of rl_decode_attn.h (-1 invalid argument, -2
 * unsupported shape / dtype / sections, -4 struct_size, -5 HIP error).
 */
int rl_kv_append_rope(const rl_kv_append_desc* desc, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif
