/*
 * rl_prefill_attn -- causal attention of every prompt over its own tokens, for
 * AMD MI355X (gfx950).  C ABI.
 *
 * The K trajectories that the rollout samples per prompt (Algorithm 1; Sec. 3.2.2
 * "Sampling stage") share their initial state s_0 = (x_0, y_0) (Sec. 3.1), so the
 * pass of the policy over the prompt is needed once per prompt, not once per
 * trajectory; for one attention layer it is this call, and the K/V it attends over
 * are what rl_decode_attn then reads as the shared prefix store (same layout).
 * The paper prints no formula; this is the causal scaled dot-product attention with
 * grouped-query heads of the policy models it names (Sec. 5.1):
 *
 *   j = h / (Hq/Hkv)
 *   s_in         = scale * <q[p,i,h,:], k[p,j,n,:]>           for n <= i < lens[p]
 *   lse[p,i,h]   = ln sum_{n<=i} exp(s_in)                     (natural log)
 *   out[p,i,h,:] = sum_{n<=i} exp(s_in - lse[p,i,h]) v[p,j,n,:]
 *
 * Positional rotation of q and k happens before the call.  Rows of out / lse at
 * positions i >= lens[p] are not written; K/V rows at or beyond lens[p] are never
 * read.  bf16 inputs, fp32 accumulation on the matrix cores, softmax weights rounded
 * to bf16 before the value contraction (the arithmetic of the decode path), fp32
 * outputs.  Unlike the decode step this pass is bound by the matrix cores, not by
 * HBM: every K/V tile is used by up to 128 query rows.
 */
#ifndef RL_PREFILL_ATTN_H
#define RL_PREFILL_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* All pointers are DEVICE memory, contiguous, borrowed until the enqueued work has run. */
typedef struct {
  uint32_t struct_size;       /* = sizeof(rl_prefill_desc)                                       */
  int32_t  dtype;             /* 1 (bf16: RLDA_BF16 of rl_decode_attn.h); nothing else           */
  int32_t  P;                 /* prompts (>= 0)                                                  */
  int32_t  Hq, Hkv, d;        /* Hq % Hkv == 0, Hq/Hkv <= 16, d = 128                            */
  int32_t  Lp_cap;            /* row capacity of q / k / v / out per prompt (>= 0)               */
  float    scale;              /* multiplies <q,k> before the softmax; any finite value           */
  const void*    q;           /* [P, Lp_cap, Hq, d]                                              */
  const void*    k;           /* [P, Hkv, Lp_cap, d]  the prefix store layout of rl_decode_attn  */
  const void*    v;           /* [P, Hkv, Lp_cap, d]                                             */
  const int32_t* lens;        /* [P] prompt lengths, clamped to [0, Lp_cap]                      */
  float*   out;               /* [P, Lp_cap, Hq, d] fp32                                         */
  float*   lse;               /* [P, Lp_cap, Hq]    fp32; may be NULL                            */
} rl_prefill_desc;

/*
 * Enqueue on `hip_stream` (hipStream_t as void*; NULL = default stream).  Asynchronous, allocates
 * nothing, needs no workspace.  Returns 0 or a negative code with the meaning of the RLDA_ERR_*
 * values of rl_decode_attn.h: -1 invalid argument (NULL tensor with work to do, negative size),
 * -2 unsupported (dtype, d, head ratio, more than 2^31 - 1 workgroups, Lp_cap >= 2^24), -4 struct_size, -5 HIP
 * error.  Results are bit-reproducible from call to call.
 */
int rl_prefill_attn(const rl_prefill_desc* desc, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif
