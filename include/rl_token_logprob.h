/*
 * rl_token_logprob -- per-token policy statistics from vocabulary logits, for
 * AMD MI355X (gfx950).  C ABI.
 *
 * The rollout samples y_t from the softmax of the policy's logits; the later
 * stages of the RL loop need, for every generated token, the quantities the
 * paper's objective is written in:
 *   - log pi(y_t | s_0, y_<t) of the behaviour policy and of the target
 *     policy, whose ratio is r_t(theta) (Sec. 2.2 "Adaptation for
 *     Off-Policy"; the L^PG term of Eq. 6; Sec. 3.2.2 policy-update stage);
 *   - the entropy of pi(. | s_0, y_<t) (entropy bonus, Sec. 2.2
 *     "Regularization");
 *   - KL(pi_theta(.|s) || pi_ref(.|s)) over the whole vocabulary (the
 *     KL-to-reference regulariser: Sec. 2.2 "Regularization" item (1), the
 *     Omega term of Eq. 6, KL_t in Sec. 3.2.2).
 * One call makes one pass over the logits (and the reference logits, if
 * given) and produces all of them; nothing of size [rows, vocab] is written.
 *
 * With z = logits * inv_temperature and w = ref_logits * inv_temperature:
 *   lse[b]         = ln sum_i exp(z[b,i])
 *   logprob[b]     = z[b, y_b] - lse[b]
 *   entropy[b]     = - sum_i p_i ln p_i,            p_i = exp(z[b,i] - lse[b])
 *   ref_logprob[b] = w[b, y_b] - ln sum_i exp(w[b,i])
 *   kl[b]          = sum_i p_i (ln p_i - ln r_i),   r = softmax(w[b,:])
 * y_b = token_ids[b].  A negative id marks an ignored position (logprob and
 * ref_logprob 0); an id >= vocab gives NaN there; no logit is read out of
 * range in either case.  A logit of -inf is a masked token (p_i = 0, nothing
 * added to the sums); a NaN logit is read as a masked token too, it does not
 * propagate.  inv_temperature must be positive and finite (else -1).
 * Arithmetic is fp32 (inputs fp32 or bf16).
 */
#ifndef RL_TOKEN_LOGPROB_H
#define RL_TOKEN_LOGPROB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* All pointers are DEVICE memory, borrowed until the enqueued work has run. */
typedef struct {
  uint32_t struct_size;      /* = sizeof(rl_token_logprob_desc)                                  */
  int32_t  dtype;            /* element type of logits / ref_logits: 0 = fp32, 1 = bf16          */
  int64_t  n_rows;           /* tokens (>= 0)                                                    */
  int64_t  row_stride;       /* elements between rows (>= vocab; multiple of 4 fp32 / 8 bf16)    */
  int32_t  vocab;            /* logits per row (>= 1)                                            */
  float    inv_temperature;  /* multiplies both logit tensors before the softmax                 */
  const void*    logits;     /* [n_rows, row_stride], 16-byte aligned                            */
  const void*    ref_logits; /* same shape, stride and dtype, or NULL                            */
  const int32_t* token_ids;  /* [n_rows]                                                         */
  float* logprob;            /* [n_rows] each; any of the five may be NULL (not computed/stored) */
  float* lse;
  float* entropy;
  float* ref_logprob;        /* needs ref_logits */
  float* kl;                 /* needs ref_logits */
  void*  workspace;          /* device scratch, 256-byte aligned, >= rl_token_logprob_workspace_bytes */
  size_t workspace_bytes;
} rl_token_logprob_desc;

/*
 * Enqueue on `hip_stream` (hipStream_t as void*; NULL = default stream).
 * Asynchronous, allocates nothing.  Returns 0 or a negative code with the
 * meaning of the RLDA_ERR_* values of rl_decode_attn.h: -1 invalid argument
 * (NULL logits/token_ids with rows > 0, ref outputs without ref_logits,
 * negative sizes), -2 unsupported (dtype, stride not a multiple of the vector
 * width or < vocab, misaligned base), -3 workspace, -4 struct_size, -5 HIP
 * error.  Results are bit-reproducible from call to call.
 */
int rl_token_logprob(const rl_token_logprob_desc* desc, void* hip_stream);

/* Bytes of workspace the call needs (0 if none or if the descriptor is invalid).  Pure host code. */
size_t rl_token_logprob_workspace_bytes(const rl_token_logprob_desc* desc);

#ifdef __cplusplus
}
#endif
#endif
