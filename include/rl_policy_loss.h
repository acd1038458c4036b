/*
 * rl_group_advantage, rl_policy_loss -- the per-trajectory and per-token
 * arithmetic between a finished rollout and the policy update, for AMD MI355X
 * (gfx950).  C ABI.
 *
 * The paper's loop (Algorithm 1; Sec. 3.2.2) scores every sampled trajectory,
 * turns the K rewards of a group into advantages, and maximises
 *     sum_t L^PG(pi_theta, pi_old, A_t) - Omega(pi_theta, pi_ref)        (Eq. 6)
 * over the generated tokens.  These two calls are that arithmetic on device
 * arrays the rollout already produced (rl_token_logprob gives logprob, KL_t
 * and the entropy per token):
 *
 *   scoring stage      r_b = sum_m alpha_m R_m(b)                          (Sec. 3.2.2 "Scoring stage")
 *   advantage stage    A = AdvEstimator(r), critic-free, over the G samples of a prompt
 *                      (Sec. 3.2.2 "Advantage estimation stage"; estimators named in Sec. 4.2):
 *                        RL_ADV_GROUP_NORM     A_i = (r_i - mean) / (std + eps)      std divisor G-1 if `unbiased` else G;
 *                                                                                     a group of one sample has std 0
 *                        RL_ADV_GROUP_CENTER   A_i = r_i - mean
 *                        RL_ADV_LEAVE_ONE_OUT  A_i = r_i - mean_{j != i} r_j          0 for a group of one
 *   policy update      rho_t = exp(logprob_t - old_logprob_t)              (Sec. 2.2 "Adaptation for Off-Policy")
 *                      L_t   = min(rho_t A, clip(rho_t, 1 - clip_low, 1 + clip_high) A)   RL_PG_PPO_CLIP, the clipped
 *                              surrogate the text under Eq. 6 names
 *                              min(rho_t, clip(rho_t, ...)) A                             RL_PG_AS_PRINTED, that text's
 *                              expression taken literally (same value for A >= 0, different for A < 0)
 *                      loss  = - agg(L_t) + beta_kl agg(KL_t) - beta_ent agg(H_t)         (Sec. 2.2 "Regularization",
 *                              Omega of Eq. 6 with the KL-to-reference term and the entropy bonus)
 *                      agg   = RL_AGG_TOKEN_MEAN: sum over valid tokens / number of valid tokens
 *                              RL_AGG_SEQ_MEAN:   mean over sequences with tokens of their token means
 *                      grad_logprob[b,t] = d loss / d logprob[b,t] = - weight_t * (rho_t A if the unclipped branch is
 *                              the minimum, else 0); 0 on padding.  (KL_t and H_t are inputs: their dependence on the
 *                              logits is the caller's autograd business.)
 * Tokens t >= lens[b] are padding and never read.  Arithmetic is fp32, the batch sums are accumulated per
 * sequence in fp32 in a fixed order and across sequences in fp64 in a fixed order: results are
 * bit-reproducible from call to call.
 */
#ifndef RL_POLICY_LOSS_H
#define RL_POLICY_LOSS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { RL_ADV_GROUP_NORM = 0, RL_ADV_GROUP_CENTER = 1, RL_ADV_LEAVE_ONE_OUT = 2 } rl_adv_mode;
typedef enum { RL_PG_PPO_CLIP = 0, RL_PG_AS_PRINTED = 1 } rl_pg_form;
typedef enum { RL_AGG_TOKEN_MEAN = 0, RL_AGG_SEQ_MEAN = 1 } rl_loss_agg;

/* All pointers are DEVICE memory, borrowed until the enqueued work has run. */
typedef struct {
  uint32_t struct_size;      /* = sizeof(rl_group_advantage_desc)                                 */
  int32_t  mode;             /* rl_adv_mode                                                      */
  int32_t  P, G;             /* prompts, samples per prompt; trajectory b = p*G + g (G <= 1024)  */
  int32_t  n_metrics;        /* reward metrics per trajectory (1 .. 64)                          */
  int32_t  unbiased;         /* RL_ADV_GROUP_NORM: nonzero = divisor G-1                         */
  float    eps;              /* RL_ADV_GROUP_NORM: added to the std (>= 0)                       */
  const float* metrics;      /* [n_metrics, B]                                                   */
  const float* weights;      /* [n_metrics] alpha_m                                              */
  float* rewards;            /* [B] combined reward; may be NULL                                 */
  float* advantages;         /* [B]                                                              */
} rl_group_advantage_desc;

typedef struct {
  uint32_t struct_size;      /* = sizeof(rl_policy_loss_desc)                                    */
  int32_t  form;             /* rl_pg_form                                                       */
  int32_t  agg;              /* rl_loss_agg                                                      */
  int32_t  B, T;             /* sequences, token capacity of a row                               */
  int64_t  row_stride;       /* elements between rows of the [B, T] arrays (>= T)                */
  float    clip_low, clip_high;   /* rho is clipped to [1 - clip_low, 1 + clip_high]; both >= 0  */
  float    beta_kl, beta_ent;
  const float*   logprob;     /* [B, row_stride]  log pi_theta(y_t | .)                          */
  const float*   old_logprob; /* [B, row_stride]  log pi_old(y_t | .)                            */
  const float*   advantages;  /* [B]              one per trajectory                             */
  const float*   kl;          /* [B, row_stride] KL_t, or NULL (then its term is 0)              */
  const float*   entropy;     /* [B, row_stride] H_t, or NULL                                    */
  const int32_t* lens;        /* [B] generated tokens per sequence; clamped to [0, T]            */
  float* grad_logprob;        /* [B, row_stride] or NULL; columns >= T are not written            */
  float* stats;               /* [8]: loss, agg(L), agg(KL), agg(H), fraction of tokens on the flat (clipped)
                                 branch, mean rho, mean (old_logprob - logprob), number of valid tokens;
                                 the last four are plain token means                               */
  void*  workspace;           /* device scratch, 256-byte aligned, >= rl_policy_loss_workspace_bytes */
  size_t workspace_bytes;
} rl_policy_loss_desc;

/*
 * Both: enqueue on `hip_stream` (hipStream_t as void*; NULL = default stream), asynchronous,
 * allocate nothing.  Return 0 or a negative code with the meaning of the RLDA_ERR_* values of
 * rl_decode_attn.h: -1 invalid argument (NULL where a tensor is required, negative sizes, negative
 * clip widths or eps), -2 unsupported (unknown mode / form / agg, G > 1024, n_metrics outside
 * 1..64, row_stride < T), -3 workspace, -4 struct_size, -5 HIP error.  Empty batches succeed;
 * rl_policy_loss then writes zeros to stats.
 */
int rl_group_advantage(const rl_group_advantage_desc* desc, void* hip_stream);
int rl_policy_loss(const rl_policy_loss_desc* desc, void* hip_stream);

/* Bytes of workspace rl_policy_loss needs (0 if the descriptor is invalid).  Pure host code. */
size_t rl_policy_loss_workspace_bytes(const rl_policy_loss_desc* desc);

#ifdef __cplusplus
}
#endif
#endif
