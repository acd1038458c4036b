/*
 * fp64 CPU oracle for shared-prefix grouped-query decode attention.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, obviously-correct statement of
 * what one decode step of a rollout computes; it exists so that tests and the
 * benchmark's CPU-baseline leg have something independent to compare the GPU
 * library with.  Product code never includes, links or calls anything here,
 * and nothing here includes or links anything from the GPU library.
 *
 * What is computed (paper Sec. 2.2 and Sec. 3.1 "The MDP of RLLaVA": a state is
 * the whole sequence so far, an action is one token, the transition appends
 * it; Algorithm 1 and Sec. 3.2.2 "Sampling stage": K trajectories are sampled
 * per prompt s_0 = (x_0, y_0), so the K samples of a group share their
 * image+text prompt).  For one decode action of every live trajectory, each
 * sequence b = p*G + g contributes one query token; its keys are the prompt's
 * prefix tokens followed by the sequence's own generated tokens.  The paper
 * does not print the attention formula; it is the scaled dot-product softmax
 * attention with grouped-query heads of the policy models it names (Sec. 5.1
 * "Models"):
 *
 *   j      = h / (Hq/Hkv)                              (KV head of query head h)
 *   K_n,V_n: n <  Lp[p] -> prefix[p, j, n, :]
 *            n >= Lp[p] -> suffix[b, j, n - Lp[p], :]  (N = Lp[p] + Ls[b] keys)
 *   s_n    = scale * sum_c q[b,h,c] * K_n[c]
 *   lse    = m + ln sum_n exp(s_n - m),  m = max_n s_n       (natural log)
 *   out[c] = sum_n exp(s_n - lse) * V_n[c]
 *   N == 0 -> lse = -inf, out = 0
 *
 * All arithmetic is IEEE fp64.  Inputs are fp32 or bf16 (bf16 passed as the
 * raw 16-bit patterns) and are widened exactly.  Two passes over the keys
 * (max, then sum); no streaming softmax, no prefix/suffix split, no blocking.
 * Lengths outside [0, cap] are clamped into that range.
 *
 * Parity pins (tests/test_oracle_pins.py): brute force in pure Python on tiny
 * inputs, constant-V, single key, q = 0, identical keys, duplicated key set,
 * empty suffix / empty prefix / empty both, prefix+suffix LSE merge equals
 * attention over the concatenation, key-permutation invariance, KV-head swap,
 * replicated-prefix equivalence, and torch CPU fp64 softmax/logsumexp.
 */
#ifndef RL_DECODE_ATTN_REF_H
#define RL_DECODE_ATTN_REF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { RLREF_F32 = 0, RLREF_BF16 = 1, RLREF_E4M3 = 2 };

/*
 * All pointers are HOST pointers, contiguous row-major:
 *   q            [B, Hq, d]            B = P*G
 *   k_prefix     [P, Hkv, Lp_cap, d]   v_prefix same
 *   prefix_lens  [P]
 *   k_suffix     [B, Hkv, Ls_cap, d]   v_suffix same
 *   suffix_lens  [B]
 *   out          [B, Hq, d] fp64       lse [B, Hq] fp64 (may be NULL)
 * elem_type: RLREF_F32 (float) or RLREF_BF16 (uint16_t bit patterns).
 * rows/n_rows: if rows != NULL only the (b, h) pairs rows[2*i], rows[2*i+1]
 *   are computed (other entries of out/lse are left untouched).
 * n_threads: OpenMP threads over (b, h); <= 0 means the OpenMP default.  The
 *   result does not depend on it (no cross-thread reduction).
 * Returns 0, or -1 on an invalid argument.  Sets *threads_used if non-NULL.
 */
int rl_decode_attn_ref_f64(int elem_type, int P, int G, int Hq, int Hkv, int d,
                           int Lp_cap, int Ls_cap, double scale,
                           const void* q,
                           const void* k_prefix, const void* v_prefix,
                           const int32_t* prefix_lens,
                           const void* k_suffix, const void* v_suffix,
                           const int32_t* suffix_lens,
                           double* out, double* lse,
                           const int32_t* rows, int64_t n_rows,
                           int n_threads, int* threads_used);

/*
 * The same attention when the K and V stores hold 8-bit floats (the e4m3 encoding of the OCP
 * 8-bit floating point format: 1 sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals,
 * no infinity, S.1111.111 = NaN, largest finite value 448), one byte per element, with one
 * dequantisation factor per KV head:
 *   K_n[c] = k_scale[j] * e4m3(k byte),   V_n[c] = v_scale[j] * e4m3(v byte)
 * (k_scale / v_scale: [Hkv] floats, NULL = 1).  The bytes are widened exactly and the products
 * with the scales are taken in fp64, so the only inputs are the stored bits; everything else is
 * as in rl_decode_attn_ref_f64.  q_type is the element type of q (RLREF_F32 or RLREF_BF16).
 * Pinned in tests/test_oracle_kv8_pins.py: the decode of all 256 byte values against the
 * format's definition (hand values and a library conversion), and equality with
 * rl_decode_attn_ref_f64 on the dequantised values whenever those are exact in fp32.
 */
int rl_decode_attn_ref_kv8_f64(int q_type, const float* k_scale, const float* v_scale,
                               int P, int G, int Hq, int Hkv, int d,
                               int Lp_cap, int Ls_cap, double scale,
                               const void* q,
                               const void* k_prefix, const void* v_prefix,
                               const int32_t* prefix_lens,
                               const void* k_suffix, const void* v_suffix,
                               const int32_t* suffix_lens,
                               double* out, double* lse,
                               const int32_t* rows, int64_t n_rows,
                               int n_threads, int* threads_used);

/* Value of one e4m3 byte (NaN for 0x7f / 0xff). */
double rl_e4m3_to_f64_ref(uint8_t bits);

/*
 * Merge of split-softmax partials (the log-sum-exp combine step): given n
 * partial results (o_i [d], lse_i) of attention of the same query over
 * disjoint key sets, the result over the union is
 *   lse = M + ln sum_i exp(lse_i - M),  M = max_i lse_i
 *   out = sum_i exp(lse_i - lse) * o_i
 * with lse = -inf, out = 0 when every lse_i = -inf (or n == 0).
 * o_parts is [n, d], lse_parts is [n]; out is [d]; *lse one value.
 */
void rl_lse_combine_ref_f64(int n, int d, const double* o_parts,
                            const double* lse_parts, double* out, double* lse);

#ifdef __cplusplus
}
#endif
#endif
