/*
 * fp64 CPU oracle for shared-prefix grouped-query decode attention.
 * TEST INFRASTRUCTURE ONLY -- see rl_decode_attn_ref.h for the definition it
 * follows and for how it is pinned.  Plain C, one (sequence, query head) at a
 * time, two passes over the keys.  Shares no code with the GPU library.
 */
#include "rl_decode_attn_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Exact widening of one stored element to fp64. */
static double widen(const void* base, int elem_type, int64_t idx) {
  if (elem_type == RLREF_F32) return (double)((const float*)base)[idx];
  /* bf16 is the upper half of an IEEE fp32 bit pattern */
  uint32_t bits = ((uint32_t)((const uint16_t*)base)[idx]) << 16;
  float f;
  memcpy(&f, &bits, sizeof f);
  return (double)f;
}

/* One e4m3 byte (8-bit float of the OCP 8-bit floating point format: sign, 4 exponent bits with
   bias 7, 3 mantissa bits; exponent 0 is subnormal, S.1111.111 is NaN, there is no infinity; the
   largest finite magnitude is 448) to fp64, exactly. */
static double e4m3_to_f64(uint8_t b) {
  const int sign = b >> 7, e = (b >> 3) & 15, m = b & 7;
  double v;
  if (e == 15 && m == 7) return NAN;
  if (e == 0) v = ldexp((double)m, -9);              /* m/8 * 2^-6 */
  else        v = ldexp((double)(8 + m), e - 10);    /* (1 + m/8) * 2^(e-7) */
  return sign ? -v : v;
}

/* Element of a K or V store: as widen(), plus RLREF_E4M3 bytes. */
static double widen_kv(const void* base, int kv_type, int64_t idx) {
  if (kv_type == RLREF_E4M3) return e4m3_to_f64(((const uint8_t*)base)[idx]);
  return widen(base, kv_type, idx);
}

static int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

/* One (b, h): Sec. 3.1 state = prompt prefix then own generated tokens. */
static void one_row(int elem_type, int kv_type, double kscale, double vscale, int G, int Hq, int Hkv, int d, int Lp_cap,
                    int Ls_cap, double scale, const void* q, const void* kp,
                    const void* vp, const int32_t* plens, const void* ks,
                    const void* vs, const int32_t* slens, int b, int h,
                    double* out_row, double* lse_val, double* s /* scratch [Lp_cap+Ls_cap+1+d] */) {
  const int p = b / G;            /* samples of one prompt are adjacent           */
  const int j = h / (Hq / Hkv);   /* contiguous blocks of query heads per KV head */
  const int Lp = clampi(plens[p], 0, Lp_cap);
  const int Ls = clampi(slens[b], 0, Ls_cap);
  const int N = Lp + Ls;
  const int64_t qoff = ((int64_t)b * Hq + h) * d;
  const int64_t poff = ((int64_t)p * Hkv + j) * (int64_t)Lp_cap * d;
  const int64_t soff = ((int64_t)b * Hkv + j) * (int64_t)Ls_cap * d;

  /* accumulate privately and store once: a row listed twice in `rows` is then written twice
     with the same values instead of two threads accumulating into the same memory */
  double* acc = s + (Lp_cap + Ls_cap + 1);
  for (int c = 0; c < d; ++c) acc[c] = 0.0;
  if (N == 0) {
    for (int c = 0; c < d; ++c) out_row[c] = 0.0;
    if (lse_val) *lse_val = -INFINITY;
    return;
  }
  /* scores over the concatenated key list */
  for (int n = 0; n < N; ++n) {
    const void* kb = n < Lp ? kp : ks;
    const int64_t ko = n < Lp ? poff + (int64_t)n * d : soff + (int64_t)(n - Lp) * d;
    double acc = 0.0;
    for (int c = 0; c < d; ++c) acc += widen(q, elem_type, qoff + c) * (kscale * widen_kv(kb, kv_type, ko + c));
    s[n] = scale * acc;
  }
  double m = s[0];
  for (int n = 1; n < N; ++n) if (s[n] > m) m = s[n];
  double z = 0.0;
  for (int n = 0; n < N; ++n) z += exp(s[n] - m);
  const double l = m + log(z);
  for (int n = 0; n < N; ++n) {
    const void* vb = n < Lp ? vp : vs;
    const int64_t vo = n < Lp ? poff + (int64_t)n * d : soff + (int64_t)(n - Lp) * d;
    const double w = exp(s[n] - l);
    for (int c = 0; c < d; ++c) acc[c] += w * (vscale * widen_kv(vb, kv_type, vo + c));
  }
  for (int c = 0; c < d; ++c) out_row[c] = acc[c];
  if (lse_val) *lse_val = l;
}

static int attn_ref(int elem_type, int kv_type, const float* k_scale, const float* v_scale,
                    int P, int G, int Hq, int Hkv, int d,
                    int Lp_cap, int Ls_cap, double scale, const void* q,
                    const void* k_prefix, const void* v_prefix,
                    const int32_t* prefix_lens, const void* k_suffix,
                    const void* v_suffix, const int32_t* suffix_lens,
                    double* out, double* lse, const int32_t* rows,
                    int64_t n_rows, int n_threads, int* threads_used) {
  if (elem_type != RLREF_F32 && elem_type != RLREF_BF16) return -1;
  if (P < 0 || G < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || Lp_cap < 0 || Ls_cap < 0) return -1;
  if (Hq % Hkv != 0) return -1;
  if (!q || !prefix_lens || !suffix_lens || !out) return -1;
  if ((Lp_cap > 0 && (!k_prefix || !v_prefix)) || (Ls_cap > 0 && (!k_suffix || !v_suffix))) return -1;
  const int64_t B = (int64_t)P * G;
  const int64_t total = rows ? n_rows : B * Hq;
  if (rows) {
    for (int64_t i = 0; i < n_rows; ++i)
      if (rows[2 * i] < 0 || rows[2 * i] >= B || rows[2 * i + 1] < 0 || rows[2 * i + 1] >= Hq) return -1;
  }
  int used = 1;
#ifdef _OPENMP
  if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
#pragma omp parallel
  {
#ifdef _OPENMP
#pragma omp single
    used = omp_get_num_threads();
#endif
    double* s = (double*)malloc(sizeof(double) * (size_t)(Lp_cap + Ls_cap + 1 + d));
#pragma omp for schedule(dynamic, 1)
    for (int64_t i = 0; i < total; ++i) {
      const int b = rows ? rows[2 * i] : (int)(i / Hq);
      const int h = rows ? rows[2 * i + 1] : (int)(i % Hq);
      const int j = h / (Hq / Hkv);
      one_row(elem_type, kv_type, k_scale ? (double)k_scale[j] : 1.0, v_scale ? (double)v_scale[j] : 1.0,
              G, Hq, Hkv, d, Lp_cap, Ls_cap, scale, q, k_prefix, v_prefix,
              prefix_lens, k_suffix, v_suffix, suffix_lens, b, h,
              out + ((int64_t)b * Hq + h) * d, lse ? lse + (int64_t)b * Hq + h : NULL, s);
    }
    free(s);
  }
  if (threads_used) *threads_used = used;
  return 0;
}

int rl_decode_attn_ref_f64(int elem_type, int P, int G, int Hq, int Hkv, int d,
                           int Lp_cap, int Ls_cap, double scale, const void* q,
                           const void* k_prefix, const void* v_prefix,
                           const int32_t* prefix_lens, const void* k_suffix,
                           const void* v_suffix, const int32_t* suffix_lens,
                           double* out, double* lse, const int32_t* rows,
                           int64_t n_rows, int n_threads, int* threads_used) {
  return attn_ref(elem_type, elem_type, NULL, NULL, P, G, Hq, Hkv, d, Lp_cap, Ls_cap, scale, q, k_prefix,
                  v_prefix, prefix_lens, k_suffix, v_suffix, suffix_lens, out, lse, rows, n_rows, n_threads,
                  threads_used);
}

int rl_decode_attn_ref_kv8_f64(int q_type, const float* k_scale, const float* v_scale,
                               int P, int G, int Hq, int Hkv, int d,
                               int Lp_cap, int Ls_cap, double scale, const void* q,
                               const void* k_prefix, const void* v_prefix,
                               const int32_t* prefix_lens, const void* k_suffix,
                               const void* v_suffix, const int32_t* suffix_lens,
                               double* out, double* lse, const int32_t* rows,
                               int64_t n_rows, int n_threads, int* threads_used) {
  return attn_ref(q_type, RLREF_E4M3, k_scale, v_scale, P, G, Hq, Hkv, d, Lp_cap, Ls_cap, scale, q, k_prefix,
                  v_prefix, prefix_lens, k_suffix, v_suffix, suffix_lens, out, lse, rows, n_rows, n_threads,
                  threads_used);
}

double rl_e4m3_to_f64_ref(uint8_t bits) { return e4m3_to_f64(bits); }

void rl_lse_combine_ref_f64(int n, int d, const double* o_parts,
                            const double* lse_parts, double* out, double* lse) {
  for (int c = 0; c < d; ++c) out[c] = 0.0;
  double M = -INFINITY;
  for (int i = 0; i < n; ++i) if (lse_parts[i] > M) M = lse_parts[i];
  if (n == 0 || M == -INFINITY) {
    *lse = -INFINITY;
    return;
  }
  double z = 0.0;
  for (int i = 0; i < n; ++i) z += exp(lse_parts[i] - M);   /* exp(-inf) = 0 */
  const double l = M + log(z);
  for (int i = 0; i < n; ++i) {
    if (lse_parts[i] == -INFINITY) continue;                /* empty part: weight 0 */
    const double w = exp(lse_parts[i] - l);
    for (int c = 0; c < d; ++c) out[c] += w * o_parts[(int64_t)i * d + c];
  }
  *lse = l;
}
