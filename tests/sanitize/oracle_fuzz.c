/* Runs the C oracle on small random problems (edge lengths included) so that a build with
 * -fsanitize=address,undefined can watch every index it forms.  Prints a checksum. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include "../../oracle/rl_decode_attn_ref.h"

static unsigned s = 777;
static int rnd(int n) { s = s * 1664525u + 1013904223u; return (int)((s >> 8) % (unsigned)n); }

int main(void) {
  double sum = 0.0;
  for (int it = 0; it < 60; ++it) {
    const int P = 1 + rnd(3), G = 1 + rnd(4), Hkv = 1 + rnd(3), r = 1 + rnd(3), Hq = Hkv * r, d = 4 * (1 + rnd(4));
    const int Lp = rnd(9), Ls = rnd(9), B = P * G, kv8 = it & 1;
    const size_t nq = (size_t)B * Hq * d, np = (size_t)P * Hkv * (Lp ? Lp : 1) * d, ns = (size_t)B * Hkv * (Ls ? Ls : 1) * d;
    float* q = malloc(nq * sizeof(float));
    void *kp, *vp, *ks, *vs;
    if (kv8) {
      kp = malloc(np); vp = malloc(np); ks = malloc(ns); vs = malloc(ns);
      for (size_t i = 0; i < np; ++i) { ((uint8_t*)kp)[i] = (uint8_t)rnd(0x7f); ((uint8_t*)vp)[i] = (uint8_t)(rnd(0x7f) | 0x80); }
      for (size_t i = 0; i < ns; ++i) { ((uint8_t*)ks)[i] = (uint8_t)rnd(0x7f); ((uint8_t*)vs)[i] = (uint8_t)rnd(0x7f); }
    } else {
      kp = malloc(np * 4); vp = malloc(np * 4); ks = malloc(ns * 4); vs = malloc(ns * 4);
      for (size_t i = 0; i < np; ++i) { ((float*)kp)[i] = rnd(200) / 100.f - 1; ((float*)vp)[i] = rnd(200) / 100.f - 1; }
      for (size_t i = 0; i < ns; ++i) { ((float*)ks)[i] = rnd(200) / 100.f - 1; ((float*)vs)[i] = rnd(200) / 100.f - 1; }
    }
    for (size_t i = 0; i < nq; ++i) q[i] = rnd(200) / 100.f - 1;
    int32_t* pl = malloc(P * sizeof(int32_t));
    int32_t* sl = malloc(B * sizeof(int32_t));
    for (int i = 0; i < P; ++i) pl[i] = rnd(Lp + 4) - 2;          /* also below 0 and above the capacity */
    for (int i = 0; i < B; ++i) sl[i] = rnd(Ls + 4) - 2;
    float ksc[3] = {0.5f, 1.5f, 0.01f}, vsc[3] = {2.f, 0.25f, 1.f};
    double* out = calloc(nq, sizeof(double));
    double* lse = calloc((size_t)B * Hq, sizeof(double));
    int used = 0, rc;
    if (kv8)
      rc = rl_decode_attn_ref_kv8_f64(RLREF_F32, ksc, it % 4 == 1 ? NULL : vsc, P, G, Hq, Hkv, d, Lp, Ls, 0.3, q, Lp ? kp : NULL,
                                      Lp ? vp : NULL, pl, Ls ? ks : NULL, Ls ? vs : NULL, sl, out, lse, NULL, 0, 1 + rnd(3), &used);
    else
      rc = rl_decode_attn_ref_f64(RLREF_F32, P, G, Hq, Hkv, d, Lp, Ls, 0.3, q, Lp ? kp : NULL, Lp ? vp : NULL, pl,
                                  Ls ? ks : NULL, Ls ? vs : NULL, sl, out, lse, NULL, 0, 1 + rnd(3), &used);
    if (rc != 0) { printf("case %d: rc %d\n", it, rc); return 1; }
    for (size_t i = 0; i < nq; ++i) sum += out[i];
    for (int i = 0; i < B * Hq; ++i) if (isfinite(lse[i])) sum += lse[i];
    free(q); free(kp); free(vp); free(ks); free(vs); free(pl); free(sl); free(out); free(lse);
  }
  /* the combine definition, including empty parts */
  double o[3 * 4] = {1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12}, l[3] = {0.5, -INFINITY, 1.5}, oo[4], ll;
  rl_lse_combine_ref_f64(3, 4, o, l, oo, &ll);
  rl_lse_combine_ref_f64(0, 4, o, l, oo, &ll);
  printf("ok %.6f\n", sum + ll);
  return 0;
}
