// Host-side fuzz of the static work partition (the library's debug hook walks it exactly as the
// kernels do), meant to be built with -fsanitize=address,undefined on the host pass and run
// without a GPU: out-of-range lengths, empty prompts, every row-part count.
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <cstdint>
#include "../../include/rl_decode_attn.h"
int main() {
  unsigned s = 12345;
  auto rnd = [&](int n) { s = s * 1664525u + 1013904223u; return (int)((s >> 8) % (unsigned)n); };
  long total = 0;
  for (int it = 0; it < 300; ++it) {
    int P = 1 + rnd(40), G = 1 + rnd(8), Hkv = 1 + rnd(4), R = 1 + rnd(256), Lp = rnd(3000), Ls = rnd(5000);
    std::vector<int32_t> pl(P), sl(P * G);
    for (auto& v : pl) v = rnd(Lp + 50) - 10;
    for (auto& v : sl) v = rnd(3) ? rnd(Ls + 50) - 10 : 0;
    int64_t cap = 4 * ((int64_t)P * (G + 2) * Hkv * 4 + 8 * 512) + 16;
    std::vector<int32_t> runs(cap * 8), parts(cap * 6);
    int64_t np = 0;
    int64_t nr = rl_decode_attn_debug_partition(P, G, Hkv, R, Lp, Ls, pl.data(), sl.data(), runs.data(), cap, parts.data(), cap, &np);
    if (nr < 0 || nr > cap || np != nr) { printf("case %d: nr %lld np %lld cap %lld\n", it, (long long)nr, (long long)np, (long long)cap); return 1; }
    total += nr;
  }
  printf("ok %ld\n", total);
  return 0;
}
