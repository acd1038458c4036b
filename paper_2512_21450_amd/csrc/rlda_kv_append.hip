// Decode-step state transition for one attention layer (Sec. 3.1 of the paper, item (3):
// s' = (s, a)): rotary embedding of the new token's q and k (RoFormer rotation in the rotate-half
// pairing, three position components over sections of the frequency index), append of the rotated
// key and the value to the sequence's suffix store (contiguous or paged), length count.
//
// One workgroup per sequence.  The d/2 angles of a sequence are shared by all heads: they are
// evaluated once, in fp64 (64 or fewer evaluations per sequence; an fp32 product pos * inv_freq
// would already be off by 2e-3 rad at position 32k), rounded to fp32 and kept in LDS.  The rest is
// a few KB of element-wise work: the kernel is launch-bound, its purpose is to be one launch.
// Stores may hold e4m3 bytes: the appended rows are then divided by the KV head's factor and
// rounded to the nearest e4m3 value with integer operations (ties to even, saturating).
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/rl_kv_append.h"

namespace {

struct Params {
  char* q; const char* k_new; const char* v_new;
  const int32_t* pos; const float* inv_freq;
  char* ks; char* vs; const int32_t* table; int32_t* lens; const uint8_t* active;
  int B, Hq, Hkv, d, Ls_cap, page_shift, max_pages, n_pages;
  int s0, s1;                      // frequency indices below s0: temporal; below s0 + s1: height; else width
  const float* kscale; const float* vscale;   // e4m3 stores: per-KV-head factors, or null
};

template <typename T> struct Elt;
template <> struct Elt<float> {
  __device__ static float ld(const char* p, size_t i) { return reinterpret_cast<const float*>(p)[i]; }
  __device__ static void st(char* p, size_t i, float v) { reinterpret_cast<float*>(p)[i] = v; }
};
template <> struct Elt<uint16_t> {
  __device__ static float ld(const char* p, size_t i) {
    return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(p)[i] << 16);
  }
  __device__ static void st(char* p, size_t i, float v) {          // round to nearest even (finite values)
    const uint32_t u = __float_as_uint(v);
    reinterpret_cast<uint16_t*>(p)[i] = (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
  }
};

// fp32 -> e4m3 byte (1 sign, 4 exponent bits with bias 7, 3 mantissa bits, subnormals, no infinity):
// nearest value, ties to the even code, |y| > 448 -> 448, NaN -> 0x7f.
__device__ __forceinline__ uint8_t f32_to_e4m3(float y) {
  const uint32_t sign = (__float_as_uint(y) >> 24) & 0x80u;
  float a = fabsf(y);
  if (!(a == a)) return (uint8_t)(sign | 0x7Fu);
  a = fminf(a, 448.f);
  uint32_t code;
  if (a < 0.015625f) {                                      // below 2^-6 the grid is 2^-9; 8 steps reach the first normal
    code = (uint32_t)__float2int_rn(a * 512.f);
  } else {
    uint32_t b = __float_as_uint(a);
    b += 0x7FFFFu + ((b >> 20) & 1u);                       // nearest even at 3 mantissa bits; a carry moves the exponent
    code = (b >> 20) - (120u << 3);                         // exponent bias 127 -> 7
  }
  return (uint8_t)(sign | code);
}

// how a rotated key element / a value element reaches the store
template <typename T, bool F8> struct Store {
  __device__ static void put(char* p, size_t i, float v, float) { Elt<T>::st(p, i, v); }
};
template <typename T> struct Store<T, true> {
  __device__ static void put(char* p, size_t i, float v, float factor) {
    reinterpret_cast<uint8_t*>(p)[i] = f32_to_e4m3(__fdiv_rn(v, factor));
  }
};

template <typename T, bool F8>
__global__ void __launch_bounds__(256) kv_append_rope_kernel(const Params P) {
  __shared__ float cs[64], sn[64];
  const int b = blockIdx.x, tid = threadIdx.x, half = P.d >> 1;
  if (tid < half) {
    const int comp = tid < P.s0 ? 0 : (tid < P.s0 + P.s1 ? 1 : 2);
    const double ang = (double)P.pos[(size_t)comp * P.B + b] * (double)P.inv_freq[tid];
    double s, c;
    sincos(ang, &s, &c);
    cs[tid] = (float)c; sn[tid] = (float)s;
  }
  // destination row of this sequence, if it takes one
  const int n = P.lens[b];
  const bool live = !P.active || P.active[b] != 0;
  const bool room = live && n >= 0 && n < P.Ls_cap;
  size_t row = 0;                                           // first element of row n, KV head 0; heads are `hstride` apart
  size_t hstride = 0;
  if (room) {
    if (P.table) {
      const int ps = 1 << P.page_shift;
      const int pg = min(max(P.table[(size_t)b * P.max_pages + (n >> P.page_shift)], 0), P.n_pages - 1);
      row = (((size_t)pg * P.Hkv) * ps + (n & (ps - 1))) * P.d;
      hstride = (size_t)ps * P.d;
    } else {
      row = (((size_t)b * P.Hkv) * P.Ls_cap + n) * P.d;
      hstride = (size_t)P.Ls_cap * P.d;
    }
  }
  __syncthreads();
  // q (in place) and k_new (to the store): one thread per (head, pair)
  const int pairs = (P.Hq + P.Hkv) * half;
  for (int idx = tid; idx < pairs; idx += 256) {
    const int head = idx / half, i = idx - head * half;
    const float c = cs[i], s = sn[i];
    if (head < P.Hq) {
      const size_t o = ((size_t)b * P.Hq + head) * P.d + i;
      const float lo = Elt<T>::ld(P.q, o), hi = Elt<T>::ld(P.q, o + half);
      Elt<T>::st(P.q, o, lo * c - hi * s);
      Elt<T>::st(P.q, o + half, hi * c + lo * s);
    } else if (room) {
      const int j = head - P.Hq;
      const size_t o = ((size_t)b * P.Hkv + j) * P.d + i;
      const float lo = Elt<T>::ld(P.k_new, o), hi = Elt<T>::ld(P.k_new, o + half);
      const size_t dst = row + j * hstride + i;
      const float f = F8 && P.kscale ? P.kscale[j] : 1.f;
      Store<T, F8>::put(P.ks, dst, lo * c - hi * s, f);
      Store<T, F8>::put(P.ks, dst + half, hi * c + lo * s, f);
    }
  }
  if (room) {
    for (int idx = tid; idx < P.Hkv * P.d; idx += 256) {    // the value row: a copy, or quantised
      const int j = idx / P.d, i = idx - j * P.d;
      const size_t src = ((size_t)b * P.Hkv + j) * P.d + i, dst = row + j * hstride + i;
      if (F8) Store<T, F8>::put(P.vs, dst, Elt<T>::ld(P.v_new, src), P.vscale ? P.vscale[j] : 1.f);
      else    reinterpret_cast<T*>(P.vs)[dst] = reinterpret_cast<const T*>(P.v_new)[src];
    }
    if (tid == 0) P.lens[b] = n + 1;                        // every thread read n before the barrier above
  }
}

}  // namespace

extern "C" int rl_kv_append_rope(const rl_kv_append_desc* d, void* hip_stream) {
  if (!d) return -1;
  if (d->struct_size != sizeof(rl_kv_append_desc)) return -4;
  if (d->B < 0 || d->Hq <= 0 || d->Hkv <= 0 || d->d <= 0) return -1;
  if (d->dtype != 0 && d->dtype != 1 && d->dtype != 2) return -2;
  if (d->d != 64 && d->d != 128) return -2;
  if (d->sections[0] < 0 || d->sections[1] < 0 || d->sections[2] < 0 ||
      d->sections[0] + d->sections[1] + d->sections[2] != d->d / 2) return -2;
  const bool paged = d->block_table != nullptr;
  int cap = d->Ls_cap, shift = 0;
  if (paged) {
    if (d->page_size <= 0 || d->max_pages < 0 || d->n_pages < 1) return -1;
    if (d->page_size < 32 || (d->page_size & (d->page_size - 1))) return -2;
    if ((int64_t)d->max_pages * d->page_size > (int64_t)1 << 30) return -2;
    cap = d->max_pages * d->page_size;
    shift = __builtin_ctz((unsigned)d->page_size);
  } else if (cap < 0) {
    return -1;
  }
  if (d->B == 0) return 0;
  if (!d->q || !d->k_new || !d->v_new || !d->positions || !d->inv_freq || !d->suffix_lens) return -1;
  if (cap > 0 && (!d->k_store || !d->v_store)) return -1;
  Params P;
  P.q = static_cast<char*>(d->q); P.k_new = static_cast<const char*>(d->k_new); P.v_new = static_cast<const char*>(d->v_new);
  P.pos = d->positions; P.inv_freq = d->inv_freq;
  P.ks = static_cast<char*>(d->k_store); P.vs = static_cast<char*>(d->v_store);
  P.table = d->block_table; P.lens = d->suffix_lens; P.active = d->seq_active;
  P.B = d->B; P.Hq = d->Hq; P.Hkv = d->Hkv; P.d = d->d; P.Ls_cap = cap;
  P.page_shift = shift; P.max_pages = d->max_pages; P.n_pages = d->n_pages;
  P.s0 = d->sections[0]; P.s1 = d->sections[1];
  P.kscale = d->dtype == 2 ? d->k_scale : nullptr; P.vscale = d->dtype == 2 ? d->v_scale : nullptr;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if (d->dtype == 0)      hipLaunchKernelGGL((kv_append_rope_kernel<float, false>), dim3(d->B), dim3(256), 0, st, P);
  else if (d->dtype == 1) hipLaunchKernelGGL((kv_append_rope_kernel<uint16_t, false>), dim3(d->B), dim3(256), 0, st, P);
  else                    hipLaunchKernelGGL((kv_append_rope_kernel<uint16_t, true>), dim3(d->B), dim3(256), 0, st, P);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}
