// Simple decode-attention kernel: one 64-lane wavefront per (sequence, query
// head).  No prefix sharing, no key split, plain vector ALU.  It is the fp32
// path and the unoptimised GPU reference row of the benchmark.  K/V stores may
// also hold e4m3 bytes (decoded here with integer operations, not with the
// hardware converter the matrix-core path uses).
//
// For its (b, h) the wavefront walks the prompt prefix of prompt p = b / G and
// then the sequence's own suffix (Sec. 3.1 of the paper: the state is the
// prompt followed by the generated tokens) in tiles of 64 keys: lane n scores
// key n, the tile's max and sum are reduced across the wavefront (online
// softmax), and for the value contraction lane c owns output columns c, c+64.
#include "rlda_internal.h"

namespace rlda {
namespace {

struct SimpleParams {
  const void* q; const void* kp; const void* vp; const void* ks; const void* vs;
  const int32_t* plens; const int32_t* slens;
  float* out; float* lse;
  int G, Hq, Hkv, Lp_cap, Ls_cap;
  float scale;
  const int32_t* table;       // paged suffix store: [B, max_pages] page ids, else null
  int page_shift, max_pages, n_pages;
  const uint8_t* active;      // finished-sequence flags or null
  const float* kscale; const float* vscale;   // per-KV-head factors of an e4m3 store, or null
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

template <typename T> struct Vec;   // 16-byte vector of T
template <> struct Vec<float> {
  static constexpr int N = 4;
  __device__ static void load(const float* p, float (&f)[4]) {
    const float4 v = *reinterpret_cast<const float4*>(p);
    f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
  }
  __device__ static float one(const float* p) { return *p; }
};
template <> struct Vec<uint16_t> {
  static constexpr int N = 8;
  __device__ static void load(const uint16_t* p, float (&f)[8]) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(w[i] << 16);
      f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  __device__ static float one(const uint16_t* p) { return bf16_to_f32(*p); }
};

// e4m3: 1 sign, 4 exponent bits (bias 7), 3 mantissa bits; exponent 0 is subnormal, S.1111.111 is NaN
__device__ __forceinline__ float e4m3_to_f32(uint32_t b) {
  const uint32_t em = b & 0x7Fu, sign = (b & 0x80u) << 24;
  float v;
  if (em == 0x7Fu) v = __uint_as_float(0x7FC00000u);
  else if (em < 8u) v = (float)em * 0.001953125f;                       // m * 2^-9
  else v = __uint_as_float((em << 20) + (120u << 23));                  // exponent e - 7 + 127
  return __uint_as_float(__float_as_uint(v) | sign);
}
template <> struct Vec<uint8_t> {
  static constexpr int N = 16;
  __device__ static void load(const uint8_t* p, float (&f)[16]) {
    const uint4 v = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 16; ++i) f[i] = e4m3_to_f32((w[i >> 2] >> (8 * (i & 3))) & 0xFFu);
  }
  __device__ static float one(const uint8_t* p) { return e4m3_to_f32(*p); }
};

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// TQ: element type of q; T: element type of the K/V stores
template <typename TQ, typename T, int D>
__global__ void __launch_bounds__(64) simple_kernel(SimpleParams P) {
  constexpr int VN = Vec<T>::N;
  constexpr int NC = D / 64;                 // output columns per lane
  __shared__ __attribute__((aligned(16))) float q_sh[D];
  __shared__ float p_sh[64];
  __shared__ size_t r_sh[64];                // element offset of each of the tile's key rows

  const int lane = threadIdx.x;
  const int b = blockIdx.x / P.Hq, h = blockIdx.x % P.Hq;
  const int p = b / P.G;
  const int j = h / (P.Hq / P.Hkv);
  const bool live = !P.active || P.active[b] != 0;   // a finished sequence has no keys: out = 0, lse = -inf
  const int Lp = live ? min(max(P.plens[p], 0), P.Lp_cap) : 0;
  const int Ls = live ? min(max(P.slens[b], 0), P.Ls_cap) : 0;

  const TQ* q = static_cast<const TQ*>(P.q) + ((size_t)b * P.Hq + h) * D;
  for (int c = lane; c < D; c += 64) q_sh[c] = Vec<TQ>::one(q + c);
  const float kfac = P.scale * (P.kscale ? P.kscale[j] : 1.f), vfac = P.vscale ? P.vscale[j] : 1.f;
  __syncthreads();

  float m = -INFINITY, l = 0.f, acc[NC];
#pragma unroll
  for (int i = 0; i < NC; ++i) acc[i] = 0.f;

  for (int seg = 0; seg < 2; ++seg) {
    const int len = seg == 0 ? Lp : Ls;
    const bool paged = seg == 1 && P.table != nullptr;
    const T* kb = seg == 0 ? static_cast<const T*>(P.kp) + ((size_t)p * P.Hkv + j) * (size_t)P.Lp_cap * D
                : paged    ? static_cast<const T*>(P.ks)
                           : static_cast<const T*>(P.ks) + ((size_t)b * P.Hkv + j) * (size_t)P.Ls_cap * D;
    const T* vb = seg == 0 ? static_cast<const T*>(P.vp) + ((size_t)p * P.Hkv + j) * (size_t)P.Lp_cap * D
                : paged    ? static_cast<const T*>(P.vs)
                           : static_cast<const T*>(P.vs) + ((size_t)b * P.Hkv + j) * (size_t)P.Ls_cap * D;
    for (int n0 = 0; n0 < len; n0 += 64) {
      const int cnt = min(64, len - n0);
      float s = -INFINITY;
      __syncthreads();                                    // r_sh of the previous tile is no longer read
      if (lane < cnt) {
        const int n = n0 + lane;
        size_t row = (size_t)n;
        if (paged) {                                      // row n % page_size of the page the table names
          const int pg = min(max(P.table[(size_t)b * P.max_pages + (n >> P.page_shift)], 0), P.n_pages - 1);
          row = (((size_t)pg * P.Hkv + j) << P.page_shift) + (n & ((1 << P.page_shift) - 1));
        }
        r_sh[lane] = row * D;
        const T* kr = kb + row * D;
        float dot = 0.f;
#pragma unroll 4
        for (int c = 0; c < D; c += VN) {
          float kf[VN];
          Vec<T>::load(kr + c, kf);
#pragma unroll
          for (int x = 0; x < VN; ++x) dot = fmaf(q_sh[c + x], kf[x], dot);
        }
        s = dot * kfac;
      }
      const float m_new = fmaxf(m, wave_max(s));          // finite: the tile has >= 1 key
      const float alpha = expf(m - m_new);               // m = -inf -> 0
      const float pr = expf(s - m_new);                  // masked lanes -> 0
      l = l * alpha + wave_sum(pr);
      m = m_new;
      __syncthreads();
      p_sh[lane] = pr;
      __syncthreads();
#pragma unroll
      for (int i = 0; i < NC; ++i) acc[i] *= alpha;
      for (int n = 0; n < cnt; ++n) {
        const float pn = p_sh[n];
        const T* vr = vb + r_sh[n];
#pragma unroll
        for (int i = 0; i < NC; ++i) acc[i] = fmaf(pn, Vec<T>::one(vr + lane + 64 * i), acc[i]);
      }
    }
  }
  float* o = P.out + ((size_t)b * P.Hq + h) * D;
  const float inv = l > 0.f ? vfac / l : 0.f;
#pragma unroll
  for (int i = 0; i < NC; ++i) o[lane + 64 * i] = acc[i] * inv;
  if (P.lse && lane == 0) P.lse[(size_t)b * P.Hq + h] = l > 0.f ? m + logf(l) : -INFINITY;
}

// ---- stand-alone combine: one thread per (row, 4 columns)
template <int D>
__global__ void __launch_bounds__(256) combine_kernel(const float* __restrict__ o_parts, const float* __restrict__ lse_parts,
                                                      int n_parts, int64_t n_rows, float* __restrict__ out,
                                                      float* __restrict__ lse) {
  constexpr int TPR = D / 4;                              // threads per row
  const int64_t row = (int64_t)blockIdx.x * (256 / TPR) + threadIdx.x / TPR;
  const int c4 = threadIdx.x % TPR;
  if (row >= n_rows) return;
  float M = -INFINITY;
  for (int i = 0; i < n_parts; ++i) M = fmaxf(M, lse_parts[(int64_t)i * n_rows + row]);
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  float z = 0.f;
  if (M > -INFINITY) {
    for (int i = 0; i < n_parts; ++i) {
      const float li = lse_parts[(int64_t)i * n_rows + row];
      if (li == -INFINITY) continue;                      // empty part: never touch its o (may be garbage)
      const float w = expf(li - M);
      const float4 o = *reinterpret_cast<const float4*>(o_parts + ((int64_t)i * n_rows + row) * D + 4 * c4);
      z += w;
      acc.x = fmaf(w, o.x, acc.x); acc.y = fmaf(w, o.y, acc.y);
      acc.z = fmaf(w, o.z, acc.z); acc.w = fmaf(w, o.w, acc.w);
    }
    const float inv = 1.f / z;
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
  }
  *reinterpret_cast<float4*>(out + row * D + 4 * c4) = acc;
  if (lse && c4 == 0) lse[row] = M > -INFINITY ? M + logf(z) : -INFINITY;
}

}  // namespace

hipError_t launch_simple(const Problem& ds, hipStream_t stream) {
  SimpleParams P{ds.q, ds.k_prefix, ds.v_prefix, ds.k_suffix, ds.v_suffix, ds.prefix_lens, ds.suffix_lens,
                 ds.out, ds.lse, ds.G, ds.Hq, ds.Hkv, ds.Lp_cap, ds.Ls_cap, ds.scale,
                 ds.block_table, ds.page_shift, ds.max_pages, ds.n_pages, ds.seq_active, ds.k_scale, ds.v_scale};
  const int64_t blocks = (int64_t)ds.P * ds.G * ds.Hq;
  if (blocks == 0) return hipSuccess;
  const dim3 grid((unsigned)blocks), block(64);
  if (ds.dtype == RLDA_F32) {
    if (ds.d == 64) hipLaunchKernelGGL((simple_kernel<float, float, 64>), grid, block, 0, stream, P);
    else            hipLaunchKernelGGL((simple_kernel<float, float, 128>), grid, block, 0, stream, P);
  } else if (ds.dtype == RLDA_BF16_KV8) {
    if (ds.d == 64) hipLaunchKernelGGL((simple_kernel<uint16_t, uint8_t, 64>), grid, block, 0, stream, P);
    else            hipLaunchKernelGGL((simple_kernel<uint16_t, uint8_t, 128>), grid, block, 0, stream, P);
  } else {
    if (ds.d == 64) hipLaunchKernelGGL((simple_kernel<uint16_t, uint16_t, 64>), grid, block, 0, stream, P);
    else            hipLaunchKernelGGL((simple_kernel<uint16_t, uint16_t, 128>), grid, block, 0, stream, P);
  }
  return hipGetLastError();
}

hipError_t launch_combine(const float* o_parts, const float* lse_parts, int n_parts, int64_t n_rows, int d,
                          float* out, float* lse, hipStream_t stream) {
  if (n_rows == 0) return hipSuccess;
  const int rows_per_block = 256 / (d / 4);
  const dim3 grid((unsigned)((n_rows + rows_per_block - 1) / rows_per_block)), block(256);
  if (d == 64) hipLaunchKernelGGL((combine_kernel<64>), grid, block, 0, stream, o_parts, lse_parts, n_parts, n_rows, out, lse);
  else         hipLaunchKernelGGL((combine_kernel<128>), grid, block, 0, stream, o_parts, lse_parts, n_parts, n_rows, out, lse);
  return hipGetLastError();
}

}  // namespace rlda
