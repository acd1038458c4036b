// Per-token policy statistics from vocabulary logits: log-prob of the sampled token, entropy,
// KL to a reference policy (Sec. 2.2 of the paper: importance ratio r_t, entropy bonus,
// KL-to-reference; Omega and L^PG of Eq. 6).
//
// HBM-bound streaming reduction.  A row is cut into S contiguous splits (S chosen on the host
// so that the grid fills the chip); workgroup (split, row) streams its part with 16-byte
// nontemporal loads and keeps, per thread, an online-softmax state
//   m, s = sum e^(a-m), t = sum e^(a-m) a          for a = logits * inv_temperature
//   mr, sr = sum e^(b-mr), u = sum e^(a-m) b       for b = ref_logits * inv_temperature
// which is merged over the wavefront (xor shuffles), the workgroup (LDS) and, when S > 1, the
// splits (second kernel, one wavefront per row).  Then
//   lse = m + ln s, entropy = lse - t/s, kl = (t - u)/s - lse + (mr + ln sr).
// All merges have a fixed order, so results do not change from call to call.
//
// The inner loop is close to the vector-ALU limit at HBM speed (bf16: ~12 issue slots per
// logit are available at 6.5 TB/s, the exponential alone takes 4), so the state is kept in
// base 2 (a, b pre-multiplied by inv_temperature * log2 e: the hardware exponential is 2^x) and
// masked logits (-inf) are clamped to -1e30, which makes 0 * a finite without a branch and
// cannot overflow a sum.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/rl_token_logprob.h"

namespace {

// threads per workgroup: 256 when there are thousands of workgroups, 1024 when there is about one
// per compute unit (a decode step's few hundred rows), so that either way the chip is full
constexpr int UNR = 4;             // independent 16-byte loads in flight per thread
constexpr int MAX_SPLITS = 64;     // one lane per split in the final merge

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

struct Params {
  const char* logits; const char* ref; const int32_t* ids;
  float* logprob; float* lse; float* entropy; float* ref_logprob; float* kl;
  float* part;                     // [n_rows][S][6]
  long long stride;                // elements
  int V, S, chunk;                 // chunk: elements per split, multiple of the vector width
  float k2;                        // inv_temperature * log2(e): logits -> base-2 exponents
};

constexpr float LN2 = 0.69314718055994531f;
constexpr float MASKED = -1e30f;        // stands for a logit of -inf inside the reductions

struct Acc { float m, s, t, mr, sr, u; };

__device__ __forceinline__ Acc acc_empty() { return Acc{-INFINITY, 0.f, 0.f, -INFINITY, 0.f, 0.f}; }

__device__ __forceinline__ float rescale(float m_old, float m_new) {      // 2^(m_old - m_new), 0 for an empty side
  return m_old == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_old - m_new);
}

template <bool REF>
__device__ __forceinline__ Acc acc_merge(const Acc& x, const Acc& y) {
  Acc r;
  r.m = fmaxf(x.m, y.m);
  const float cx = rescale(x.m, r.m), cy = rescale(y.m, r.m);
  r.s = x.s * cx + y.s * cy;
  r.t = x.t * cx + y.t * cy;
  r.u = x.u * cx + y.u * cy;
  r.mr = -INFINITY; r.sr = 0.f;
  if (REF) {
    r.mr = fmaxf(x.mr, y.mr);
    r.sr = x.sr * rescale(x.mr, r.mr) + y.sr * rescale(y.mr, r.mr);
  }
  return r;
}

template <bool REF>
__device__ __forceinline__ Acc acc_shfl_xor(const Acc& a, int mask) {
  Acc r;
  r.m = __shfl_xor(a.m, mask, 64); r.s = __shfl_xor(a.s, mask, 64); r.t = __shfl_xor(a.t, mask, 64);
  r.mr = -INFINITY; r.sr = 0.f; r.u = 0.f;
  if (REF) { r.mr = __shfl_xor(a.mr, mask, 64); r.sr = __shfl_xor(a.sr, mask, 64); r.u = __shfl_xor(a.u, mask, 64); }
  return r;
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int VN = 4;
  __device__ static void unpack(const u32x4& v, float (&f)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(v[i]);
  }
  __device__ static float one(const char* p, long long i) { return reinterpret_cast<const float*>(p)[i]; }
};
template <> struct Elem<uint16_t> {
  static constexpr int VN = 8;
  __device__ static void unpack(const u32x4& v, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = __uint_as_float(v[i] << 16);
      f[2 * i + 1] = __uint_as_float(v[i] & 0xffff0000u);
    }
  }
  __device__ static float one(const char* p, long long i) {
    return __uint_as_float((uint32_t)reinterpret_cast<const uint16_t*>(p)[i] << 16);
  }
};

// N values of the row (and of the reference row), already in base-2 units and >= MASKED, into the
// thread's state.  Next to a live logit a masked one gives e = 2^(MASKED - m) = 0 and adds 0 * MASKED = 0; a state
// that has seen masked logits only (m = MASKED) is wiped by the rescale when the first live one arrives.
template <bool REF, int N>
__device__ __forceinline__ void absorb(Acc& A, const float (&a)[N], const float (&b)[N]) {
  float cm = a[0];
#pragma unroll
  for (int i = 1; i < N; ++i) cm = fmaxf(cm, a[i]);
  const float mn = fmaxf(A.m, cm);
  const float c = rescale(A.m, mn);
  float s = A.s * c, t = A.t * c, u = A.u * c;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const float e = __builtin_amdgcn_exp2f(a[i] - mn);
    s += e;
    t = fmaf(e, a[i], t);
    if (REF) u = fmaf(e, b[i], u);
  }
  A.m = mn; A.s = s; A.t = t; A.u = u;
  if (REF) {
    float cr = b[0];
#pragma unroll
    for (int i = 1; i < N; ++i) cr = fmaxf(cr, b[i]);
    const float mrn = fmaxf(A.mr, cr);
    float sr = A.sr * rescale(A.mr, mrn);
#pragma unroll
    for (int i = 0; i < N; ++i) sr += __builtin_amdgcn_exp2f(b[i] - mrn);
    A.mr = mrn; A.sr = sr;
  }
}

// State (base-2 units) -> outputs (natural units).  a_y, b_y: the sampled token's scaled logits.
template <bool REF>
__device__ __forceinline__ void finish_row(const Params& P, long long row, const Acc& A, float a_y, float b_y, int y) {
  const bool dead = A.m <= MASKED;                           // every logit masked: no distribution
  const float lse2 = A.m + __log2f(A.s);
  const float mean_a = A.t / A.s;                           // sum_i p_i a_i
  const float lse = dead ? -INFINITY : lse2 * LN2;
  if (P.lse) P.lse[row] = lse;
  if (P.entropy) P.entropy[row] = dead ? NAN : (lse2 - mean_a) * LN2;
  // !(x > MASKED): masked, also when the sampled token's logit is NaN (read as masked like every NaN logit)
  if (P.logprob) P.logprob[row] = y < 0 ? 0.f : (y >= P.V ? NAN : (!(a_y > MASKED) ? -INFINITY : (a_y - lse2) * LN2));
  if (REF) {
    const float lse_r2 = A.mr + __log2f(A.sr);
    float mean_b = A.u / A.s;                               // sum_i p_i b_i; a masked reference logit under p > 0
    if (mean_b < -1e6f) mean_b = -INFINITY;                 // drags it towards MASKED: the KL is infinite
    if (P.kl) P.kl[row] = dead ? NAN : (mean_a - mean_b - lse2 + lse_r2) * LN2;
    if (P.ref_logprob)
      P.ref_logprob[row] = y < 0 ? 0.f : (y >= P.V ? NAN : (!(b_y > MASKED) ? -INFINITY : (b_y - lse_r2) * LN2));
  }
}

// workgroup row * S + split: partial state of elements [split * chunk, min(V, (split + 1) * chunk)) of a row
template <typename T, bool REF, int NT>
__global__ void __launch_bounds__(NT) token_partial_kernel(const Params P) {
  constexpr int VN = Elem<T>::VN;
  __shared__ Acc red[NT / 64];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const long long row = blockIdx.x / P.S;
  const int split = blockIdx.x % P.S;
  const char* za = P.logits + (size_t)row * P.stride * sizeof(T);
  const char* zb = REF ? P.ref + (size_t)row * P.stride * sizeof(T) : nullptr;
  const int c0 = split * P.chunk, c1 = min(P.V, c0 + P.chunk);
  const int v0 = c0 / VN, v1 = max(c1, c0) / VN;           // whole vectors [v0, v1)
  Acc A = acc_empty();
  for (int v = v0 + tid; v < v1; v += NT * UNR) {
    u32x4 ra[UNR], rb[UNR];
#pragma unroll
    for (int k = 0; k < UNR; ++k) {
      const int vk = v + k * NT;
      if (vk < v1) {                                        // past the end: no load, the slot is not used
        ra[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(za) + vk);
        if (REF) rb[k] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(zb) + vk);
      }
    }
#pragma unroll
    for (int k = 0; k < UNR; ++k) {
      if (v + k * NT < v1) {
        float a[VN], b[VN];
        Elem<T>::unpack(ra[k], a);
        if (REF) Elem<T>::unpack(rb[k], b);
#pragma unroll
        for (int i = 0; i < VN; ++i) {
          a[i] = fmaxf(a[i] * P.k2, MASKED);
          b[i] = REF ? fmaxf(b[i] * P.k2, MASKED) : 0.f;
        }
        absorb<REF, VN>(A, a, b);
      }
    }
  }
  // the row's last V % VN elements, one per thread, belong to the split that holds them
  const int tail0 = v1 * VN;
  if (c1 == P.V && c1 > c0 && tail0 + tid < c1) {
    float a[1] = {fmaxf(Elem<T>::one(za, tail0 + tid) * P.k2, MASKED)};
    float b[1] = {REF ? fmaxf(Elem<T>::one(zb, tail0 + tid) * P.k2, MASKED) : 0.f};
    absorb<REF, 1>(A, a, b);
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) A = acc_merge<REF>(A, acc_shfl_xor<REF>(A, o));
  if (lane == 0) red[wv] = A;
  __syncthreads();
  if (tid == 0) {
    Acc R = red[0];
#pragma unroll
    for (int k = 1; k < NT / 64; ++k) R = acc_merge<REF>(R, red[k]);
    if (P.S == 1) {
      const int y = P.ids[row];
      const bool ok = y >= 0 && y < P.V;
      finish_row<REF>(P, row, R, ok ? Elem<T>::one(za, y) * P.k2 : 0.f,
                      REF && ok ? Elem<T>::one(zb, y) * P.k2 : 0.f, y);
    } else {
      float* o = P.part + ((size_t)row * P.S + split) * 6;
      o[0] = R.m; o[1] = R.s; o[2] = R.t; o[3] = R.mr; o[4] = R.sr; o[5] = R.u;
    }
  }
}

// one wavefront per row: lane i takes split i, merged in a fixed butterfly order
template <typename T, bool REF>
__global__ void __launch_bounds__(64) token_final_kernel(const Params P) {
  const long long row = blockIdx.x;
  const int lane = threadIdx.x;
  Acc A = acc_empty();
  if (lane < P.S) {
    const float* o = P.part + ((size_t)row * P.S + lane) * 6;
    A = Acc{o[0], o[1], o[2], o[3], o[4], o[5]};
  }
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) A = acc_merge<REF>(A, acc_shfl_xor<REF>(A, o));
  if (lane == 0) {
    const char* za = P.logits + (size_t)row * P.stride * sizeof(T);
    const char* zb = REF ? P.ref + (size_t)row * P.stride * sizeof(T) : nullptr;
    const int y = P.ids[row];
    const bool ok = y >= 0 && y < P.V;
    finish_row<REF>(P, row, A, ok ? Elem<T>::one(za, y) * P.k2 : 0.f,
                    REF && ok ? Elem<T>::one(zb, y) * P.k2 : 0.f, y);
  }
}

int check(const rl_token_logprob_desc* d) {
  if (!d) return -1;
  if (d->struct_size != sizeof(rl_token_logprob_desc)) return -4;
  if (d->n_rows < 0 || d->vocab < 1 || d->row_stride < 0) return -1;
  if (!(d->inv_temperature > 0.f) || d->inv_temperature > 3.0e38f) return -1;   // masked (-inf) logits must stay -inf after scaling
  if (d->dtype != 0 && d->dtype != 1) return -2;
  const int vn = d->dtype == 0 ? 4 : 8;
  if (d->row_stride < d->vocab || d->row_stride % vn != 0) return -2;
  if (d->n_rows > ((long long)1 << 31) / MAX_SPLITS - 1) return -2;   // rows * splits is the grid size
  if (d->vocab > (1 << 30)) return -2;
  return 0;
}

// Splits per row.  From about one row per compute unit upwards a row is not split (one kernel, no
// merge pass, which costs more than a slightly uneven last wave of workgroups); fewer rows are
// split until there is a workgroup per compute unit, but never below 8192 logits per workgroup.
int splits_for(const rl_token_logprob_desc* d) {
  if (d->n_rows <= 0 || d->n_rows >= 192) return 1;
  long long s = (256 + d->n_rows - 1) / d->n_rows;
  const long long by_size = d->vocab / 8192;
  if (s > by_size) s = by_size;
  if (s > MAX_SPLITS) s = MAX_SPLITS;
  return s < 1 ? 1 : (int)s;
}

thread_local hipError_t g_last = hipSuccess;

}  // namespace

extern "C" {

size_t rl_token_logprob_workspace_bytes(const rl_token_logprob_desc* d) {
  if (check(d) != 0) return 0;
  const int S = splits_for(d);
  return S == 1 ? 0 : (size_t)d->n_rows * S * 6 * sizeof(float);
}

int rl_token_logprob(const rl_token_logprob_desc* d, void* hip_stream) {
  const int rc = check(d);
  if (rc != 0) return rc;
  if (d->n_rows == 0) return 0;
  if (!d->logits || !d->token_ids) return -1;
  if (!d->ref_logits && (d->kl || d->ref_logprob)) return -1;
  if ((reinterpret_cast<uintptr_t>(d->logits) & 15u) || (reinterpret_cast<uintptr_t>(d->ref_logits) & 15u)) return -2;
  const int S = splits_for(d);
  const size_t need = S == 1 ? 0 : (size_t)d->n_rows * S * 6 * sizeof(float);
  if (need > 0 && (!d->workspace || d->workspace_bytes < need || (reinterpret_cast<uintptr_t>(d->workspace) & 255u)))
    return -3;
  const int vn = d->dtype == 0 ? 4 : 8;
  Params P;
  P.logits = static_cast<const char*>(d->logits); P.ref = static_cast<const char*>(d->ref_logits);
  P.ids = d->token_ids;
  P.logprob = d->logprob; P.lse = d->lse; P.entropy = d->entropy; P.ref_logprob = d->ref_logprob; P.kl = d->kl;
  P.part = static_cast<float*>(d->workspace);
  P.stride = d->row_stride; P.V = d->vocab; P.S = S;
  const int per = (d->vocab + S - 1) / S;
  P.chunk = (per + vn - 1) / vn * vn;
  P.k2 = d->inv_temperature * 1.4426950408889634f;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const dim3 grid((unsigned)(d->n_rows * S)), fin((unsigned)d->n_rows);
  const bool ref = d->ref_logits != nullptr;
  const bool wide = d->n_rows * S <= 512;                  // few workgroups: make each one 16 wavefronts
#define RLTL_LAUNCH(T)                                                                                      \
  do {                                                                                                      \
    if (wide) {                                                                                             \
      if (ref) hipLaunchKernelGGL((token_partial_kernel<T, true, 1024>), grid, dim3(1024), 0, st, P);       \
      else     hipLaunchKernelGGL((token_partial_kernel<T, false, 1024>), grid, dim3(1024), 0, st, P);      \
    } else {                                                                                                \
      if (ref) hipLaunchKernelGGL((token_partial_kernel<T, true, 256>), grid, dim3(256), 0, st, P);         \
      else     hipLaunchKernelGGL((token_partial_kernel<T, false, 256>), grid, dim3(256), 0, st, P);        \
    }                                                                                                       \
    if (S > 1) {                                                                                            \
      if (ref) hipLaunchKernelGGL((token_final_kernel<T, true>), fin, dim3(64), 0, st, P);                  \
      else     hipLaunchKernelGGL((token_final_kernel<T, false>), fin, dim3(64), 0, st, P);                 \
    }                                                                                                       \
  } while (0)
  if (d->dtype == 0) RLTL_LAUNCH(float); else RLTL_LAUNCH(uint16_t);
#undef RLTL_LAUNCH
  g_last = hipGetLastError();
  return g_last == hipSuccess ? 0 : -5;
}

}  // extern "C"
