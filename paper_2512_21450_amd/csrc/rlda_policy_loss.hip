// Scoring, group advantage estimation and the clipped policy loss (Eq. 6 of the paper; Sec. 3.2.2
// scoring, advantage-estimation and policy-update stages).  Element-wise work over [B] and [B, T]
// arrays with deterministic reductions: per-thread partial sums in a fixed order, a fixed tree
// inside the workgroup, and a further kernel that folds the per-sequence sums in fp64.
//
// rl_group_advantage: one workgroup per prompt.  The group's mean and deviations are taken in
// fp64: with fp32 a group whose samples all earned the same reward can get a mean one ulp off and,
// after division by (std + eps), advantages of several percent out of pure rounding.
//
// rl_policy_loss: one workgroup per sequence streams its valid tokens once (HBM-bound: 2 to 4
// input arrays and one output array of 4 bytes per token).
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/rl_policy_loss.h"

namespace {

constexpr int NT = 256;

// fixed-order tree over the workgroup; every thread returns the total
template <typename T>
__device__ __forceinline__ T block_sum(T v, T* sh) {
  const int tid = threadIdx.x;
  __syncthreads();                                          // sh may still be read from a previous call
  sh[tid] = v;
  __syncthreads();
#pragma unroll
  for (int s = NT / 2; s > 0; s >>= 1) {
    if (tid < s) sh[tid] += sh[tid + s];
    __syncthreads();
  }
  return sh[0];
}

struct AdvParams {
  const float* metrics; const float* weights; float* rewards; float* adv;
  int P, G, M, mode, unbiased;
  float eps;
};

__global__ void __launch_bounds__(NT) group_advantage_kernel(const AdvParams A) {
  __shared__ double sh[NT];
  const int p = blockIdx.x, tid = threadIdx.x;
  const size_t B = (size_t)A.P * A.G;
  float r[4];                                               // G <= 4 * NT samples per prompt
  double s = 0.0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int g = tid + k * NT;
    r[k] = 0.f;
    if (g < A.G) {
      const size_t b = (size_t)p * A.G + g;
      float acc = 0.f;
      for (int m = 0; m < A.M; ++m) acc = fmaf(A.weights[m], A.metrics[(size_t)m * B + b], acc);
      r[k] = acc;
      if (A.rewards) A.rewards[b] = acc;
      s += (double)acc;
    }
  }
  const double sum = block_sum<double>(s, sh), mean = sum / A.G;
  double q = 0.0;
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (tid + k * NT < A.G) { const double d = (double)r[k] - mean; q += d * d; }
  const double ss = block_sum<double>(q, sh);
  const int div = A.unbiased ? A.G - 1 : A.G;
  const double sd = div > 0 ? sqrt(ss / div) : 0.0;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int g = tid + k * NT;
    if (g >= A.G) continue;
    const double d = (double)r[k] - mean;
    double a;
    if (A.mode == RL_ADV_GROUP_CENTER) a = d;
    else if (A.mode == RL_ADV_LEAVE_ONE_OUT) a = A.G > 1 ? (double)r[k] - (sum - (double)r[k]) / (A.G - 1) : 0.0;
    else a = d / (sd + (double)A.eps);
    A.adv[(size_t)p * A.G + g] = (float)a;
  }
}

struct LossParams {
  const float* lp; const float* old; const float* adv; const float* kl; const float* ent;
  const int32_t* lens;
  float* grad; float* stats;
  long long* counts;                                        // [2] valid tokens, sequences with tokens (first 256 workspace bytes)
  float* part;                                              // [B][8] per-sequence sums
  int B, T, form, agg;
  int64_t stride;
  float lo, hi, beta_kl, beta_ent;
};

__device__ __forceinline__ int clamp_len(int v, int T) { return v < 0 ? 0 : (v > T ? T : v); }

// batch totals the token weights need: valid tokens, sequences with tokens (one workgroup)
__global__ void __launch_bounds__(NT) policy_count_kernel(const LossParams L) {
  __shared__ long long sh[NT];
  long long a = 0, c = 0;
  for (int b = threadIdx.x; b < L.B; b += NT) {
    const int n = clamp_len(L.lens[b], L.T);
    a += n; c += n > 0;
  }
  a = block_sum<long long>(a, sh);
  c = block_sum<long long>(c, sh);
  if (threadIdx.x == 0) { L.counts[0] = a; L.counts[1] = c; }
}

// per-token arithmetic; accumulates into sums[6] = (term, kl, entropy, flat-branch count, rho, old - new)
__device__ __forceinline__ float token_term(const LossParams& L, float lp, float old, float kl, float ent, float A,
                                            float w, float (&sums)[6]) {
  const float rho = expf(lp - old);
  const float ra = rho * A;
  float term;
  bool flat;
  if (L.form == RL_PG_AS_PRINTED) {
    flat = rho > L.hi;
    term = fminf(rho, L.hi) * A;
  } else {
    const float ca = fminf(fmaxf(rho, L.lo), L.hi) * A;
    flat = !(ra <= ca);                                     // inside the range both products are equal: not flat
    term = fminf(ra, ca);
  }
  sums[0] += term; sums[1] += kl; sums[2] += ent; sums[3] += flat ? 1.f : 0.f; sums[4] += rho; sums[5] += old - lp;
  return flat ? 0.f : -w * ra;
}

// One workgroup per sequence.  VEC: rows are 16-byte aligned and T is handled four tokens per thread
// and step (one 16-byte load per array); otherwise one token per thread and step.  Either way a
// thread adds its tokens in increasing t, the 64 lanes of a wavefront are folded by a fixed
// butterfly and the four wavefronts in order, so the sums do not depend on anything but the data.
template <bool VEC>
__global__ void __launch_bounds__(NT) policy_loss_kernel(const LossParams L) {
  __shared__ float shf[NT / 64][6];
  const int b = blockIdx.x, tid = threadIdx.x;
  const long long n_tok = L.counts[0], n_seq = L.counts[1];
  const int len = clamp_len(L.lens[b], L.T);
  float w = 0.f;                                            // weight of one of this sequence's tokens in the aggregate
  if (len > 0) w = L.agg == RL_AGG_SEQ_MEAN ? (float)(1.0 / ((double)len * (double)n_seq)) : (float)(1.0 / (double)n_tok);
  const float A = L.adv[b];
  const size_t row = (size_t)b * L.stride;
  float sums[6] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (VEC) {
    for (int t = 4 * tid; t < L.T; t += 4 * NT) {
      float g[4] = {0.f, 0.f, 0.f, 0.f};
      if (t < len) {                                        // the four tokens t .. t+3 exist as memory (T % 4 == 0); some may be padding
        const float4 lp = *reinterpret_cast<const float4*>(L.lp + row + t), old = *reinterpret_cast<const float4*>(L.old + row + t);
        const float4 kl = L.kl ? *reinterpret_cast<const float4*>(L.kl + row + t) : make_float4(0.f, 0.f, 0.f, 0.f);
        const float4 en = L.ent ? *reinterpret_cast<const float4*>(L.ent + row + t) : make_float4(0.f, 0.f, 0.f, 0.f);
        const float lpv[4] = {lp.x, lp.y, lp.z, lp.w}, ov[4] = {old.x, old.y, old.z, old.w};
        const float kv[4] = {kl.x, kl.y, kl.z, kl.w}, ev[4] = {en.x, en.y, en.z, en.w};
#pragma unroll
        for (int k = 0; k < 4; ++k)
          if (t + k < len) g[k] = token_term(L, lpv[k], ov[k], kv[k], ev[k], A, w, sums);
      }
      if (L.grad) *reinterpret_cast<float4*>(L.grad + row + t) = make_float4(g[0], g[1], g[2], g[3]);
    }
  } else {
    for (int t = tid; t < L.T; t += NT) {
      float g = 0.f;
      if (t < len)
        g = token_term(L, L.lp[row + t], L.old[row + t], L.kl ? L.kl[row + t] : 0.f, L.ent ? L.ent[row + t] : 0.f, A, w, sums);
      if (L.grad) L.grad[row + t] = g;
    }
  }
#pragma unroll
  for (int k = 0; k < 6; ++k) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sums[k] += __shfl_xor(sums[k], o, 64);
  }
  if ((tid & 63) == 0) {
#pragma unroll
    for (int k = 0; k < 6; ++k) shf[tid >> 6][k] = sums[k];
  }
  __syncthreads();
  if (tid < 6) L.part[(size_t)b * 8 + tid] = ((shf[0][tid] + shf[1][tid]) + shf[2][tid]) + shf[3][tid];
}

__global__ void __launch_bounds__(NT) policy_loss_reduce_kernel(const LossParams L) {
  __shared__ double shd[NT];
  const int tid = threadIdx.x;
  const long long n_tok = L.counts[0], n_seq = L.counts[1];
  double acc[6] = {0, 0, 0, 0, 0, 0};
  for (int b = tid; b < L.B; b += NT) {
    const int len = clamp_len(L.lens[b], L.T);
    if (len == 0) continue;
    const float* p = L.part + (size_t)b * 8;
    const double wa = L.agg == RL_AGG_SEQ_MEAN ? 1.0 / ((double)len * (double)n_seq) : 1.0 / (double)n_tok;
    const double wt = 1.0 / (double)n_tok;
    acc[0] += wa * p[0]; acc[1] += wa * p[1]; acc[2] += wa * p[2];
    acc[3] += wt * p[3]; acc[4] += wt * p[4]; acc[5] += wt * p[5];
  }
#pragma unroll
  for (int k = 0; k < 6; ++k) acc[k] = block_sum<double>(acc[k], shd);
  if (tid == 0) {
    L.stats[0] = (float)(-acc[0] + (double)L.beta_kl * acc[1] - (double)L.beta_ent * acc[2]);
    L.stats[1] = (float)acc[0]; L.stats[2] = (float)acc[1]; L.stats[3] = (float)acc[2];
    L.stats[4] = (float)acc[3]; L.stats[5] = (float)acc[4]; L.stats[6] = (float)acc[5];
    L.stats[7] = (float)n_tok;
  }
}

int check(const rl_policy_loss_desc* d) {
  if (!d) return -1;
  if (d->struct_size != sizeof(rl_policy_loss_desc)) return -4;
  if (d->B < 0 || d->T < 0) return -1;
  if (!(d->clip_low >= 0.f) || !(d->clip_high >= 0.f)) return -1;
  if (d->form != RL_PG_PPO_CLIP && d->form != RL_PG_AS_PRINTED) return -2;
  if (d->agg != RL_AGG_TOKEN_MEAN && d->agg != RL_AGG_SEQ_MEAN) return -2;
  if (d->row_stride < d->T) return -2;
  return 0;
}

}  // namespace

extern "C" {

int rl_group_advantage(const rl_group_advantage_desc* d, void* hip_stream) {
  if (!d) return -1;
  if (d->struct_size != sizeof(rl_group_advantage_desc)) return -4;
  if (d->P < 0 || d->G < 0 || !(d->eps >= 0.f)) return -1;
  if (d->mode != RL_ADV_GROUP_NORM && d->mode != RL_ADV_GROUP_CENTER && d->mode != RL_ADV_LEAVE_ONE_OUT) return -2;
  if (d->G > 4 * NT || d->n_metrics < 1 || d->n_metrics > 64) return -2;
  if (d->P == 0 || d->G == 0) return 0;
  if (!d->metrics || !d->weights || !d->advantages) return -1;
  const AdvParams A{d->metrics, d->weights, d->rewards, d->advantages, d->P, d->G, d->n_metrics, d->mode,
                    d->unbiased, d->eps};
  hipLaunchKernelGGL(group_advantage_kernel, dim3(d->P), dim3(NT), 0, static_cast<hipStream_t>(hip_stream), A);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

size_t rl_policy_loss_workspace_bytes(const rl_policy_loss_desc* d) {
  if (check(d) != 0) return 0;
  return 256 + (size_t)d->B * 8 * sizeof(float);
}

int rl_policy_loss(const rl_policy_loss_desc* d, void* hip_stream) {
  const int rc = check(d);
  if (rc != 0) return rc;
  if (!d->stats) return -1;
  if (d->B > 0 && (!d->advantages || !d->lens)) return -1;
  if (d->B > 0 && d->T > 0 && (!d->logprob || !d->old_logprob)) return -1;
  const size_t need = rl_policy_loss_workspace_bytes(d);
  if (need > 0 && (!d->workspace || d->workspace_bytes < need)) return -3;
  if (need > 0 && (reinterpret_cast<uintptr_t>(d->workspace) & 255u)) return -3;
  LossParams L;
  L.lp = d->logprob; L.old = d->old_logprob; L.adv = d->advantages; L.kl = d->kl; L.ent = d->entropy;
  L.lens = d->lens; L.grad = d->grad_logprob; L.stats = d->stats;
  L.counts = static_cast<long long*>(d->workspace);
  L.part = reinterpret_cast<float*>(static_cast<char*>(d->workspace) + 256);
  L.B = d->B; L.T = d->T; L.form = d->form; L.agg = d->agg; L.stride = d->row_stride;
  L.lo = 1.f - d->clip_low; L.hi = 1.f + d->clip_high; L.beta_kl = d->beta_kl; L.beta_ent = d->beta_ent;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  hipLaunchKernelGGL(policy_count_kernel, dim3(1), dim3(NT), 0, st, L);
  if (hipGetLastError() != hipSuccess) return -5;
  if (d->B > 0) {
    auto aligned = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; };
    const bool vec = d->T % 4 == 0 && d->row_stride % 4 == 0 && aligned(d->logprob) && aligned(d->old_logprob) &&
                     aligned(d->kl) && aligned(d->entropy) && aligned(d->grad_logprob);
    if (vec) hipLaunchKernelGGL(policy_loss_kernel<true>, dim3(d->B), dim3(NT), 0, st, L);
    else     hipLaunchKernelGGL(policy_loss_kernel<false>, dim3(d->B), dim3(NT), 0, st, L);
    if (hipGetLastError() != hipSuccess) return -5;
  }
  hipLaunchKernelGGL(policy_loss_reduce_kernel, dim3(1), dim3(NT), 0, st, L);
  return hipGetLastError() == hipSuccess ? 0 : -5;
}

}  // extern "C"
