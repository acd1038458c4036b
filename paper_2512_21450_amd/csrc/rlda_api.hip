// C-ABI layer: argument validation, kernel-family selection, enqueue.
// Validation and the workspace/plan queries are pure host code and work
// without a GPU; only rl_decode_attn / rl_lse_combine touch the HIP runtime.
#include "rlda_internal.h"

namespace {

int check_shape(const rlda_desc* ds) {
  if (!ds) return RLDA_ERR_INVALID;
  if (ds->struct_size != sizeof(rlda_desc)) return RLDA_ERR_STRUCT_SIZE;
  if (ds->P < 0 || ds->G < 0 || ds->Hq <= 0 || ds->Hkv <= 0 || ds->d <= 0 || ds->Lp_cap < 0 || ds->Ls_cap < 0)
    return RLDA_ERR_INVALID;
  if (ds->dtype != RLDA_F32 && ds->dtype != RLDA_BF16) return RLDA_ERR_UNSUPPORTED;
  if (ds->algo != RLDA_ALGO_AUTO && ds->algo != RLDA_ALGO_SIMPLE && ds->algo != RLDA_ALGO_SHARED)
    return RLDA_ERR_UNSUPPORTED;
  if (ds->d != 64 && ds->d != 128) return RLDA_ERR_UNSUPPORTED;
  if (ds->Hq % ds->Hkv != 0) return RLDA_ERR_UNSUPPORTED;
  // index arithmetic in the kernels is 32-bit for (sequence, head) counts
  if ((int64_t)ds->P * ds->G * ds->Hq > (int64_t)1 << 30) return RLDA_ERR_UNSUPPORTED;
  return RLDA_OK;
}

int plan(const rlda_desc* ds) {
  const int rc = check_shape(ds);
  if (rc != RLDA_OK) return rc;
  if (ds->algo == RLDA_ALGO_SIMPLE) return RLDA_ALGO_SIMPLE;
  if (rlda::shared_supported(*ds)) return RLDA_ALGO_SHARED;
  return ds->algo == RLDA_ALGO_SHARED ? RLDA_ERR_UNSUPPORTED : RLDA_ALGO_SIMPLE;
}

thread_local hipError_t g_last_hip_error = hipSuccess;

}  // namespace

extern "C" {

const char* rl_decode_attn_last_hip_error(void) { return hipGetErrorString(g_last_hip_error); }

int rl_decode_attn_version(void) { return 100; }

const char* rl_decode_attn_strerror(int code) {
  switch (code) {
    case RLDA_OK: return "success";
    case RLDA_ERR_INVALID: return "invalid argument (null pointer or negative size)";
    case RLDA_ERR_UNSUPPORTED: return "unsupported shape, dtype or algorithm";
    case RLDA_ERR_WORKSPACE: return "workspace missing or too small";
    case RLDA_ERR_STRUCT_SIZE: return "descriptor struct_size does not match this library";
    case RLDA_ERR_LAUNCH: return "HIP runtime error while enqueuing";
    default: return "unknown error code";
  }
}

int rl_decode_attn_plan(const rlda_desc* desc) { return plan(desc); }

size_t rl_decode_attn_workspace_bytes(const rlda_desc* desc) {
  return plan(desc) == RLDA_ALGO_SHARED ? rlda::shared_workspace_bytes(*desc) : 0;
}

int rl_decode_attn(const rlda_desc* desc, void* hip_stream) {
  const int pl = plan(desc);
  if (pl < 0) return pl;
  const rlda_desc& ds = *desc;
  const int64_t B = (int64_t)ds.P * ds.G;
  if (!ds.q || !ds.prefix_lens || !ds.suffix_lens || !ds.out) {
    if (B > 0) return RLDA_ERR_INVALID;
  }
  if (ds.P > 0 && ds.Lp_cap > 0 && (!ds.k_prefix || !ds.v_prefix)) return RLDA_ERR_INVALID;
  if (B > 0 && ds.Ls_cap > 0 && (!ds.k_suffix || !ds.v_suffix)) return RLDA_ERR_INVALID;
  if (B == 0) return RLDA_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (pl == RLDA_ALGO_SHARED) {
    const size_t need = rlda::shared_workspace_bytes(ds);
    if (need > 0 && (!ds.workspace || ds.workspace_bytes < need)) return RLDA_ERR_WORKSPACE;
    if (need > 0 && (reinterpret_cast<uintptr_t>(ds.workspace) & 255u)) return RLDA_ERR_WORKSPACE;
    e = rlda::launch_shared(ds, stream);
  } else {
    e = rlda::launch_simple(ds, stream);
  }
  g_last_hip_error = e;
  return e == hipSuccess ? RLDA_OK : RLDA_ERR_LAUNCH;
}

int rl_lse_combine(const float* o_parts, const float* lse_parts, int32_t n_parts, int64_t n_rows, int32_t d,
                   float* out, float* lse, void* hip_stream) {
  if (n_parts < 0 || n_rows < 0) return RLDA_ERR_INVALID;
  if (d != 64 && d != 128) return RLDA_ERR_UNSUPPORTED;
  if (n_rows == 0) return RLDA_OK;
  if (!out || (n_parts > 0 && (!o_parts || !lse_parts))) return RLDA_ERR_INVALID;
  if (n_rows > (int64_t)1 << 31) return RLDA_ERR_UNSUPPORTED;
  const hipError_t e = rlda::launch_combine(o_parts, lse_parts, n_parts, n_rows, d, out, lse,
                                            static_cast<hipStream_t>(hip_stream));
  g_last_hip_error = e;
  return e == hipSuccess ? RLDA_OK : RLDA_ERR_LAUNCH;
}

}  // extern "C"
