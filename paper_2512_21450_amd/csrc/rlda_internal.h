// Internal launcher interface between the C-ABI layer and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/rl_decode_attn.h"

namespace rlda {

// ---- simple path: one wavefront per (sequence, query head); fp32 or bf16; d in {64,128}
hipError_t launch_simple(const rlda_desc& ds, hipStream_t stream);

// ---- shared-prefix MFMA path (bf16, d = 128)
bool   shared_supported(const rlda_desc& ds);
size_t shared_workspace_bytes(const rlda_desc& ds);
// `mid`, if not null, is recorded between the partial kernel and the combine kernel
hipError_t launch_shared(const rlda_desc& ds, hipStream_t stream, hipEvent_t mid);

// ---- stand-alone log-sum-exp combine over [n_parts, n_rows, d] partials
hipError_t launch_combine(const float* o_parts, const float* lse_parts, int n_parts, int64_t n_rows,
                          int d, float* out, float* lse, hipStream_t stream);

}  // namespace rlda
