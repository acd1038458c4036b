// Internal launcher interface between the C-ABI layer and the gfx950 kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/rl_decode_attn.h"

namespace rlda {

// One decode step in the form the kernels take it: the union of rlda_desc (contiguous suffix
// store) and rlda_paged_desc (page pool + block table, finished-sequence flags).
struct Problem {
  int dtype, algo;
  int P, G, Hq, Hkv, d;
  int Lp_cap;
  int Ls_cap;                     // suffix row capacity per sequence (paged: max_pages * page_size)
  float scale;
  const void* q;
  const void* k_prefix; const void* v_prefix; const int32_t* prefix_lens;
  const void* k_suffix; const void* v_suffix;   // [B, Hkv, Ls_cap, d], or the pools [n_pages, Hkv, page_size, d]
  const int32_t* suffix_lens;
  bool paged;                     // the suffix store is a page pool with a block table (rlda_paged_desc)
  const int32_t* block_table;     // null: contiguous suffix store
  int page_shift;                 // log2(page_size)
  int max_pages, n_pages;
  const uint8_t* seq_active;      // null: every sequence is live
  float* out; float* lse;
  void* workspace; size_t workspace_bytes;
  const float* k_scale; const float* v_scale;   // per-KV-head factors of an e4m3 K/V store, or null
  // tree form (rl_decode_attn_tree): n_levels > 0 levels of shared segments in place of k_prefix / v_prefix /
  // prefix_lens / P / G / Lp_cap; level l has n_seg segments of `cap` rows, each shared by `group` consecutive
  // sequences (n_seg * group == tree_B)
  int n_levels;
  struct Level { const void* k; const void* v; const int32_t* lens; int n_seg, group, cap; } levels[RLDA_MAX_TREE_LEVELS];
  int tree_B;
};

// sequences, entries of the prefix line (prompts, or the segments of all tree levels), largest sharing group
inline int64_t n_sequences(const Problem& p) { return p.n_levels > 0 ? p.tree_B : (int64_t)p.P * p.G; }
inline int64_t n_prefix_entries(const Problem& p) {
  if (p.n_levels == 0) return p.P;
  int64_t n = 0;
  for (int l = 0; l < p.n_levels; ++l) n += p.levels[l].n_seg;
  return n;
}
inline int max_group(const Problem& p) {
  if (p.n_levels == 0) return p.G;
  int g = 1;
  for (int l = 0; l < p.n_levels; ++l) g = p.levels[l].group > g ? p.levels[l].group : g;
  return g;
}

// bytes per stored K/V element
inline int kv_elem_bytes(int dtype) { return dtype == RLDA_F32 ? 4 : (dtype == RLDA_BF16_KV8 ? 1 : 2); }

// ---- simple path: one wavefront per (sequence, query head); fp32, bf16 or bf16 with e4m3 K/V; d in {64,128}
hipError_t launch_simple(const Problem& pb, hipStream_t stream);

// ---- shared-prefix MFMA path (bf16 or bf16 with e4m3 K/V, d = 128)
bool   shared_supported(const Problem& pb);
size_t shared_workspace_bytes(const Problem& pb);
// `mid`, if not null, is recorded between the partial kernel and the combine kernel
hipError_t launch_shared(const Problem& pb, hipStream_t stream, hipEvent_t mid);

// ---- causal prefill attention over each prompt (bf16, d = 128, Hq/Hkv <= 16)
bool prefill_supported(int dtype, int Hq, int Hkv, int d);
hipError_t launch_prefill(const void* q, const void* k, const void* v, const int32_t* lens, float* out, float* lse,
                          int P, int Hq, int Hkv, int Lp_cap, float scale, hipStream_t stream);

// ---- stand-alone log-sum-exp combine over [n_parts, n_rows, d] partials
hipError_t launch_combine(const float* o_parts, const float* lse_parts, int n_parts, int64_t n_rows,
                          int d, float* out, float* lse, hipStream_t stream);

}  // namespace rlda
