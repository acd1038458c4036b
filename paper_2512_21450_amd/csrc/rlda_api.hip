// C-ABI layer: argument validation, kernel-family selection, enqueue.
// Validation and the workspace/plan queries are pure host code and work
// without a GPU; only rl_decode_attn / rl_lse_combine touch the HIP runtime.
#include "rlda_internal.h"
#include "rlda_sched.h"
#include "../../include/rl_prefill_attn.h"

#include <mutex>
#include <vector>

namespace {

using rlda::Problem;

thread_local hipError_t g_last_hip_error = hipSuccess;

// Descriptor -> Problem.  Returns RLDA_OK or the error the descriptor itself shows.
int to_problem(const rlda_desc* ds, Problem& pb) {
  if (!ds) return RLDA_ERR_INVALID;
  if (ds->struct_size != sizeof(rlda_desc)) return RLDA_ERR_STRUCT_SIZE;
  pb = Problem{};
  pb.dtype = ds->dtype; pb.algo = ds->algo;
  pb.P = ds->P; pb.G = ds->G; pb.Hq = ds->Hq; pb.Hkv = ds->Hkv; pb.d = ds->d;
  pb.Lp_cap = ds->Lp_cap; pb.Ls_cap = ds->Ls_cap; pb.scale = ds->scale;
  pb.q = ds->q; pb.k_prefix = ds->k_prefix; pb.v_prefix = ds->v_prefix; pb.prefix_lens = ds->prefix_lens;
  pb.k_suffix = ds->k_suffix; pb.v_suffix = ds->v_suffix; pb.suffix_lens = ds->suffix_lens;
  pb.out = ds->out; pb.lse = ds->lse; pb.workspace = ds->workspace; pb.workspace_bytes = ds->workspace_bytes;
  if (ds->dtype == RLDA_BF16_KV8) { pb.k_scale = ds->k_scale; pb.v_scale = ds->v_scale; }
  return RLDA_OK;
}

int to_problem(const rlda_paged_desc* ds, Problem& pb) {
  if (!ds) return RLDA_ERR_INVALID;
  if (ds->struct_size != sizeof(rlda_paged_desc)) return RLDA_ERR_STRUCT_SIZE;
  if (ds->max_pages < 0 || ds->n_pages < 0 || ds->page_size <= 0) return RLDA_ERR_INVALID;
  if (ds->page_size & (ds->page_size - 1)) return RLDA_ERR_UNSUPPORTED;   // below 32 rows: the simple kernel only
  if ((int64_t)ds->max_pages * ds->page_size > (int64_t)1 << 30) return RLDA_ERR_UNSUPPORTED;
  if (ds->max_pages > 0 && ds->n_pages < 1) return RLDA_ERR_INVALID;
  pb = Problem{};
  pb.dtype = ds->dtype; pb.algo = ds->algo;
  pb.P = ds->P; pb.G = ds->G; pb.Hq = ds->Hq; pb.Hkv = ds->Hkv; pb.d = ds->d;
  pb.Lp_cap = ds->Lp_cap; pb.Ls_cap = ds->max_pages * ds->page_size; pb.scale = ds->scale;
  pb.q = ds->q; pb.k_prefix = ds->k_prefix; pb.v_prefix = ds->v_prefix; pb.prefix_lens = ds->prefix_lens;
  pb.k_suffix = ds->k_pages; pb.v_suffix = ds->v_pages; pb.suffix_lens = ds->suffix_lens;
  pb.paged = true;
  pb.block_table = ds->block_table;
  pb.page_shift = __builtin_ctz((unsigned)ds->page_size);
  pb.max_pages = ds->max_pages; pb.n_pages = ds->n_pages;
  pb.seq_active = ds->seq_active;
  pb.out = ds->out; pb.lse = ds->lse; pb.workspace = ds->workspace; pb.workspace_bytes = ds->workspace_bytes;
  if (ds->dtype == RLDA_BF16_KV8) { pb.k_scale = ds->k_scale; pb.v_scale = ds->v_scale; }
  return RLDA_OK;
}

int check_shape(const Problem& pb) {
  if (pb.P < 0 || pb.G < 0 || pb.Hq <= 0 || pb.Hkv <= 0 || pb.d <= 0 || pb.Lp_cap < 0 || pb.Ls_cap < 0)
    return RLDA_ERR_INVALID;
  if (pb.dtype != RLDA_F32 && pb.dtype != RLDA_BF16 && pb.dtype != RLDA_BF16_KV8) return RLDA_ERR_UNSUPPORTED;
  if (pb.algo != RLDA_ALGO_AUTO && pb.algo != RLDA_ALGO_SIMPLE && pb.algo != RLDA_ALGO_SHARED)
    return RLDA_ERR_UNSUPPORTED;
  if (pb.d != 64 && pb.d != 128) return RLDA_ERR_UNSUPPORTED;
  if (pb.Hq % pb.Hkv != 0) return RLDA_ERR_UNSUPPORTED;
  // index arithmetic in the kernels is 32-bit for (sequence, head) counts
  if ((int64_t)pb.P * pb.G * pb.Hq > (int64_t)1 << 30) return RLDA_ERR_UNSUPPORTED;
  return RLDA_OK;
}

int plan(const Problem& pb) {
  const int rc = check_shape(pb);
  if (rc != RLDA_OK) return rc;
  if (pb.algo == RLDA_ALGO_SIMPLE) return RLDA_ALGO_SIMPLE;
  if (rlda::shared_supported(pb)) return RLDA_ALGO_SHARED;
  return pb.algo == RLDA_ALGO_SHARED ? RLDA_ERR_UNSUPPORTED : RLDA_ALGO_SIMPLE;
}

template <class Desc>
int plan_of(const Desc* desc) {
  Problem pb;
  const int rc = to_problem(desc, pb);
  return rc != RLDA_OK ? rc : plan(pb);
}

template <class Desc>
size_t workspace_of(const Desc* desc) {
  Problem pb;
  if (to_problem(desc, pb) != RLDA_OK) return 0;
  return plan(pb) == RLDA_ALGO_SHARED ? rlda::shared_workspace_bytes(pb) : 0;
}

// Tree descriptor -> Problem.  Returns RLDA_OK or the error the descriptor itself shows.
int to_problem(const rlda_tree_desc* ds, Problem& pb) {
  if (!ds) return RLDA_ERR_INVALID;
  if (ds->struct_size != sizeof(rlda_tree_desc)) return RLDA_ERR_STRUCT_SIZE;
  if (ds->B < 0 || ds->Hq <= 0 || ds->Hkv <= 0 || ds->d <= 0 || ds->Ls_cap < 0) return RLDA_ERR_INVALID;
  if (ds->n_levels < 0 || ds->n_levels > RLDA_MAX_TREE_LEVELS) return RLDA_ERR_INVALID;
  pb = Problem{};
  pb.dtype = ds->dtype; pb.algo = RLDA_ALGO_SHARED;
  pb.P = 0; pb.G = 1; pb.Hq = ds->Hq; pb.Hkv = ds->Hkv; pb.d = ds->d;
  pb.Lp_cap = 0; pb.Ls_cap = ds->Ls_cap; pb.scale = ds->scale;
  pb.q = ds->q; pb.k_suffix = ds->k_suffix; pb.v_suffix = ds->v_suffix; pb.suffix_lens = ds->suffix_lens;
  pb.out = ds->out; pb.lse = ds->lse; pb.workspace = ds->workspace; pb.workspace_bytes = ds->workspace_bytes;
  pb.tree_B = ds->B;
  pb.n_levels = ds->n_levels;
  for (int l = 0; l < ds->n_levels; ++l) {
    const rlda_tree_level& lv = ds->levels[l];
    if (lv.group < 1 || lv.cap < 0 || ds->B % lv.group != 0) return RLDA_ERR_INVALID;
    pb.levels[l] = Problem::Level{lv.k, lv.v, lv.lens, ds->B / lv.group, lv.group, lv.cap};
  }
  return RLDA_OK;
}

// what the tree form runs on, or the reason it cannot
int check_tree(const Problem& pb) {
  if (pb.dtype != RLDA_F32 && pb.dtype != RLDA_BF16 && pb.dtype != RLDA_BF16_KV8) return RLDA_ERR_UNSUPPORTED;
  if (pb.Hq % pb.Hkv != 0) return RLDA_ERR_UNSUPPORTED;
  if ((int64_t)pb.tree_B * pb.Hq > (int64_t)1 << 30) return RLDA_ERR_UNSUPPORTED;
  if (pb.n_levels == 0 || !rlda::shared_supported(pb)) return RLDA_ERR_UNSUPPORTED;   // no level: rl_decode_attn with P = B covers it
  return RLDA_OK;
}

int enqueue_tree(const rlda_tree_desc* desc, void* hip_stream) {
  Problem pb;
  int rc = to_problem(desc, pb);
  if (rc != RLDA_OK) return rc;
  rc = check_tree(pb);
  if (rc != RLDA_OK) return rc;
  if (pb.tree_B == 0) return RLDA_OK;
  if (!pb.q || !pb.suffix_lens || !pb.out) return RLDA_ERR_INVALID;
  if (pb.Ls_cap > 0 && (!pb.k_suffix || !pb.v_suffix)) return RLDA_ERR_INVALID;
  for (int l = 0; l < pb.n_levels; ++l)
    if (!pb.levels[l].lens || (pb.levels[l].cap > 0 && (!pb.levels[l].k || !pb.levels[l].v))) return RLDA_ERR_INVALID;
  const size_t need = rlda::shared_workspace_bytes(pb);
  if (!pb.workspace || pb.workspace_bytes < need) return RLDA_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(pb.workspace) & 255u) return RLDA_ERR_WORKSPACE;
  const hipError_t e = rlda::launch_shared(pb, static_cast<hipStream_t>(hip_stream), nullptr);
  g_last_hip_error = e;
  return e == hipSuccess ? RLDA_OK : RLDA_ERR_LAUNCH;
}

// the tensors a non-empty batch needs
int check_pointers(const Problem& pb) {
  const int64_t B = (int64_t)pb.P * pb.G;
  if (B > 0 && (!pb.q || !pb.prefix_lens || !pb.suffix_lens || !pb.out)) return RLDA_ERR_INVALID;
  if (pb.P > 0 && pb.Lp_cap > 0 && (!pb.k_prefix || !pb.v_prefix)) return RLDA_ERR_INVALID;
  if (B > 0 && pb.Ls_cap > 0 && (!pb.k_suffix || !pb.v_suffix)) return RLDA_ERR_INVALID;
  if (B > 0 && pb.max_pages > 0 && !pb.block_table) return RLDA_ERR_INVALID;
  return RLDA_OK;
}

int enqueue(const Problem& pb, void* hip_stream, void* mid_event) {
  const int pl = plan(pb);
  if (pl < 0) return pl;
  const int rc = check_pointers(pb);
  if (rc != RLDA_OK) return rc;
  if ((int64_t)pb.P * pb.G == 0) return RLDA_OK;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  hipError_t e;
  if (pl == RLDA_ALGO_SHARED) {
    const size_t need = rlda::shared_workspace_bytes(pb);
    if (need > 0 && (!pb.workspace || pb.workspace_bytes < need)) return RLDA_ERR_WORKSPACE;
    if (need > 0 && (reinterpret_cast<uintptr_t>(pb.workspace) & 255u)) return RLDA_ERR_WORKSPACE;
    e = rlda::launch_shared(pb, stream, static_cast<hipEvent_t>(mid_event));
  } else {
    e = rlda::launch_simple(pb, stream);
    if (e == hipSuccess && mid_event) e = hipEventRecord(static_cast<hipEvent_t>(mid_event), stream);
  }
  g_last_hip_error = e;
  return e == hipSuccess ? RLDA_OK : RLDA_ERR_LAUNCH;
}

template <class Desc>
int enqueue_of(const Desc* desc, void* hip_stream, void* mid_event) {
  Problem pb;
  const int rc = to_problem(desc, pb);
  return rc != RLDA_OK ? rc : enqueue(pb, hip_stream, mid_event);
}

// ---- rl_decode_attn_static: the same step for callers that cannot bring (or allocate) a workspace.
// The scan of tile counts and the partial results live in this file-scope device array instead.
// Every GPU the library runs on holds its own copy at its own address until the process ends; the
// array's name is only a host-side stand-in for it, so the address is asked for once per device
// (with that device current) and kept.
__device__ __align__(256) unsigned char g_static_workspace[RLDA_STATIC_WORKSPACE_BYTES];

constexpr int MAX_DEVICES = 64;
std::mutex g_static_mu;
void* g_static_ptr[MAX_DEVICES] = {};

hipError_t static_workspace(void** ptr) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_workspace));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_static_ptr[dev] = p;
  }
  *ptr = g_static_ptr[dev];
  return hipSuccess;
}

int enqueue_static(const rlda_desc* desc, void* hip_stream) {
  Problem pb;
  const int rc = to_problem(desc, pb);
  if (rc != RLDA_OK) return rc;
  pb.workspace = nullptr; pb.workspace_bytes = 0;           // the descriptor's own workspace fields are not used
  const int pl = plan(pb);
  if (pl < 0) return pl;
  if (pl == RLDA_ALGO_SHARED) {
    const size_t need = rlda::shared_workspace_bytes(pb);
    if (need > (size_t)RLDA_STATIC_WORKSPACE_BYTES) return RLDA_ERR_WORKSPACE;
    const int rp = check_pointers(pb);                       // before the device is asked for anything
    if (rp != RLDA_OK) return rp;
    if ((int64_t)pb.P * pb.G > 0) {
      void* p = nullptr;
      const hipError_t e = static_workspace(&p);
      if (e != hipSuccess) { g_last_hip_error = e; return RLDA_ERR_LAUNCH; }
      pb.workspace = p; pb.workspace_bytes = RLDA_STATIC_WORKSPACE_BYTES;
    }
  }
  return enqueue(pb, hip_stream, nullptr);
}

}  // namespace

extern "C" {

const char* rl_decode_attn_last_hip_error(void) { return hipGetErrorString(g_last_hip_error); }

int rl_decode_attn_version(void) { return 300; }

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

int rl_decode_attn_plan(const rlda_desc* desc) { return plan_of(desc); }
size_t rl_decode_attn_workspace_bytes(const rlda_desc* desc) { return workspace_of(desc); }
int rl_decode_attn(const rlda_desc* desc, void* hip_stream) { return enqueue_of(desc, hip_stream, nullptr); }
int rl_decode_attn_profiled(const rlda_desc* desc, void* hip_stream, void* mid_event) {
  return enqueue_of(desc, hip_stream, mid_event);
}

int rl_decode_attn_static(const rlda_desc* desc, void* hip_stream) { return enqueue_static(desc, hip_stream); }
size_t rl_decode_attn_static_workspace_limit(void) { return RLDA_STATIC_WORKSPACE_BYTES; }

int rl_decode_attn_tree(const rlda_tree_desc* desc, void* hip_stream) { return enqueue_tree(desc, hip_stream); }
size_t rl_decode_attn_tree_workspace_bytes(const rlda_tree_desc* desc) {
  Problem pb;
  if (to_problem(desc, pb) != RLDA_OK || check_tree(pb) != RLDA_OK) return 0;
  return rlda::shared_workspace_bytes(pb);
}

int rl_decode_attn_paged_plan(const rlda_paged_desc* desc) { return plan_of(desc); }
size_t rl_decode_attn_paged_workspace_bytes(const rlda_paged_desc* desc) { return workspace_of(desc); }
int rl_decode_attn_paged(const rlda_paged_desc* desc, void* hip_stream, void* mid_event) {
  return enqueue_of(desc, hip_stream, mid_event);
}

}  // extern "C"

extern "C" {

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

int32_t rl_decode_attn_debug_pairs(int32_t compute_units) {
  return compute_units < 1 ? RLDA_ERR_INVALID : rlda::pairs_for(compute_units);
}

int64_t rl_decode_attn_debug_partition(int32_t P, int32_t G, int32_t Hkv, int32_t rows_per_kv_group,
                                       int32_t Lp_cap, int32_t Ls_cap, const int32_t* prefix_lens, const int32_t* suffix_lens,
                                       int32_t* runs, int64_t runs_cap, int32_t* parts, int64_t parts_cap,
                                       int64_t* n_parts) {
  return rl_decode_attn_debug_partition_on(256, P, G, Hkv, rows_per_kv_group, Lp_cap, Ls_cap, prefix_lens, suffix_lens,
                                           runs, runs_cap, parts, parts_cap, n_parts);
}

int64_t rl_decode_attn_debug_partition_on(int32_t compute_units, int32_t P, int32_t G, int32_t Hkv, int32_t rows_per_kv_group,
                                          int32_t Lp_cap, int32_t Ls_cap, const int32_t* prefix_lens, const int32_t* suffix_lens,
                                          int32_t* runs, int64_t runs_cap, int32_t* parts, int64_t parts_cap,
                                          int64_t* n_parts) {
  using namespace rlda;
  if (P < 0 || G < 0 || Hkv <= 0 || rows_per_kv_group <= 0 || !prefix_lens || !suffix_lens || !n_parts || compute_units < 1)
    return RLDA_ERR_INVALID;
  const int n_cu = pairs_for(compute_units);
  const int B = P * G;
  if (rows_per_kv_group > MAX_GROUP_ROWS) return RLDA_ERR_INVALID;
  // prefix units per prompt on the line, (KV head, line part); with SM = 2 twin pairs walk it, for row halves
  // 2 * part + side.  Runs and parts are reported with j = head * row_parts + half.
  const int NHl = line_parts(rows_per_kv_group, n_cu), SM = side_parts(rows_per_kv_group, n_cu);
  const int HkvP = Hkv * NHl;
  auto unit_j = [&](int jl, int side) { return (jl / NHl) * NHl * SM + (jl % NHl) * SM + side; };
  std::vector<int> X(P + B + 2, 0);
  auto tp = [&](int p) { return ceil_div(clampi(prefix_lens[p], 0, Lp_cap), TK); };
  auto ts = [&](int b) { return ceil_div(clampi(suffix_lens[b], 0, Ls_cap), TK); };
  for (int i = 0; i < P; ++i) X[i + 1] = X[i] + tp(i);
  for (int i = 0; i < B; ++i) X[P + i + 1] = X[P + i] + ts(i);
  const int cumP = X[P];
  const Sched sc = make_sched(cumP * HkvP, (X[P + B] - cumP) * Hkv, n_cu, SM == 2);
  int64_t nr = 0, np = 0;
  auto put_run = [&](int kind, int major, int j, int t0, int n, int w, int v, int slot) {
    if (runs && nr < runs_cap) {
      int32_t* o = runs + nr * 8;
      o[0] = kind; o[1] = major; o[2] = j; o[3] = t0; o[4] = n; o[5] = w; o[6] = v; o[7] = slot;
    }
    ++nr;
  };
  for (int x = 0; x < 2 * n_cu; ++x) {           // the partial kernel's walk; runs are reported by grid index
    const int w = wg_name(sc, x);
    int ilo, ihi, klo, khi;
    wg_prefix_range(sc, w, ilo, ihi);
    wg_suffix_range(sc, w, klo, khi);
    if (ilo < ihi) {
      int p, j, t;
      locate(X.data(), P, HkvP, ilo, p, j, t);
      for_each_run(ilo, ihi, P, HkvP, p, j, t, tp,
                   [&](int pp, int jj, int t0, int n) {
                     const int side = prefix_side(sc, wg_pair(sc, w));
                     put_run(0, pp, unit_j(jj, side), t0, n, x, -1, (pp * HkvP + jj + wg_prefix_rank(sc, w)) * SM + side);
                   });
    }
    for (int v = 0; v < WG_WAVES; ++v) {
      int ka, kb;
      wave_suffix_range(klo, khi, v, ka, kb);
      if (ka >= kb) continue;
      int b, j, t;
      locate(X.data() + P, B, Hkv, ka + cumP * Hkv, b, j, t);
      for_each_run(ka, kb, B, Hkv, b, j, t, ts, [&](int bb, int jj, int t0, int n) {
        put_run(1, bb, jj, t0, n, x, v, bb * Hkv + jj + WG_WAVES * wg_rank(sc, w) + v);
      });
    }
  }
  auto put_part = [&](int kind, int major, int j, int w, int v, int slot) {
    if (parts && np < parts_cap) {
      int32_t* o = parts + np * 6;
      o[0] = kind; o[1] = major; o[2] = j; o[3] = w; o[4] = v; o[5] = slot;
    }
    ++np;
  };
  for (int p = 0; p < P; ++p)                    // the combine kernel's enumeration
    for (int j = 0; j < HkvP; ++j)
      for (int side = 0; side < SM; ++side)
        for_each_prefix_part(sc, X.data(), HkvP, p, j, side, [&](int rank) {
          const int c = share_pair(sc, rank / 2, side);
          put_part(0, p, unit_j(j, side), wg_grid_index(sc, c, rank % 2), -1, (p * HkvP + j + rank) * SM + side);
        });
  for (int b = 0; b < B; ++b)
    for (int j = 0; j < Hkv; ++j)
      for_each_suffix_part(sc, X.data() + P, cumP, Hkv, b, j, [&](int rank, int v) {
        put_part(1, b, j, wg_grid_index(sc, rank / 2, rank % 2), v, b * Hkv + j + WG_WAVES * rank + v);
      });
  *n_parts = np;
  return nr;
}

}  // extern "C"

extern "C" int rl_prefill_attn(const rl_prefill_desc* d, void* hip_stream) {
  if (!d) return RLDA_ERR_INVALID;
  if (d->struct_size != sizeof(rl_prefill_desc)) return RLDA_ERR_STRUCT_SIZE;
  if (d->P < 0 || d->Hq <= 0 || d->Hkv <= 0 || d->d <= 0 || d->Lp_cap < 0) return RLDA_ERR_INVALID;
  if (!rlda::prefill_supported(d->dtype, d->Hq, d->Hkv, d->d)) return RLDA_ERR_UNSUPPORTED;
  const int qb = 64 / (d->Hq / d->Hkv);                     // a lower bound of the positions per workgroup
  if ((int64_t)((d->Lp_cap + qb - 1) / qb) * ((int64_t)d->P * d->Hkv + 7) > 0x7fffffffLL) return RLDA_ERR_UNSUPPORTED;
  if ((int64_t)d->Lp_cap * d->Hq * 256 >= (int64_t)1 << 40) return RLDA_ERR_UNSUPPORTED;
  if (d->Lp_cap >= 1 << 24) return RLDA_ERR_UNSUPPORTED;    // byte offsets inside one (prompt, KV head) store are 32-bit
  if (d->P == 0 || d->Lp_cap == 0) return RLDA_OK;
  if (!d->q || !d->k || !d->v || !d->lens || !d->out) return RLDA_ERR_INVALID;
  const hipError_t e = rlda::launch_prefill(d->q, d->k, d->v, d->lens, d->out, d->lse, d->P, d->Hq, d->Hkv, d->Lp_cap,
                                            d->scale, static_cast<hipStream_t>(hip_stream));
  g_last_hip_error = e;
  return e == hipSuccess ? RLDA_OK : RLDA_ERR_LAUNCH;
}

