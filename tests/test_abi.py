"""The C-ABI library without a GPU: it loads, exports what the header
declares, and every host-side validation path returns its documented code
without launching anything."""
import ctypes
import os
import re

import pytest

from paper_2512_21450_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if not f.endswith(".h"):
            continue
        src = open(os.path.join(inc, f)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names += re.findall(r"\b(rl_[a-z0-9_]+)\s*\(", src)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"rl_decode_attn", "rl_decode_attn_workspace_bytes", "rl_decode_attn_plan",
            "rl_decode_attn_strerror", "rl_decode_attn_version", "rl_lse_combine"} <= set(names)
    lib = ctypes.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/ but not exported"


def test_version_and_strerror():
    assert B.rl_decode_attn_version() >= 100
    for code in (0, -1, -2, -3, -4, -5):
        assert B.rl_decode_attn_strerror(code) not in ("", "unknown error code")
    assert B.rl_decode_attn_strerror(-99) == "unknown error code"


def good(**kw):
    args = dict(dtype=B.RLDA_BF16, P=2, G=4, Hq=8, Hkv=2, d=128, Lp_cap=64, Ls_cap=64, scale=0.1)
    args.update(kw)
    return B.make_desc(**args)


def test_descriptor_layout_matches_the_header():
    # 11 four-byte fields, padding to 8, 9 pointers, pointer + size_t, the two scale pointers
    assert ctypes.sizeof(B.rlda_desc) == 48 + 9 * 8 + 16 + 16
    assert B.rlda_desc.q.offset == 48 and B.rlda_desc.workspace_bytes.offset == 48 + 10 * 8
    assert B.rlda_desc.k_scale.offset == 48 + 11 * 8 and B.rlda_desc.v_scale.offset == 48 + 12 * 8


def test_e4m3_store_dtype_is_planned_like_bf16():
    from paper_2512_21450_amd import workloads as wl
    W = wl.WORKLOADS["vlm7b"]
    ds = B.make_desc(B.RLDA_BF16_KV8, W.P, W.G, W.Hq, W.Hkv, W.d, W.Lp_cap, W.Ls_cap, W.scale)
    ref = B.make_desc(B.RLDA_BF16, W.P, W.G, W.Hq, W.Hkv, W.d, W.Lp_cap, W.Ls_cap, W.scale)
    assert B.rl_decode_attn_plan(ds) == B.RLDA_ALGO_SHARED
    assert B.rl_decode_attn_workspace_bytes(ds) == B.rl_decode_attn_workspace_bytes(ref)   # partials do not depend on the store
    assert B.rl_decode_attn_plan(good(dtype=B.RLDA_BF16_KV8, d=64)) == B.RLDA_ALGO_SIMPLE
    assert B.rl_decode_attn_plan(good(dtype=3)) == B.RLDA_ERR_UNSUPPORTED


def test_only_positive_scales_are_planned_onto_the_shared_path():
    assert B.rl_decode_attn_plan(good()) == B.RLDA_ALGO_SHARED
    for sc in (0.0, -0.1, float("nan")):
        assert B.rl_decode_attn_plan(good(scale=sc)) == B.RLDA_ALGO_SIMPLE
        assert B.rl_decode_attn_plan(good(scale=sc, algo=B.RLDA_ALGO_SHARED)) == B.RLDA_ERR_UNSUPPORTED
        assert B.rl_decode_attn_workspace_bytes(good(scale=sc)) == 0


@pytest.mark.parametrize("kw,code", [
    (dict(d=96), B.RLDA_ERR_UNSUPPORTED),
    (dict(d=256), B.RLDA_ERR_UNSUPPORTED),
    (dict(Hq=7, Hkv=2), B.RLDA_ERR_UNSUPPORTED),
    (dict(dtype=5), B.RLDA_ERR_UNSUPPORTED),
    (dict(algo=9), B.RLDA_ERR_UNSUPPORTED),
    (dict(P=-1), B.RLDA_ERR_INVALID),
    (dict(Lp_cap=-3), B.RLDA_ERR_INVALID),
    (dict(Hkv=0), B.RLDA_ERR_INVALID),
    (dict(dtype=B.RLDA_F32, algo=B.RLDA_ALGO_SHARED), B.RLDA_ERR_UNSUPPORTED),
])
def test_shape_errors(kw, code):
    ds = good(**kw)
    assert B.rl_decode_attn_plan(ds) == code
    assert B.rl_decode_attn_raw(ds) == code
    assert B.rl_decode_attn_workspace_bytes(ds) == 0


def test_struct_size_mismatch_and_null_descriptor():
    ds = good()
    ds.struct_size = 8
    assert B.rl_decode_attn_raw(ds) == B.RLDA_ERR_STRUCT_SIZE
    assert B._lib.rl_decode_attn(None, None) == B.RLDA_ERR_INVALID
    assert B._lib.rl_decode_attn_workspace_bytes(None) == 0


def test_null_pointers_are_rejected_before_any_launch():
    fake = 0x1000  # never dereferenced on the host; the call must fail before enqueuing
    full = dict(q=fake, k_prefix=fake, v_prefix=fake, prefix_lens=fake, k_suffix=fake, v_suffix=fake,
                suffix_lens=fake, out=fake)
    for missing in full:
        ptrs = {k: v for k, v in full.items() if k != missing}
        ds = good(algo=B.RLDA_ALGO_SIMPLE, **ptrs)
        assert B.rl_decode_attn_raw(ds) == B.RLDA_ERR_INVALID, missing


def test_plan_and_workspace_query():
    assert B.rl_decode_attn_plan(good(algo=B.RLDA_ALGO_SIMPLE)) == B.RLDA_ALGO_SIMPLE
    assert B.rl_decode_attn_workspace_bytes(good(algo=B.RLDA_ALGO_SIMPLE)) == 0
    assert B.rl_decode_attn_plan(good(dtype=B.RLDA_F32, d=64)) == B.RLDA_ALGO_SIMPLE
    # empty batch is a successful no-op that touches no device
    assert B.rl_decode_attn_raw(good(P=0)) == B.RLDA_OK


def test_lse_combine_argument_checks():
    f = B._lib.rl_lse_combine
    assert f(None, None, 2, 4, 96, None, None, None) == B.RLDA_ERR_UNSUPPORTED
    assert f(None, None, -1, 4, 128, None, None, None) == B.RLDA_ERR_INVALID
    assert f(None, None, 2, 4, 128, 0x1000, None, None) == B.RLDA_ERR_INVALID
    assert f(None, None, 2, 0, 128, None, None, None) == B.RLDA_OK


def test_auto_selects_the_shared_prefix_path_for_bf16_d128():
    for w in ("vlm3b", "vlm7b", "agentic", "highbatch"):
        from paper_2512_21450_amd import workloads as wl
        W = wl.WORKLOADS[w]
        ds = B.make_desc(B.RLDA_BF16, W.P, W.G, W.Hq, W.Hkv, W.d, W.Lp_cap, W.Ls_cap, W.scale)
        assert B.rl_decode_attn_plan(ds) == B.RLDA_ALGO_SHARED
        assert B.rl_decode_attn_workspace_bytes(ds) > 0
    # shapes outside the MFMA path fall back to the simple kernel under AUTO
    assert B.rl_decode_attn_plan(good(d=64)) == B.RLDA_ALGO_SIMPLE
    assert B.rl_decode_attn_plan(good(Hq=64, Hkv=2)) == B.RLDA_ALGO_SIMPLE          # 32 heads per KV head
    assert B.rl_decode_attn_plan(good(Hq=64, Hkv=2, algo=B.RLDA_ALGO_SHARED)) == B.RLDA_ERR_UNSUPPORTED


# ---------------------------------------------------------------- paged descriptor
def good_paged(**kw):
    args = dict(dtype=B.RLDA_BF16, P=2, G=4, Hq=8, Hkv=2, d=128, Lp_cap=64, page_size=64, max_pages=4,
                n_pages=40, scale=0.1)
    args.update(kw)
    return B.make_paged_desc(**args)


def test_paged_descriptor_layout_matches_the_header():
    # 13 four-byte fields, padding to 8, 11 pointers, pointer + size_t, the two scale pointers
    assert ctypes.sizeof(B.rlda_paged_desc) == 56 + 11 * 8 + 16 + 16
    assert B.rlda_paged_desc.q.offset == 56 and B.rlda_paged_desc.workspace_bytes.offset == 56 + 12 * 8
    assert B.rlda_paged_desc.k_scale.offset == 56 + 13 * 8 and B.rlda_paged_desc.v_scale.offset == 56 + 14 * 8


@pytest.mark.parametrize("kw,code", [
    (dict(page_size=48), B.RLDA_ERR_UNSUPPORTED),       # not a power of two
    (dict(page_size=0), B.RLDA_ERR_INVALID),
    (dict(max_pages=-1), B.RLDA_ERR_INVALID),
    (dict(n_pages=0), B.RLDA_ERR_INVALID),              # a table with columns needs a pool
    (dict(max_pages=1 << 26, page_size=64), B.RLDA_ERR_UNSUPPORTED),
    (dict(d=96), B.RLDA_ERR_UNSUPPORTED),
    (dict(Hq=7), B.RLDA_ERR_UNSUPPORTED),
])
def test_paged_shape_errors(kw, code):
    ds = good_paged(**kw)
    assert B.rl_decode_attn_paged_plan(ds) == code
    assert B.rl_decode_attn_paged_raw(ds) == code
    assert B.rl_decode_attn_paged_workspace_bytes(ds) == 0


def test_small_pages_plan_onto_the_simple_kernel():
    # a page shorter than a 32-key tile: the shared-prefix path cannot take it, the simple kernel resolves pages key by key
    for ps in (1, 8, 16):
        assert B.rl_decode_attn_paged_plan(good_paged(page_size=ps)) == B.RLDA_ALGO_SIMPLE
        assert B.rl_decode_attn_paged_workspace_bytes(good_paged(page_size=ps)) == 0
        assert B.rl_decode_attn_paged_plan(good_paged(page_size=ps, algo=B.RLDA_ALGO_SHARED)) == B.RLDA_ERR_UNSUPPORTED
    assert B.rl_decode_attn_paged_plan(good_paged(page_size=32)) == B.RLDA_ALGO_SHARED


def test_paged_plan_workspace_and_pointer_checks():
    ds = good_paged()
    assert B.rl_decode_attn_paged_plan(ds) == B.RLDA_ALGO_SHARED
    # same partial layout as the contiguous call of the same shape
    assert B.rl_decode_attn_paged_workspace_bytes(ds) == B.rl_decode_attn_workspace_bytes(good(Ls_cap=256))
    assert B.rl_decode_attn_paged_plan(good_paged(dtype=B.RLDA_F32)) == B.RLDA_ALGO_SIMPLE
    assert B.rl_decode_attn_paged_raw(ds) == B.RLDA_ERR_INVALID                 # null tensors
    ds.struct_size = 12
    assert B.rl_decode_attn_paged_raw(ds) == B.RLDA_ERR_STRUCT_SIZE
    assert B._lib.rl_decode_attn_paged(None, None, None) == B.RLDA_ERR_INVALID
    fake = 0x1000
    ds = good_paged(q=fake, k_prefix=fake, v_prefix=fake, prefix_lens=fake, k_pages=fake, v_pages=fake,
                    suffix_lens=fake, out=fake)
    assert B.rl_decode_attn_paged_raw(ds) == B.RLDA_ERR_INVALID                 # block table missing
    ds.block_table = fake
    assert B.rl_decode_attn_paged_raw(ds) == B.RLDA_ERR_WORKSPACE               # every pointer set, no workspace
    assert B.rl_decode_attn_paged_raw(good_paged(P=0)) == B.RLDA_OK             # empty batch: nothing to enqueue


# ---------------------------------------------------------------- rl_token_logprob
def good_tl(**kw):
    args = dict(dtype=B.RLDA_BF16, n_rows=8, vocab=1000, row_stride=1000)
    args.update(kw)
    return B.make_token_logprob_desc(**args)


def test_token_logprob_descriptor_layout():
    assert ctypes.sizeof(B.rl_token_logprob_desc) == 32 + 9 * 8 + 8
    assert B.rl_token_logprob_desc.logits.offset == 32


@pytest.mark.parametrize("kw,code", [
    (dict(dtype=3), -2), (dict(row_stride=1004), -2), (dict(row_stride=992), -2), (dict(vocab=0), -1),
    (dict(n_rows=-1), -1), (dict(dtype=B.RLDA_F32, row_stride=1002), -2), (dict(n_rows=1 << 40), -2),
])
def test_token_logprob_shape_errors(kw, code):
    ds = good_tl(**kw)
    assert B.rl_token_logprob_raw(ds) == code
    assert B.rl_token_logprob_workspace_bytes(ds) == 0


def test_token_logprob_temperature_must_be_positive_and_finite():
    for t in (0.0, -1.0, float("nan"), float("inf")):
        ds = good_tl()
        ds.inv_temperature = t
        assert B.rl_token_logprob_raw(ds) == -1
        assert B.rl_token_logprob_workspace_bytes(ds) == 0


def test_token_logprob_pointer_and_workspace_checks():
    assert B.rl_token_logprob_raw(good_tl(n_rows=0)) == 0
    assert B.rl_token_logprob_raw(good_tl()) == -1                           # logits missing
    fake = 0x1000
    assert B.rl_token_logprob_raw(good_tl(logits=fake, token_ids=fake, kl=fake)) == -1   # kl without reference
    assert B.rl_token_logprob_raw(good_tl(logits=fake + 4, token_ids=fake)) == -2        # misaligned rows
    big = good_tl(vocab=152000, row_stride=152000, logits=fake, token_ids=fake)
    assert B.rl_token_logprob_workspace_bytes(big) == 8 * 18 * 6 * 4                     # 18 splits of >= 8192 logits each
    assert B.rl_token_logprob_workspace_bytes(good_tl(n_rows=200, vocab=152000, row_stride=152000)) == 0   # unsplit
    assert B.rl_token_logprob_raw(big) == -3
    ds = good_tl(); ds.struct_size = 4
    assert B.rl_token_logprob_raw(ds) == -4
    assert B._lib.rl_token_logprob(None, None) == -1


# ---------------------------------------------------------------- rl_kv_append_rope
def good_ka(**kw):
    args = dict(dtype=B.RLDA_BF16, B=4, Hq=8, Hkv=2, d=128, sections=(16, 24, 24), Ls_cap=64)
    args.update(kw)
    return B.make_kv_append_desc(**args)


def test_kv_append_descriptor_layout_and_errors():
    assert ctypes.sizeof(B.rl_kv_append_desc) == 56 + 12 * 8          # 10 tensor pointers, the two factor arrays
    assert B.rl_kv_append_desc.q.offset == 56 and B.rl_kv_append_desc.k_scale.offset == 56 + 10 * 8
    fake = 0x1000
    ptrs = dict(q=fake, k_new=fake, v_new=fake, positions=fake, inv_freq=fake, k_store=fake, v_store=fake, suffix_lens=fake)
    for kw, code in [(dict(d=96), -2), (dict(sections=(16, 24, 23)), -2), (dict(sections=(-1, 41, 24)), -2),
                     (dict(dtype=7), -2), (dict(Hkv=0), -1), (dict(B=-1), -1), (dict(Ls_cap=-1), -1),
                     (dict(block_table=fake, page_size=48, max_pages=2, n_pages=4), -2),
                     (dict(block_table=fake, page_size=64, max_pages=2, n_pages=0), -1)]:
        assert B.rl_kv_append_rope_raw(good_ka(**ptrs, **kw)) == code, kw
    assert B.rl_kv_append_rope_raw(good_ka()) == -1                  # null tensors
    assert B.rl_kv_append_rope_raw(good_ka(B=0)) == 0
    ds = good_ka(**ptrs); ds.struct_size = 16
    assert B.rl_kv_append_rope_raw(ds) == -4
    assert B._lib.rl_kv_append_rope(None, None) == -1


# ---------------------------------------------------------------- rl_policy_loss.h
def good_pl(**kw):
    args = dict(B=4, T=16, row_stride=16, clip_low=0.2, clip_high=0.2)
    args.update(kw)
    return B.make_policy_loss_desc(**args)


def test_policy_loss_descriptor_layout_and_errors():
    assert ctypes.sizeof(B.rl_policy_loss_desc) == 48 + 8 * 8 + 16 and B.rl_policy_loss_desc.logprob.offset == 48
    assert ctypes.sizeof(B.rl_group_advantage_desc) == 32 + 4 * 8 and B.rl_group_advantage_desc.metrics.offset == 32
    fake = 0x1000
    full = dict(logprob=fake, old_logprob=fake, advantages=fake, lens=fake, stats=fake, workspace=0x1000, workspace_bytes=1 << 20)
    for kw, code in [(dict(form=3), -2), (dict(agg=2), -2), (dict(row_stride=8), -2), (dict(B=-1), -1), (dict(T=-2), -1),
                     (dict(clip_low=-0.1), -1), (dict(clip_high=float("nan")), -1)]:
        ds = good_pl(**full, **kw)
        assert B.rl_policy_loss_raw(ds) == code, kw
        assert B.rl_policy_loss_workspace_bytes(ds) == 0
    for missing in ("logprob", "old_logprob", "advantages", "lens", "stats"):
        assert B.rl_policy_loss_raw(good_pl(**{k: v for k, v in full.items() if k != missing})) == -1, missing
    assert B.rl_policy_loss_workspace_bytes(good_pl()) == 256 + 4 * 32
    assert B.rl_policy_loss_raw(good_pl(**{**full, "workspace_bytes": 64})) == -3
    assert B.rl_policy_loss_raw(good_pl(**{**full, "workspace": 0x1010})) == -3          # not 256-byte aligned
    ds = good_pl(**full); ds.struct_size = 12
    assert B.rl_policy_loss_raw(ds) == -4
    assert B._lib.rl_policy_loss(None, None) == -1 and B._lib.rl_policy_loss_workspace_bytes(None) == 0


def test_group_advantage_argument_checks():
    fake = 0x1000
    ok = dict(metrics=fake, weights=fake, advantages=fake)
    for kw, code in [(dict(mode=5), -2), (dict(G=1025), -2), (dict(n_metrics=0), -2), (dict(n_metrics=65), -2),
                     (dict(P=-1), -1), (dict(eps=-1.0), -1)]:
        args = dict(P=2, G=4, n_metrics=1); args.update(kw)
        assert B.rl_group_advantage_raw(B.make_group_advantage_desc(**args, **ok)) == code, kw
    assert B.rl_group_advantage_raw(B.make_group_advantage_desc(2, 4, 1)) == -1              # null tensors
    assert B.rl_group_advantage_raw(B.make_group_advantage_desc(0, 4, 1)) == 0               # empty batch
    ds = B.make_group_advantage_desc(2, 4, 1, **ok); ds.struct_size = 8
    assert B.rl_group_advantage_raw(ds) == -4
    assert B._lib.rl_group_advantage(None, None) == -1


# ---------------------------------------------------------------- rl_prefill_attn.h
def test_prefill_descriptor_layout_and_errors():
    assert ctypes.sizeof(B.rl_prefill_desc) == 32 + 6 * 8 and B.rl_prefill_desc.q.offset == 32
    fake = 0x1000
    ptrs = dict(q=fake, k=fake, v=fake, lens=fake, out=fake)
    mk = lambda **kw: B.make_prefill_desc(**{**dict(dtype=B.RLDA_BF16, P=2, Hq=28, Hkv=4, d=128, Lp_cap=100, scale=0.1), **kw})
    for kw, code in [(dict(dtype=B.RLDA_F32), -2), (dict(d=64), -2), (dict(Hq=64, Hkv=2), -2), (dict(Hq=7, Hkv=2), -2),
                     (dict(P=-1), -1), (dict(Lp_cap=-1), -1), (dict(Hkv=0), -1)]:
        assert B.rl_prefill_attn_raw(mk(**ptrs, **kw)) == code, kw
    for missing in ptrs:
        assert B.rl_prefill_attn_raw(mk(**{k: v for k, v in ptrs.items() if k != missing})) == -1, missing
    assert B.rl_prefill_attn_raw(mk(P=0)) == 0 and B.rl_prefill_attn_raw(mk(Lp_cap=0)) == 0   # nothing to do
    ds = mk(**ptrs); ds.struct_size = 4
    assert B.rl_prefill_attn_raw(ds) == -4
    assert B._lib.rl_prefill_attn(None, None) == -1


def test_static_entry_point_validates_on_the_host_and_knows_its_limit():
    lim = B.rl_decode_attn_static_workspace_limit()
    assert lim == 64 << 20
    # a problem whose partial results do not fit the library's own array: refused before anything is enqueued
    huge = good(P=900, G=16, Hq=32, Hkv=2, Lp_cap=64, Ls_cap=64)
    assert B.rl_decode_attn_plan(huge) == B.RLDA_ALGO_SHARED
    assert B.rl_decode_attn_workspace_bytes(huge) > lim
    assert B.rl_decode_attn_static_raw(huge) == B.RLDA_ERR_WORKSPACE
    assert B.rl_decode_attn_static_raw(good(d=96)) == B.RLDA_ERR_UNSUPPORTED
    bad = good()
    bad.struct_size = 8
    assert B.rl_decode_attn_static_raw(bad) == B.RLDA_ERR_STRUCT_SIZE
    assert B.rl_decode_attn_static_raw(good()) == B.RLDA_ERR_INVALID     # fits, but q / lengths / out are NULL
    assert B.rl_decode_attn_static_raw(good(P=0)) == B.RLDA_OK           # empty batch: nothing to do


def test_tree_descriptor_layout_and_host_side_validation():
    # 9 four-byte fields, padding to 8, four levels of 3 pointers + 2 ints, 6 pointers, pointer + size_t
    assert ctypes.sizeof(B.rlda_tree_level) == 32
    assert ctypes.sizeof(B.rlda_tree_desc) == 40 + 4 * 32 + 6 * 8 + 16
    lv = lambda g, cap: (None, None, None, g, cap)
    ok = B.make_tree_desc(B.RLDA_BF16, 64, 28, 4, 128, 512, 0.088, [lv(8, 300), lv(4, 100)])
    assert B.rl_decode_attn_tree_workspace_bytes(ok) > 0
    assert B.rl_decode_attn_tree_raw(ok) == B.RLDA_ERR_INVALID                  # supported, but every pointer is NULL
    # a group that does not divide the batch, a negative capacity, too many levels
    assert B.rl_decode_attn_tree_raw(B.make_tree_desc(B.RLDA_BF16, 64, 28, 4, 128, 512, 0.088, [lv(5, 300)])) == B.RLDA_ERR_INVALID
    assert B.rl_decode_attn_tree_raw(B.make_tree_desc(B.RLDA_BF16, 64, 28, 4, 128, 512, 0.088, [lv(8, -1)])) == B.RLDA_ERR_INVALID
    bad = B.make_tree_desc(B.RLDA_BF16, 64, 28, 4, 128, 512, 0.088, [lv(8, 300)])
    bad.n_levels = 5
    assert B.rl_decode_attn_tree_raw(bad) == B.RLDA_ERR_INVALID
    bad = B.make_tree_desc(B.RLDA_BF16, 64, 28, 4, 128, 512, 0.088, [lv(8, 300)])
    bad.struct_size = 16
    assert B.rl_decode_attn_tree_raw(bad) == B.RLDA_ERR_STRUCT_SIZE
    # outside what the tree form runs on: more than 64 query rows per segment and KV head, fp32, d = 64, scale <= 0, no level
    for d_ in (B.make_tree_desc(B.RLDA_BF16, 64, 28, 4, 128, 512, 0.088, [lv(16, 300)]),
               B.make_tree_desc(B.RLDA_F32, 64, 28, 4, 128, 512, 0.088, [lv(8, 300)]),
               B.make_tree_desc(B.RLDA_BF16, 64, 28, 4, 64, 512, 0.088, [lv(8, 300)]),
               B.make_tree_desc(B.RLDA_BF16, 64, 28, 4, 128, 512, -1.0, [lv(8, 300)]),
               B.make_tree_desc(B.RLDA_BF16, 64, 28, 4, 128, 512, 0.088, [])):
        assert B.rl_decode_attn_tree_raw(d_) == B.RLDA_ERR_UNSUPPORTED
        assert B.rl_decode_attn_tree_workspace_bytes(d_) == 0
    assert B.rl_decode_attn_tree_raw(B.make_tree_desc(B.RLDA_BF16, 0, 28, 4, 128, 512, 0.088, [lv(8, 300)])) == B.RLDA_OK


def _cpu_case(**over):
    import torch
    P, G, Hq, Hkv, d, Lp, Ls = 2, 3, 4, 2, 128, 40, 24
    t = dict(q=torch.zeros(P * G, Hq, d, dtype=torch.bfloat16),
             k_prefix=torch.zeros(P, Hkv, Lp, d, dtype=torch.bfloat16), v_prefix=torch.zeros(P, Hkv, Lp, d, dtype=torch.bfloat16),
             prefix_lens=torch.zeros(P, dtype=torch.int32),
             k_suffix=torch.zeros(P * G, Hkv, Ls, d, dtype=torch.bfloat16), v_suffix=torch.zeros(P * G, Hkv, Ls, d, dtype=torch.bfloat16),
             suffix_lens=torch.zeros(P * G, dtype=torch.int32),
             out=torch.zeros(P * G, Hq, d), lse=torch.zeros(P * G, Hq))
    t.update(over)
    return t, G


def _desc(t, G):
    return B.desc_from_tensors(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], t["k_suffix"], t["v_suffix"],
                               t["suffix_lens"], 0.1, G, t["out"], t["lse"])


def test_descriptor_helper_rejects_what_the_kernels_would_misread():
    import torch
    t, G = _cpu_case()
    assert _desc(t, G).P == 2                                   # the well-formed case goes through
    for over, exc in [
        (dict(suffix_lens=torch.zeros(6, dtype=torch.int64)), TypeError),      # torch's default integer: read as pairs of int32
        (dict(prefix_lens=torch.zeros(2, dtype=torch.int64)), TypeError),
        (dict(suffix_lens=torch.zeros(5, dtype=torch.int32)), ValueError),     # one length per sequence
        (dict(prefix_lens=torch.zeros(3, dtype=torch.int32)), ValueError),
        (dict(out=torch.zeros(6, 4, 128, dtype=torch.bfloat16)), TypeError),   # out is written as fp32
        (dict(out=torch.zeros(6, 4, 64)), ValueError),                         # too small: would be overrun
        (dict(lse=torch.zeros(6, 4, dtype=torch.float64)), TypeError),
        (dict(lse=torch.zeros(6, 3)), ValueError),
        (dict(v_prefix=torch.zeros(2, 2, 39, 128, dtype=torch.bfloat16)), ValueError),
        (dict(v_suffix=torch.zeros(6, 2, 25, 128, dtype=torch.bfloat16)), ValueError),
        (dict(out=torch.zeros(6, 4, 256)[:, :, ::2]), ValueError),             # not contiguous
    ]:
        t, G = _cpu_case(**over)
        with pytest.raises(exc):
            _desc(t, G)


def test_tree_descriptor_helper_rejects_misshaped_levels():
    import torch
    t, G = _cpu_case()
    lv = lambda n, g, dt=torch.int32: (torch.zeros(n, 2, 16, 128, dtype=torch.bfloat16), torch.zeros(n, 2, 16, 128, dtype=torch.bfloat16),
                                       torch.zeros(n, dtype=dt), g)
    mk = lambda levels: B.tree_desc_from_tensors(t["q"], levels, t["k_suffix"], t["v_suffix"], t["suffix_lens"], 0.1, t["out"], t["lse"])
    assert mk([lv(2, 3), lv(3, 2)]).n_levels == 2
    with pytest.raises(ValueError):
        mk([lv(2, 2)])                                          # 2 segments x 2 sequences do not cover 6
    with pytest.raises(TypeError):
        mk([lv(2, 3, torch.int64)])
    with pytest.raises(ValueError):
        mk([lv(6, 1)] * 5)                                      # more levels than the descriptor holds
