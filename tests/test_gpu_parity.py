"""Parity of the HIP path with the fp64 CPU oracle, through the C ABI (GPU).

Tolerances are the acceptance bar: fp32 inputs 1e-5 abs on out and lse; bf16
inputs (fp32 accumulation) 1e-2 abs on out and 1e-3 abs on lse.
"""
import math

import numpy as np
import pytest

from paper_2512_21450_amd import workloads as wl
from tests import util

pytestmark = pytest.mark.gpu

ALGOS = {"auto": 0, "simple": 1}


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2512_21450_amd import binding
    return binding


def check(x, scale, G, dtype, algo, what, B):
    t = util.to_device(x)
    out, lse = util.gpu_run(t, scale, G, algo=ALGOS[algo])
    ro, rl = util.oracle(x, scale, G)
    return util.compare(out, lse, ro, rl, dtype, what)


# ------------------------------------------------------------------ the five configurations, full size
@pytest.mark.parametrize("name", ["tiny", "vlm3b", "vlm7b", "agentic", "highbatch"])
def test_full_size_configs_auto(name, B):
    import torch
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    t = util.to_device(x)
    out, lse = util.gpu_run(t, w.scale, w.G)
    torch.cuda.synchronize()
    ro, rl = util.oracle(x, w.scale, w.G)
    eo, el = util.compare(out, lse, ro, rl, w.dtype, name)
    print(f"\n{name}: max|out err| {eo:.2e}  max|lse err| {el:.2e}  "
          f"Ls mean {x['suffix_lens'].mean():.0f} max {x['suffix_lens'].max()}")


@pytest.mark.parametrize("name", ["tiny", "vlm3b"])
def test_full_size_configs_simple(name, B):
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    check(x, w.scale, w.G, w.dtype, "simple", name, B)


def test_vlm7b_simple_kernel_on_sampled_sequences(B):
    """The unshared kernel at the 7B shape, checked on a subset of rows."""
    w = wl.WORKLOADS["vlm7b"]
    x = wl.make_inputs(w)
    t = util.to_device(x)
    out, lse = util.gpu_run(t, w.scale, w.G, algo=1)
    rng = np.random.default_rng(5)
    rows = np.stack([rng.integers(0, w.B, 200), rng.integers(0, w.Hq, 200)], 1).astype(np.int32)
    ro, rl = util.oracle(x, w.scale, w.G, rows=rows)
    o = out.cpu().numpy().astype(np.float64)
    l = lse.cpu().numpy().astype(np.float64)
    for b, h in rows:
        assert np.abs(o[b, h] - ro[b, h]).max() <= 1e-2
        assert abs(l[b, h] - rl[b, h]) <= 1e-3


# ------------------------------------------------------------------ reduced sizes: several tiles, ragged tails
CASES = [
    # P, G, Hq, Hkv, d, Lp_cap, Ls_cap, dtype
    (2, 3, 4, 2, 64, 70, 45, "f32"),
    (1, 4, 2, 1, 128, 33, 130, "f32"),
    (3, 8, 28, 4, 128, 200, 300, "bf16"),     # r = 7, R = 56
    (2, 8, 16, 2, 128, 131, 257, "bf16"),     # r = 8, R = 64
    (2, 16, 16, 2, 128, 97, 65, "bf16"),      # R = 128
    (2, 5, 12, 4, 128, 64, 95, "bf16"),       # r = 3, R = 15 (fewer rows than one MFMA tile)
    (3, 1, 8, 8, 128, 50, 40, "bf16"),        # G = 1, r = 1
    (1, 2, 32, 2, 128, 40, 33, "bf16"),       # r = 16
    (2, 4, 8, 2, 64, 77, 91, "bf16"),         # d = 64 bf16
    (5, 7, 6, 3, 128, 31, 1, "bf16"),         # one-row suffix buffers
    (2, 10, 16, 2, 128, 140, 90, "bf16"),     # R = 80: a full row half and one of a single 16-row block
    (3, 9, 14, 2, 128, 75, 120, "bf16"),      # r = 7, R = 63 / and next line R = 65: one row in the second half
    (2, 13, 10, 2, 128, 100, 64, "bf16"),     # r = 5, R = 65
    (2, 8, 32, 2, 128, 260, 70, "bf16"),      # r = 16, R = 128 with long prefixes
    (2, 32, 14, 2, 128, 150, 60, "bf16"),     # G = 32, r = 7: R = 224, four row parts (the last one short)
    (1, 16, 32, 2, 128, 100, 40, "bf16"),     # r = 16, R = 256
    (2, 17, 16, 2, 128, 70, 33, "bf16"),      # R = 136: three of four parts used
]


@pytest.mark.parametrize("algo", ["auto", "simple"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "P{}G{}H{}-{}d{}Lp{}Ls{}{}".format(*c))
def test_reduced_sizes(case, algo, B):
    P, G, Hq, Hkv, d, Lp_cap, Ls_cap, dtype = case
    x = util.random_case(100 + CASES.index(case), P, G, Hq, Hkv, d, Lp_cap, Ls_cap, dtype)
    check(x, 1.0 / math.sqrt(d), G, dtype, algo, str(case), B)


# ------------------------------------------------------------------ edge cases
@pytest.mark.parametrize("algo", ["auto", "simple"])
@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("f32", 64)])
def test_empty_and_full_lengths(algo, dtype, d, B):
    P, G, Hq, Hkv, Lp_cap, Ls_cap = 3, 4, 8, 2, 96, 80
    plens = [0, Lp_cap, 17]
    slens = [0, Ls_cap, 1, 33,  0, 0, Ls_cap, 5,  0, 64, 32, Ls_cap]
    x = util.random_case(3, P, G, Hq, Hkv, d, Lp_cap, Ls_cap, dtype, plens, slens)
    t = util.to_device(x)
    out, lse = util.gpu_run(t, 0.2, G, algo=ALGOS[algo])
    ro, rl = util.oracle(x, 0.2, G)
    util.compare(out, lse, ro, rl, dtype, "empty/full")
    # sequence 0 (prompt 0 has no prefix, own suffix empty) has no key at all
    assert np.isneginf(rl[0]).all() and (out[0] == 0).all().item()
    # all-empty and all-full batches
    for pl, sl in (([0] * P, [0] * (P * G)), ([Lp_cap] * P, [Ls_cap] * (P * G)), ([0] * P, [Ls_cap] * (P * G)),
                   ([Lp_cap] * P, [0] * (P * G))):
        y = dict(x, prefix_lens=np.array(pl, np.int32), suffix_lens=np.array(sl, np.int32))
        check(y, 0.2, G, dtype, algo, f"lens {pl[0]},{sl[0]}", B)


@pytest.mark.parametrize("algo", ["auto", "simple"])
def test_rows_beyond_length_may_hold_nan_and_lengths_clamp(algo, B):
    P, G, Hq, Hkv, d, Lp_cap, Ls_cap = 2, 4, 14, 2, 128, 75, 140
    x = util.random_case(11, P, G, Hq, Hkv, d, Lp_cap, Ls_cap, "bf16")
    ro, rl = util.oracle(x, 0.09, G)
    y = {k: v.copy() for k, v in x.items()}
    nan = np.uint16(0x7FC0)
    for p in range(P):
        y["k_prefix"][p, :, x["prefix_lens"][p]:] = nan
        y["v_prefix"][p, :, x["prefix_lens"][p]:] = nan
    for b in range(P * G):
        y["k_suffix"][b, :, x["suffix_lens"][b]:] = nan
        y["v_suffix"][b, :, x["suffix_lens"][b]:] = nan
    t = util.to_device(y)
    out, lse = util.gpu_run(t, 0.09, G, algo=ALGOS[algo])
    util.compare(out, lse, ro, rl, "bf16", "nan poison")
    # out-of-range lengths behave as clamped to [0, cap]
    z = dict(x, prefix_lens=np.array([Lp_cap + 1000, -7], np.int32),
             suffix_lens=np.array([-1, Ls_cap + 5, 3, 2 ** 30, 0, 9, -2 ** 31, Ls_cap], np.int32))
    check(z, 0.09, G, "bf16", algo, "clamp", B)


@pytest.mark.parametrize("algo", ["auto", "simple"])
def test_constant_v_and_sharp_softmax(algo, B):
    P, G, Hq, Hkv, d = 2, 8, 28, 4, 128
    x = util.random_case(21, P, G, Hq, Hkv, d, 150, 210, "bf16", gain=6.0)   # scores with std ~6
    c = wl.f32_to_bf16_bits(np.linspace(-3, 3, d).astype(np.float32))
    y = dict(x)
    y["v_prefix"] = np.broadcast_to(c, x["v_prefix"].shape).copy()
    y["v_suffix"] = np.broadcast_to(c, x["v_suffix"].shape).copy()
    t = util.to_device(y)
    out, lse = util.gpu_run(t, 1 / math.sqrt(d), G, algo=ALGOS[algo])
    cf = wl.bf16_bits_to_f32(c)
    has_key = (np.repeat(y["prefix_lens"], G) + y["suffix_lens"]) > 0
    o = out.cpu().numpy()
    assert np.abs(o[has_key] - cf).max() <= 5e-5       # weights sum to one: far below bf16 rounding
    check(x, 1 / math.sqrt(d), G, "bf16", algo, "sharp", B)


def test_sharing_is_invisible_replicated_prefix(B):
    """Shared prefix == the prefix physically copied in front of every sequence's own keys."""
    P, G, Hq, Hkv, d, Lp_cap, Ls_cap = 3, 8, 28, 4, 128, 120, 100
    x = util.random_case(31, P, G, Hq, Hkv, d, Lp_cap, Ls_cap, "bf16")
    Bn = P * G
    ks = np.zeros((Bn, Hkv, Lp_cap + Ls_cap, d), np.uint16)
    vs = np.zeros_like(ks)
    sl = np.zeros(Bn, np.int32)
    for b in range(Bn):
        p, Lp, Ls = b // G, int(x["prefix_lens"][b // G]), int(x["suffix_lens"][b])
        ks[b, :, :Lp], vs[b, :, :Lp] = x["k_prefix"][p, :, :Lp], x["v_prefix"][p, :, :Lp]
        ks[b, :, Lp:Lp + Ls], vs[b, :, Lp:Lp + Ls] = x["k_suffix"][b, :, :Ls], x["v_suffix"][b, :, :Ls]
        sl[b] = Lp + Ls
    y = dict(x, k_suffix=ks, v_suffix=vs, suffix_lens=sl, prefix_lens=np.zeros(P, np.int32))
    ro, rl = util.oracle(x, 0.1, G)
    for inp in (x, y):
        out, lse = util.gpu_run(util.to_device(inp), 0.1, G)
        util.compare(out, lse, ro, rl, "bf16", "replicated prefix")


@pytest.mark.parametrize("algo", ["auto", "simple"])
def test_bitwise_determinism(algo, B):
    import torch
    w = wl.scaled(wl.WORKLOADS["agentic"], P=4, Ls_cap=1024)
    x = wl.make_inputs(w)
    t = util.to_device(x)
    o1, l1 = util.gpu_run(t, w.scale, w.G, algo=ALGOS[algo])
    o1, l1 = o1.clone(), l1.clone()
    for _ in range(3):
        o2, l2 = util.gpu_run(t, w.scale, w.G, algo=ALGOS[algo])
        assert torch.equal(o1, o2) and torch.equal(l1, l2)


def test_long_tail_load_balance_case(B):
    """One 4096-token outlier next to short suffixes (agentic shape)."""
    w = wl.scaled(wl.WORKLOADS["agentic"], P=2)
    x = wl.make_inputs(w)
    x["suffix_lens"][:] = np.minimum(x["suffix_lens"], 300)
    x["suffix_lens"][5] = 4096
    check(x, w.scale, w.G, "bf16", "auto", "outlier", B)


def test_lse_null_and_caller_buffers(B):
    import torch
    x = util.random_case(41, 2, 4, 8, 2, 128, 60, 70, "bf16")
    t = util.to_device(x)
    out = torch.full((8, 8, 128), 7.0, device="cuda:0")
    ds = B.desc_from_tensors(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], t["k_suffix"], t["v_suffix"],
                             t["suffix_lens"], 0.1, 4, out, None)
    need = B.rl_decode_attn_workspace_bytes(ds)
    ws = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda:0")
    ds.workspace, ds.workspace_bytes = ws.data_ptr(), need
    assert B.rl_decode_attn_raw(ds, torch.cuda.current_stream().cuda_stream) == 0
    ro, rl = util.oracle(x, 0.1, 4)
    assert np.abs(out.cpu().numpy() - ro).max() <= 1e-2
    if need:
        ds.workspace_bytes = need - 1
        assert B.rl_decode_attn_raw(ds, None) == B.RLDA_ERR_WORKSPACE
        ds.workspace, ds.workspace_bytes = None, need
        assert B.rl_decode_attn_raw(ds, None) == B.RLDA_ERR_WORKSPACE


def test_non_default_stream(B):
    import torch
    x = util.random_case(43, 2, 8, 16, 2, 128, 90, 110, "bf16")
    t = util.to_device(x)
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        out, lse = util.gpu_run(t, 0.1, 8, stream=s)
    s.synchronize()
    ro, rl = util.oracle(x, 0.1, 8)
    util.compare(out, lse, ro, rl, "bf16", "side stream")


# ------------------------------------------------------------------ the combine step on its own
@pytest.mark.parametrize("d", [64, 128])
def test_lse_combine_against_oracle(d, B):
    import torch
    from oracle import ref
    rng = np.random.default_rng(7)
    n_parts, n_rows = 5, 37
    o = rng.standard_normal((n_parts, n_rows, d)).astype(np.float32)
    l = (rng.standard_normal((n_parts, n_rows)) * 3).astype(np.float32)
    l[rng.random((n_parts, n_rows)) < 0.3] = -np.inf
    l[:, 0] = -np.inf                       # a row with every part empty
    o[np.isneginf(l)] = np.nan              # empty parts may hold anything
    out, lse = B.rl_lse_combine(torch.from_numpy(o).cuda(), torch.from_numpy(l).cuda())
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    for r in range(n_rows):
        ro, rl = ref.lse_combine_ref(np.nan_to_num(o[:, r].astype(np.float64)), l[:, r].astype(np.float64))
        if np.isneginf(rl):
            assert np.isneginf(lse[r]) and not out[r].any()
        else:
            assert abs(lse[r] - rl) <= 1e-5 and np.abs(out[r] - ro).max() <= 1e-5


def test_one_workspace_reused_across_shapes_and_steps(B):
    """A decode loop reuses one workspace; stale partials of an earlier, larger call must not leak."""
    import torch
    big = util.random_case(51, 4, 8, 28, 4, 128, 300, 500, "bf16")
    small = util.random_case(52, 2, 8, 28, 4, 128, 300, 500, "bf16", plens=[40, 0], slens=[3, 0, 70, 0, 0, 0, 1, 33, 0, 0, 0, 0, 0, 0, 0, 5])
    tb, tsm = util.to_device(big), util.to_device(small)
    out_b = torch.empty((32, 28, 128), dtype=torch.float32, device="cuda:0")
    ds_b = B.desc_from_tensors(tb["q"], tb["k_prefix"], tb["v_prefix"], tb["prefix_lens"], tb["k_suffix"], tb["v_suffix"],
                               tb["suffix_lens"], 0.1, 8, out_b, None)
    ws = torch.empty(B.rl_decode_attn_workspace_bytes(ds_b), dtype=torch.uint8, device="cuda:0")
    ws.fill_(0xFF)                                   # NaN patterns everywhere
    sh = torch.cuda.current_stream().cuda_stream
    for t, x, P in ((tb, big, 4), (tsm, small, 2), (tb, big, 4), (tsm, small, 2)):
        out = torch.empty((P * 8, 28, 128), dtype=torch.float32, device="cuda:0")
        lse = torch.empty((P * 8, 28), dtype=torch.float32, device="cuda:0")
        ds = B.desc_from_tensors(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], t["k_suffix"], t["v_suffix"],
                                 t["suffix_lens"], 0.1, 8, out, lse, ws)
        assert B.rl_decode_attn_workspace_bytes(ds) <= ws.numel()
        assert B.rl_decode_attn_raw(ds, sh) == 0
        ro, rl = util.oracle(x, 0.1, 8)
        util.compare(out, lse, ro, rl, "bf16", f"reused workspace P={P}")


def test_profiled_entry_point_records_the_middle_event(B):
    import torch
    w = wl.scaled(wl.WORKLOADS["vlm7b"], P=4)
    x = wl.make_inputs(w)
    t = util.to_device(x)
    out = torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device="cuda:0")
    lse = torch.empty((w.B, w.Hq), dtype=torch.float32, device="cuda:0")
    ds = B.desc_from_tensors(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], t["k_suffix"], t["v_suffix"],
                             t["suffix_lens"], w.scale, w.G, out, lse)
    ws = torch.empty(B.rl_decode_attn_workspace_bytes(ds), dtype=torch.uint8, device="cuda:0")
    ds.workspace, ds.workspace_bytes = ws.data_ptr(), ws.numel()
    s = torch.cuda.current_stream()
    e0, em, e1 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
    em.record(s)
    torch.cuda.synchronize()
    e0.record(s)
    assert B.rl_decode_attn_profiled(ds, s.cuda_stream, em.cuda_event) == 0
    e1.record(s)
    torch.cuda.synchronize()
    assert 0.0 < e0.elapsed_time(em) <= e0.elapsed_time(e1)
    ro, rl = util.oracle(x, w.scale, w.G)
    util.compare(out, lse, ro, rl, "bf16", "profiled")


def test_two_level_shared_prefix_by_composition(B):
    """A prefix tree (prompt shared by the group, a first turn shared by sub-groups, own suffix) needs no
    new kernel: one call per level yields (o, lse) partials over disjoint key sets and rl_lse_combine
    merges them.  Checked against the oracle on the concatenated keys."""
    import torch
    P, G, sub, Hq, Hkv, d = 3, 8, 4, 28, 4, 128
    L0, L1, Ls = 300, 150, 90
    rng = np.random.default_rng(61)
    t16 = lambda shape: wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    q = t16((P * G, Hq, d))
    k0, v0 = t16((P, Hkv, L0, d)), t16((P, Hkv, L0, d))                       # level 0: one per prompt
    k1, v1 = t16((P * G // sub, Hkv, L1, d)), t16((P * G // sub, Hkv, L1, d))  # level 1: one per sub-group
    ks, vs = t16((P * G, Hkv, Ls, d)), t16((P * G, Hkv, Ls, d))
    len0 = rng.integers(1, L0 + 1, P).astype(np.int32)
    len1 = rng.integers(0, L1 + 1, P * G // sub).astype(np.int32)
    lens = rng.integers(0, Ls + 1, P * G).astype(np.int32)
    # oracle: level 1 and the own suffix concatenated per sequence behind the prompt
    cat_k = np.zeros((P * G, Hkv, L1 + Ls, d), np.uint16); cat_v = np.zeros_like(cat_k)
    cat_len = np.zeros(P * G, np.int32)
    for b in range(P * G):
        a, n = int(len1[b // sub]), int(lens[b])
        cat_k[b, :, :a] = k1[b // sub, :, :a]; cat_v[b, :, :a] = v1[b // sub, :, :a]
        cat_k[b, :, a:a + n] = ks[b, :, :n]; cat_v[b, :, a:a + n] = vs[b, :, :n]
        cat_len[b] = a + n
    from oracle import ref
    ro, rl = ref.decode_attn_ref(q, k0, v0, len0, cat_k, cat_v, cat_len, 0.09, G)
    # GPU: level 0 with no suffix; level 1 as the "prefix" of groups of `sub` plus the own suffix; merge
    dev = lambda a: (torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16) if a.dtype == np.uint16
                     else torch.from_numpy(a).cuda())
    qd = dev(q)
    zero = torch.zeros(P * G, dtype=torch.int32, device="cuda")
    o0, l0 = B.rl_decode_attn(qd, dev(k0), dev(v0), dev(len0), dev(ks), dev(vs), zero, 0.09, G)
    o1, l1 = B.rl_decode_attn(qd, dev(k1), dev(v1), dev(len1), dev(ks), dev(vs), dev(lens), 0.09, sub)
    parts_o = torch.stack([o0.reshape(-1, d), o1.reshape(-1, d)])
    parts_l = torch.stack([l0.reshape(-1), l1.reshape(-1)])
    out, lse = B.rl_lse_combine(parts_o, parts_l)
    torch.cuda.synchronize()
    util.compare(out.reshape(P * G, Hq, d), lse.reshape(P * G, Hq), ro, rl, "bf16", "two-level prefix")


@pytest.mark.parametrize("P,plan", [(3000, "shared"), (3300, "shared"), (7001, "shared")])
def test_many_short_sequences_fill_the_length_scan(B, P, plan):
    """Thousands of prompts and sequences: the in-kernel length scan and the owner search run at their
    capacity (16 384 entries: 3000 prompts of 4 sequences fit, 3300 do not); beyond it the call stays on
    the shared-prefix kernels and runs whole prompts in two or three launches."""
    import torch
    G, Hq, Hkv, d = 4, 4, 2, 128
    x = util.random_case(70 + P, P, G, Hq, Hkv, d, 40, 40, "bf16")
    t = util.to_device(x)
    out = torch.empty((P * G, Hq, d), dtype=torch.float32, device="cuda:0")
    ds = B.desc_from_tensors(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], t["k_suffix"], t["v_suffix"],
                             t["suffix_lens"], 0.1, G, out, None)
    assert B.rl_decode_attn_plan(ds) == {"shared": B.RLDA_ALGO_SHARED, "simple": B.RLDA_ALGO_SIMPLE}[plan]
    check(x, 0.1, G, "bf16", "auto", f"P={P}", B)


@pytest.mark.parametrize("tiles", [2047, 2048, 2049])
def test_around_the_tile_count_where_half_the_workgroup_pairs_take_over(B, tiles):
    """A batch of fewer than 2048 tiles is cut among half the workgroup pairs; the streaming kernel and the
    combine kernel each decide that from the tile totals on the device.  One KV head, so that one sequence's
    length moves the total by single tiles: 4 prompts x 16 tiles + 32 sequences x 62 tiles = 2048."""
    P, G, Hq, Hkv, d = 4, 8, 8, 1, 128
    pl = np.full(P, 16 * 32, np.int32)
    sl = np.full(P * G, 62 * 32, np.int32)
    sl[13] += (tiles - 2048) * 32
    x = util.random_case(600 + tiles, P, G, Hq, Hkv, d, 16 * 32, 63 * 32, "bf16", plens=pl, slens=sl)
    assert int((-(-x["prefix_lens"] // 32)).sum() + (-(-x["suffix_lens"] // 32)).sum()) == tiles
    check(x, 0.09, G, "bf16", "auto", f"{tiles} tiles", B)


@pytest.mark.parametrize("paged", [False, True])
def test_rows_with_many_parts_in_the_16_lane_combine(B, paged):
    """128 prefix units select the 16-lane combine kernel; one prompt and one sequence hold nearly all
    keys, so their rows are cut among most workgroups: more parts per row than one request (4) and than
    one batch of lanes (16) hold, next to rows with a single part and rows with none."""
    import torch
    P, G, Hq, Hkv, d = 64, 2, 4, 2, 128
    pl = np.full(P, 8, np.int32)
    pl[0], pl[9], pl[63] = 6000, 0, 700
    sl = np.full(P * G, 5, np.int32)
    sl[1], sl[18], sl[19], sl[127] = 4000, 0, 0, 900
    x = util.random_case(77, P, G, Hq, Hkv, d, 6016, 4000, "bf16", plens=pl, slens=sl)
    if not paged:
        check(x, 0.1, G, "bf16", "auto", "many parts", B)
        return
    y = wl.to_pages(x, 64, seed=3)
    t = util.to_device(y)
    out, lse = util.gpu_run_paged(t, 0.1, G)
    torch.cuda.synchronize()
    ro, rl = util.oracle_paged(y, 0.1, G)
    util.compare(out, lse, ro, rl, "bf16", "many parts, paged")


@pytest.mark.parametrize("scale", [-0.09, 0.0])
def test_non_positive_scale_runs_on_the_simple_kernel(B, scale):
    """The shared-prefix path takes its row maxima before scaling and therefore positive scales only; anything
    else (anti-attention, a uniform average) is planned onto the simple kernel, with the same result."""
    import torch
    x = util.random_case(91, 3, 4, 8, 2, 128, 150, 90, "bf16")
    t = util.to_device(x)
    out = torch.empty((12, 8, 128), dtype=torch.float32, device="cuda:0")
    ds = B.desc_from_tensors(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], t["k_suffix"], t["v_suffix"],
                             t["suffix_lens"], scale, 4, out, None)
    assert B.rl_decode_attn_plan(ds) == B.RLDA_ALGO_SIMPLE
    check(x, scale, 4, "bf16", "auto", f"scale {scale}", B)
    with pytest.raises(B.RldaError):
        util.gpu_run(t, scale, 4, algo=B.RLDA_ALGO_SHARED)
