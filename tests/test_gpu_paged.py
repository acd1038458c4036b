"""GPU parity of the paged-suffix entry point against the fp64 oracle, through the C ABI."""
import numpy as np
import pytest

from paper_2512_21450_amd import workloads as wl
from tests import util

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2512_21450_amd import binding
    return binding


def check(y, w_dtype, scale, G, active=None, what="", **kw):
    import torch
    t = util.to_device(y)
    act = None if active is None else torch.from_numpy(active).to("cuda:0")
    out, lse = util.gpu_run_paged(t, scale, G, active=act, **kw)
    torch.cuda.synchronize()
    ro, rl = util.oracle_paged(y, scale, G, active=active)
    return util.compare(out, lse, ro, rl, w_dtype, what)


@pytest.mark.parametrize("name,ps", [("tiny", 32), ("vlm3b", 64), ("vlm7b", 128), ("agentic", 256), ("highbatch", 32)])
def test_full_size_configs_paged(B, name, ps):
    w = wl.WORKLOADS[name]
    y = wl.to_pages(wl.make_inputs(w, threads=8), ps, seed=w.seed)
    print(f"paged {name} page {ps} pool {y['k_pages'].shape}", flush=True)
    check(y, w.dtype, w.scale, w.G, what=f"paged {name}")


@pytest.mark.parametrize("ps", [16, 32, 64, 128, 256, 512])     # 16 rows: shorter than a key tile, the simple kernel's
@pytest.mark.parametrize("dtype,d,algo", [("bf16", 128, "auto"), ("bf16", 128, "simple"), ("f32", 64, "auto")])
def test_page_sizes_on_both_kernel_families(B, ps, dtype, d, algo):
    x = util.random_case(100 + ps, 3, 4, 8, 2, d, 150, 700, dtype)
    y = wl.to_pages(x, ps, seed=ps)
    a = {"auto": B.RLDA_ALGO_AUTO, "simple": B.RLDA_ALGO_SIMPLE}[algo]
    check(y, dtype, 0.11, 4, algo=a, what=f"page {ps} {dtype} {algo}")


def test_finished_sequences_and_finished_groups(B):
    w = wl.scaled(wl.WORKLOADS["vlm7b"], P=6)
    y = wl.to_pages(wl.make_inputs(w), 64, seed=5)
    rng = np.random.default_rng(5)
    act = (rng.random(w.B) < 0.6).astype(np.uint8)
    act[0:w.G] = 0                                  # prompt 0: whole group finished, its prefix is skipped
    act[w.G:2 * w.G] = 1                            # prompt 1: all live
    act[2 * w.G] = 1; act[2 * w.G + 1:3 * w.G] = 0  # prompt 2: one survivor
    check(y, w.dtype, w.scale, w.G, active=act, what="finished mix")
    check(y, w.dtype, w.scale, w.G, active=np.zeros(w.B, np.uint8), what="all finished")
    check(y, w.dtype, w.scale, w.G, active=np.ones(w.B, np.uint8), what="all live")
    check(y, w.dtype, w.scale, w.G, active=act, algo=B.RLDA_ALGO_SIMPLE, what="finished mix, simple kernel")


def test_finished_sequences_may_hold_garbage(B):
    # a finished sequence's table row and length are never used
    x = util.random_case(7, 2, 4, 28, 4, 128, 200, 300, "bf16")
    y = wl.to_pages(x, 32, seed=7)
    act = np.array([1, 0, 1, 1, 0, 0, 1, 1], np.uint8)
    ro, rl = util.oracle_paged(y, 0.1, 4, active=act)
    z = dict(y)
    z["block_table"] = y["block_table"].copy()
    z["suffix_lens"] = y["suffix_lens"].copy()
    for b in np.flatnonzero(act == 0):
        z["block_table"][b] = 2_000_000_000
        z["suffix_lens"][b] = 1 << 30
    import torch
    t = util.to_device(z)
    out, lse = util.gpu_run_paged(t, 0.1, 4, active=torch.from_numpy(act).cuda())
    util.compare(out, lse, ro, rl, "bf16", "garbage rows of finished sequences")


def test_out_of_range_page_ids_are_clamped_not_followed(B):
    # a wrong id in a used entry gives a wrong result for that sequence only, and no stray access
    x = util.random_case(8, 2, 4, 28, 4, 128, 100, 260, "bf16", slens=[260, 100, 64, 1, 0, 33, 200, 129])
    y = wl.to_pages(x, 64, seed=8, poison=False)
    ro, rl = util.oracle_paged(y, 0.1, 4)
    z = dict(y); z["block_table"] = y["block_table"].copy()
    z["block_table"][0, 1] = -5
    z["block_table"][6, 0] = 1_000_000
    import torch
    out, lse = util.gpu_run_paged(util.to_device(z), 0.1, 4)
    torch.cuda.synchronize()
    keep = [1, 2, 3, 4, 5, 7]
    util.compare(out[keep], lse[keep], ro[keep], rl[keep], "bf16", "neighbours of a bad page id")
    assert torch.isfinite(out).all()


def test_paged_equals_contiguous_bitwise_when_pages_are_whole_tiles(B):
    # same tiles in the same order: the two entry points must agree to the last bit
    import torch
    w = wl.scaled(wl.WORKLOADS["agentic"], P=4)
    x = wl.make_inputs(w)
    y = wl.to_pages(x, 128, seed=3)
    o1, l1 = util.gpu_run(util.to_device(x), w.scale, w.G)
    o2, l2 = util.gpu_run_paged(util.to_device(y), w.scale, w.G)
    assert torch.equal(o1, o2) and torch.equal(l1, l2)


def test_decode_loop_captured_in_a_graph(B):
    """Several decode steps (attention, then every live sequence grows by one key) recorded once
    and replayed: each replay must reproduce the eager run of the same steps."""
    import torch
    w = wl.scaled(wl.WORKLOADS["vlm7b"], P=4, Ls_cap=512, suffix=("uniform", 400))
    x = wl.make_inputs(w)
    x["suffix_lens"] = np.minimum(x["suffix_lens"], 400).astype(np.int32)
    full = dict(x); full["suffix_lens"] = np.full(w.B, 512, np.int32)     # pages for the whole capacity
    y = wl.to_pages(full, 64, seed=11, poison=False)
    y["suffix_lens"] = x["suffix_lens"]
    act_np = (np.arange(w.B) % 5 != 0).astype(np.uint8)
    t = util.to_device(y)
    act = torch.from_numpy(act_np).cuda()
    lens0 = t["suffix_lens"].clone()
    steps = 3
    outs = [torch.empty((w.B, w.Hq, w.d), dtype=torch.float32, device="cuda") for _ in range(steps)]
    lses = [torch.empty((w.B, w.Hq), dtype=torch.float32, device="cuda") for _ in range(steps)]
    ds0 = B.paged_desc_from_tensors(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], t["k_pages"], t["v_pages"],
                                    t["block_table"], t["suffix_lens"], w.scale, w.G, outs[0], lses[0], act)
    ws = torch.empty(B.rl_decode_attn_paged_workspace_bytes(ds0), dtype=torch.uint8, device="cuda")
    inc = act.to(torch.int32)

    def run_steps():
        s = torch.cuda.current_stream().cuda_stream
        for i in range(steps):
            ds = B.paged_desc_from_tensors(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], t["k_pages"],
                                           t["v_pages"], t["block_table"], t["suffix_lens"], w.scale, w.G,
                                           outs[i], lses[i], act, ws)
            assert B.rl_decode_attn_paged_raw(ds, s, None) == 0
            t["suffix_lens"].add_(inc)

    run_steps()                                           # eager
    torch.cuda.synchronize()
    eager = [(o.clone(), l.clone()) for o, l in zip(outs, lses)]
    # the eager result itself against the oracle, step by step
    for i in range(steps):
        yi = dict(y); yi["suffix_lens"] = (x["suffix_lens"] + i * act_np).astype(np.int32)
        ro, rl = util.oracle_paged(yi, w.scale, w.G, active=act_np)
        util.compare(eager[i][0], eager[i][1], ro, rl, "bf16", f"eager step {i}")
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    t["suffix_lens"].copy_(lens0)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            run_steps()
    for rep in range(3):
        t["suffix_lens"].copy_(lens0)
        for o, l in zip(outs, lses):
            o.fill_(float("nan")); l.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for i in range(steps):
            assert torch.equal(outs[i], eager[i][0]) and torch.equal(lses[i], eager[i][1]), f"replay {rep} step {i}"
        assert torch.equal(t["suffix_lens"], lens0 + steps * inc)


def test_no_suffix_pages_at_all_and_very_large_pages(B):
    import torch
    x = util.random_case(9, 2, 4, 28, 4, 128, 130, 64, "bf16")
    t = util.to_device(x)
    # a batch right after the prompt: no page allocated yet, table with zero columns, empty pools
    empty_pool = torch.empty((0, 4, 64, 128), dtype=torch.bfloat16, device="cuda")
    table = torch.empty((8, 0), dtype=torch.int32, device="cuda")
    out, lse = B.rl_decode_attn_paged(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], empty_pool, empty_pool,
                                      table, t["suffix_lens"], 0.1, 4)
    z = dict(x); z["suffix_lens"] = np.zeros(8, np.int32)
    ro, rl = util.oracle(z, 0.1, 4)
    util.compare(out, lse, ro, rl, "bf16", "no pages")
    # one page of 1024 rows per sequence
    y = wl.to_pages(util.random_case(10, 2, 4, 28, 4, 128, 130, 900, "bf16"), 1024, seed=1)
    check(y, "bf16", 0.1, 4, what="page 1024")
