"""rl_decode_attn_static (the entry point that allocates nothing: its scratch is an array inside the
library's device image) against rl_decode_attn on the same inputs, through the C ABI: two calls in a
row, the second on a smaller problem, so that whatever the first call left in the shared array is
there when the second one runs.  Same kernels, same static partition: the results must be equal bit
for bit, and the first one is checked against the oracle as well."""
import ctypes

import numpy as np
import pytest

from paper_2512_21450_amd import binding as B
from paper_2512_21450_amd import workloads as wl
from tests import util

pytestmark = pytest.mark.gpu


def both(t, w, torch):
    """(out, lse) of rl_decode_attn with a caller workspace, and of rl_decode_attn_static, on preallocated outputs"""
    res = []
    for static in (False, True):
        out = torch.full((w.B, w.Hq, w.d), float("nan"), dtype=torch.float32, device="cuda:0")
        lse = torch.full((w.B, w.Hq), float("nan"), dtype=torch.float32, device="cuda:0")
        ds = B.desc_from_tensors(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], t["k_suffix"], t["v_suffix"],
                                 t["suffix_lens"], w.scale, w.G, out, lse, None, B.RLDA_ALGO_AUTO,
                                 t.get("k_scale"), t.get("v_scale"))
        need = B.rl_decode_attn_workspace_bytes(ds)
        assert need <= B.rl_decode_attn_static_workspace_limit()
        sh = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
        if static:
            rc = B.rl_decode_attn_static_raw(ds, sh)          # workspace fields left NULL / 0 on purpose
        else:
            ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda:0")
            ds.workspace, ds.workspace_bytes = ws.data_ptr(), ws.numel()
            rc = B.rl_decode_attn_raw(ds, sh)
        assert rc == B.RLDA_OK, B.rl_decode_attn_strerror(rc)
        torch.cuda.synchronize()
        res.append((out, lse))
    return res


def test_static_workspace_entry_point_two_calls_second_smaller():
    import torch
    big = wl.scaled(wl.WORKLOADS["vlm7b"], P=6, Lp_cap=300, Ls_cap=400, prefix=("uniform", 300), suffix=("uniform", 400))
    small = wl.scaled(wl.WORKLOADS["vlm7b"], P=2, Lp_cap=100, Ls_cap=77, prefix=("uniform", 100), suffix=("uniform", 77))
    for w in (big, small):
        x = wl.make_inputs(w)
        t = util.to_device(x)
        ds0 = B.make_desc(B.RLDA_BF16, w.P, w.G, w.Hq, w.Hkv, w.d, w.Lp_cap, w.Ls_cap, w.scale)
        assert B.rl_decode_attn_plan(ds0) == B.RLDA_ALGO_SHARED  # the path that has a scratch buffer
        (o_ws, l_ws), (o_st, l_st) = both(t, w, torch)
        assert torch.equal(o_ws, o_st), f"{w.P} prompts: out differs between the two entry points"
        assert torch.equal(l_ws, l_st), f"{w.P} prompts: lse differs between the two entry points"
        ro, rl = util.oracle(x, w.scale, w.G)
        util.compare(o_st, l_st, ro, rl, w.dtype, f"static entry point, {w.P} prompts")


def test_static_entry_point_on_the_path_without_scratch():
    import torch
    w = wl.WORKLOADS["tiny"]                                  # fp32: one kernel, no partial results
    x = wl.make_inputs(w)
    t = util.to_device(x)
    (o_ws, l_ws), (o_st, l_st) = both(t, w, torch)
    assert torch.equal(o_ws, o_st) and torch.equal(l_ws, l_st)
