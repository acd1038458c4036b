"""rl_decode_attn_tree on the GPU against the fp64 oracle on the concatenated keys: two and three levels of
shared segments with ragged (and empty) segments and suffixes, sharing widths down to one sequence, levels
that do not nest, and the single-level case against rl_decode_attn bit for bit."""
import numpy as np
import pytest

from paper_2512_21450_amd import binding as B
from paper_2512_21450_amd import workloads as wl
from tests import util

pytestmark = pytest.mark.gpu


def to_dev(a):
    import torch
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def run_tree(x, scale):
    import torch
    lv = [(to_dev(k), to_dev(v), to_dev(l), g) for k, v, l, g in x["levels"]]
    out, lse = B.rl_decode_attn_tree(to_dev(x["q"]), lv, to_dev(x["k_suffix"]), to_dev(x["v_suffix"]),
                                     to_dev(x["suffix_lens"]), scale)
    torch.cuda.synchronize()
    return out, lse


def oracle_tree(x, scale, **kw):
    from oracle import ref
    return ref.decode_attn_tree_ref(x["q"], x["levels"], x["k_suffix"], x["v_suffix"], x["suffix_lens"], scale, **kw)


CASES = [
    # (B, Hq, Hkv, levels (group, cap, lengths), Ls_cap, suffix lengths, empty fraction)
    ("two levels, 7 heads per KV head", 32, 28, 4, [(8, 300, ("uniform", 300)), (4, 150, ("uniform", 150))], 400, ("uniform", 400), 0.15),
    ("three nested levels", 32, 28, 4, [(8, 200, ("uniform", 200)), (4, 90, ("uniform", 90)), (2, 70, ("uniform", 70))], 260, ("uniform", 260), 0.2),
    ("a level of width one", 24, 16, 2, [(8, 130, ("uniform", 130)), (1, 45, ("uniform", 45))], 100, ("uniform", 100), 0.1),
    ("levels that do not nest", 24, 16, 2, [(4, 100, ("uniform", 100)), (6, 77, ("uniform", 77))], 64, ("uniform", 64), 0.1),
    ("64 rows per segment, four levels", 32, 16, 2, [(8, 64, ("const", 64)), (8, 33, ("uniform", 33)), (2, 40, ("uniform", 40)), (4, 31, ("const", 31))], 50, ("uniform", 50), 0.0),
    ("one head per KV head, long ragged segments", 16, 4, 4, [(16, 1500, ("uniform", 1500)), (2, 700, ("lognormal", 200.0, 1.0))], 900, ("lognormal", 150.0, 1.0), 0.1),
    ("nothing but empty segments", 16, 8, 2, [(4, 40, ("const", 0)), (2, 40, ("const", 0))], 40, ("uniform", 40), 0.5),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_tree_against_the_oracle(case):
    _, Bn, Hq, Hkv, levels, Ls_cap, suffix, empty = case
    x = wl.make_tree_inputs(4100 + Bn + len(levels), Bn, Hq, Hkv, 128, levels, Ls_cap, suffix, q_gain=1.5, empty=empty)
    scale = 1.0 / np.sqrt(128)
    out, lse = run_tree(x, scale)
    ro, rl = oracle_tree(x, scale)
    util.compare(out, lse, ro, rl, "bf16", case[0])


def test_one_level_equals_the_shared_prefix_call_bit_for_bit():
    import torch
    w = wl.scaled(wl.WORKLOADS["vlm7b"], P=3, Lp_cap=333, Ls_cap=211, prefix=("uniform", 333), suffix=("uniform", 211))
    x = wl.make_inputs(w)
    t = util.to_device(x)
    o1, l1 = util.gpu_run(t, w.scale, w.G)
    o2, l2 = B.rl_decode_attn_tree(t["q"], [(t["k_prefix"], t["v_prefix"], t["prefix_lens"], w.G)], t["k_suffix"],
                                   t["v_suffix"], t["suffix_lens"], w.scale)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(l1, l2)      # same partition, same order of additions


def test_agentic_two_level_workload_at_full_size_and_repeatable():
    import torch
    x = wl.make_tree_inputs(1004, 128, 28, 4, 128, [(8, 1344, ("agentic", 3, 256, 64, 192)), (4, 512, ("uniform", 512))],
                            4096, ("lognormal", 300.0, 1.0), threads=16)
    scale = 1.0 / np.sqrt(128)
    out, lse = run_tree(x, scale)
    out2, lse2 = run_tree(x, scale)
    assert torch.equal(out, out2) and torch.equal(lse, lse2)
    rng = np.random.default_rng(1)
    rows = np.stack([rng.integers(0, 128, 96), rng.integers(0, 28, 96)], 1).astype(np.int32)
    ro, rl = oracle_tree(x, scale, rows=rows)
    o, l = out.cpu().numpy(), lse.cpu().numpy()
    eo = max(float(np.abs(o[b, h] - ro[b, h]).max()) for b, h in rows)
    el = max(abs(float(l[b, h]) - rl[b, h]) for b, h in rows)
    assert eo <= 1e-2 and el <= 1e-3, (eo, el)
