"""GPU parity of rl_prefill_attn with the fp64 oracle, through the C ABI.

Bar: the decode path's bf16 bar (same arithmetic: bf16 inputs, fp32 accumulation, softmax weights
rounded to bf16 before the value contraction): 1e-2 abs on out, 1e-3 abs on lse; rows at positions
beyond a prompt's length untouched; and consistency with the decode entry point on the K/V it
leaves behind.
"""
import math

import numpy as np
import pytest

from oracle.prefill_ref import prefill_attn_ref
from paper_2512_21450_amd import workloads as wl
from tests import util

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2512_21450_amd import binding
    return binding


def case(seed, P, L, Hq, Hkv, lens=None, gain=1.0):
    rng = np.random.default_rng(seed)
    t = lambda s, g=1.0: wl.f32_to_bf16_bits((rng.standard_normal(s) * g).astype(np.float32))
    return dict(q=t((P, L, Hq, 128), gain), k=t((P, Hkv, L, 128)), v=t((P, Hkv, L, 128)),
                lens=(rng.integers(1, L + 1, P) if lens is None else np.asarray(lens)).astype(np.int32))


def run(B, x, scale, poison=True):
    import torch
    t = util.to_device(x)
    P, L, Hq, d = x["q"].shape
    out = torch.full((P, L, Hq, d), -7.0, device="cuda")
    lse = torch.full((P, L, Hq), -7.0, device="cuda")
    B.rl_prefill_attn(t["q"], t["k"], t["v"], t["lens"], scale, out=out, lse=lse)
    torch.cuda.synchronize()
    return out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)


def check(B, x, scale, what):
    out, lse = run(B, x, scale)
    ro, rl = prefill_attn_ref(x["q"], x["k"], x["v"], x["lens"], scale)
    valid = ~np.isnan(rl)
    assert np.isfinite(out).all() and np.isfinite(lse).all(), what
    assert (out[~valid] == -7.0).all() and (lse[~valid] == -7.0).all(), f"{what}: padding rows were written"
    eo = np.abs(out[valid] - ro[valid]).max() if valid.any() else 0.0
    el = np.abs(lse[valid] - rl[valid]).max() if valid.any() else 0.0
    assert eo <= 1e-2 and el <= 1e-3, (what, eo, el)
    return eo, el


CASES = [
    # P, L_cap, Hq, Hkv
    (2, 200, 28, 4),       # r = 7: 9 positions per workgroup, 63 of 64 rows
    (3, 131, 16, 2),       # r = 8
    (2, 97, 8, 8),         # r = 1: 64 positions per workgroup
    (1, 75, 32, 2),        # r = 16: 4 positions per workgroup
    (2, 64, 12, 4),        # r = 3: 21 positions, 63 rows
    (4, 33, 10, 2),        # r = 5: 12 positions, 60 rows; one tile and one key
    (1, 1, 28, 4),         # a single token
]


@pytest.mark.parametrize("case_", CASES, ids=lambda c: "P{}L{}H{}-{}".format(*c))
def test_reduced_sizes(B, case_):
    P, L, Hq, Hkv = case_
    x = case(500 + CASES.index(case_), P, L, Hq, Hkv)
    x["lens"][0] = L                                         # one prompt fills its buffer
    check(B, x, 1.0 / math.sqrt(128), str(case_))


@pytest.mark.parametrize("P,L,Hq,Hkv", [(64, 400, 12, 4), (100, 330, 14, 2), (33, 500, 16, 16), (48, 200, 32, 2),
                                         (96, 300, 10, 2), (64, 260, 16, 2)])
def test_many_prompts_take_the_two_block_kernel(B, P, L, Hq, Hkv):
    # enough workgroups for the variant with 128 rows per workgroup (r = 3, 7, 1, 16, 5, 8: 42, 18, 128, 8, 25, 16
    # positions per block)
    x = case(900 + P, P, L, Hq, Hkv)
    x["lens"][:3] = [L, 1, 0]
    check(B, x, 1.0 / math.sqrt(128), f"P{P} L{L} {Hq}/{Hkv}")


@pytest.mark.parametrize("Hq,Hkv", [(4, 2), (14, 2)])
def test_every_length_in_the_128_row_kernel(B, Hq, Hkv):
    """Prompt lengths 0 .. 161 over 360 prompts (enough workgroups for the 128-row kernel at a capacity of 161):
    every number of tiles from one to six, every size of a partial last tile, first and last rounds of one and
    of two tiles, blocks whose last wavefronts hold no row, NaN beyond every length."""
    L = 161
    lens = np.arange(360) % (L + 1)
    x = case(31 + Hq, 360, L, Hq, Hkv, lens=lens, gain=2.0)
    for p, n in enumerate(lens):
        x["k"][p, :, n:] = 0x7FC0; x["v"][p, :, n:] = 0x7FC0; x["q"][p, n:] = 0x7FC0
    check(B, x, 0.11, f"all lengths {Hq}/{Hkv}")


def test_edge_lengths_nan_padding_and_sharp_scores(B):
    x = case(7, 5, 70, 28, 4, lens=[0, 70, 1, 32, 33], gain=3.0)
    for p, n in enumerate(x["lens"]):                       # rows beyond a length hold NaN and are never read
        x["k"][p, :, n:] = 0x7FC0; x["v"][p, :, n:] = 0x7FC0; x["q"][p, n:] = 0x7FC0
    check(B, x, 0.3, "edges")
    y = case(8, 2, 90, 16, 2, lens=[500, -4])                # lengths clamp to [0, capacity]
    out, lse = run(B, y, 0.1)
    ro, rl = prefill_attn_ref(y["q"], y["k"], y["v"], y["lens"], 0.1)
    assert np.abs(out[0] - ro[0]).max() <= 1e-2 and (out[1] == -7.0).all()


def test_determinism_and_agreement_with_the_decode_entry_point(B):
    import torch
    x = case(9, 2, 150, 28, 4, lens=[150, 77])
    t = util.to_device(x)
    o1, l1 = B.rl_prefill_attn(t["q"], t["k"], t["v"], t["lens"], 0.09)
    o2, l2 = B.rl_prefill_attn(t["q"], t["k"], t["v"], t["lens"], 0.09)
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    # the last token of each prompt is a decode query over the whole prompt as prefix (G = 1, no suffix)
    last = x["lens"] - 1
    qd = torch.stack([t["q"][p, int(last[p])] for p in range(2)])
    none = torch.zeros((2, 4, 1, 128), dtype=torch.bfloat16, device="cuda")
    od, ld = B.rl_decode_attn(qd, t["k"], t["v"], t["lens"], none, none, torch.zeros(2, dtype=torch.int32, device="cuda"),
                              0.09, 1)
    for p in range(2):
        assert (o1[p, int(last[p])] - od[p]).abs().max().item() <= 2e-3
        assert (l1[p, int(last[p])] - ld[p]).abs().max().item() <= 1e-5


def test_vlm7b_prompt_shape_on_sampled_rows(B):
    # 8 of the 32 prompts of the 7B-shaped workload: 1280 tokens (1024 visual + 256 text), 28/4 heads
    w = wl.WORKLOADS["vlm7b"]
    x = case(11, 8, w.Lp_cap, w.Hq, w.Hkv, lens=[w.Lp_cap] * 8, gain=w.q_gain)
    out, lse = run(B, x, w.scale)
    ro, rl = prefill_attn_ref(x["q"][:1], x["k"][:1], x["v"][:1], x["lens"][:1], w.scale)      # prompt 0 in full
    eo, el = np.abs(out[0] - ro[0]).max(), np.abs(lse[0] - rl[0]).max()
    print(f"\nprefill 1280 x 28/4: max|out err| {eo:.2e}  max|lse err| {el:.2e}")
    assert eo <= 1e-2 and el <= 1e-3
    ro7, rl7 = prefill_attn_ref(x["q"][7:], x["k"][7:], x["v"][7:], x["lens"][7:], w.scale)
    assert np.abs(out[7] - ro7[0]).max() <= 1e-2 and np.abs(lse[7] - rl7[0]).max() <= 1e-3


@pytest.mark.parametrize("scale", [-0.07, 0.0])
def test_non_positive_scale(B, scale):
    # large enough for the 128-row kernel, whose softmax needs a positive scale: such calls take the other kernel
    x = case(77, 100, 330, 14, 2)
    check(B, x, scale, f"scale {scale}")
