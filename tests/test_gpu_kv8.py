"""8-bit (e4m3) K/V stores on the GPU, through the C ABI, against the fp64 oracle.

The decode of every byte value is checked exactly with one-key attentions
(out = v_scale * value, lse = scale * k_scale * <q, k>), on the matrix-core
path (which widens the bytes with the hardware converter) and on the simple
kernel (which decodes them with integer operations); then the usual parity
cases at the bf16 tolerance (1e-2 abs on out, 1e-3 abs on lse).
"""
import math

import numpy as np
import pytest

from oracle import ref
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


def byte_rows():
    """Four rows of 128 bytes that together hold every non-NaN e4m3 byte; the magnitudes inside
    a row span less than 2^11, so a row survives the fp16 staging of partial results exactly."""
    lo = np.arange(0x00, 0x40, dtype=np.uint8)            # 0 .. 1.875
    hi = np.arange(0x40, 0x7F, dtype=np.uint8)            # 2 .. 448 (0x7f is NaN)
    hi = np.concatenate([hi, hi[-1:]])
    rows = [np.concatenate([r, r[::-1]]) for r in (lo, hi, lo | 0x80, hi | 0x80)]
    return np.stack(rows)                                  # [4, 128]


@pytest.mark.parametrize("algo", ["auto", "simple"])
@pytest.mark.parametrize("where", ["prefix", "suffix"])
def test_every_byte_value_decodes_exactly(where, algo, B):
    import torch
    G, H, d = 128, 4, 128                                   # r = 1: KV head j serves query head j
    rows = byte_rows()
    vals = ref.e4m3_to_f64(rows)
    q = np.zeros((G, H, d), np.float32)
    q[np.arange(G), :, np.arange(G)] = 1.0                  # sequence g asks for column g
    x = dict(q=wl.f32_to_bf16_bits(q), prefix_lens=np.array([1 if where == "prefix" else 0], np.int32),
             suffix_lens=np.full(G, 0 if where == "prefix" else 1, np.int32))
    pre = np.full((1, H, 2, d), 0x7F, np.uint8)             # NaN bytes wherever no key lives
    suf = np.full((G, H, 2, d), 0x7F, np.uint8)
    if where == "prefix":
        pre[0, :, 0, :] = rows
    else:
        suf[:, :, 0, :] = rows[None]
    x.update(k_prefix=pre, v_prefix=pre.copy(), k_suffix=suf, v_suffix=suf.copy())
    x["k_scale"] = np.array([1.0, 0.5, 0.75, 0.011], np.float32)
    x["v_scale"] = np.array([1.0, 2.0, 0.3, 0.0131], np.float32)
    scale = 1.0 / 64
    t = util.to_device(x)
    out, lse = util.gpu_run(t, scale, G, algo=ALGOS[algo])
    torch.cuda.synchronize()
    out, lse = out.cpu().numpy(), lse.cpu().numpy()
    for h in range(H):
        want_v = (np.float32(x["v_scale"][h]) * vals[h].astype(np.float32)).astype(np.float32)   # one fp32 product
        for g in range(0, G, 17):
            got = out[g, h]
            # the value row times an fp32 scale, then the row-scaled fp16 staging of the partial (2^-11 of the row maximum)
            assert np.abs(got - want_v).max() <= np.abs(want_v).max() * 2.0 ** -11, (where, algo, h, g)
            if x["v_scale"][h] in (1.0, 2.0):
                assert np.array_equal(got, want_v), (where, algo, h, g)
        want_l = scale * float(x["k_scale"][h]) * vals[h]
        assert np.abs(lse[:, h] - want_l).max() <= 1e-5, (where, algo, h)
    # the oracle says the same
    ro, rl = util.oracle(x, scale, G)
    util.compare(torch.from_numpy(out), torch.from_numpy(lse), ro, rl, "bf16", f"bytes {where} {algo}")


CASES = [
    # P, G, Hq, Hkv, d, Lp_cap, Ls_cap
    (3, 8, 28, 4, 128, 200, 300),      # r = 7, R = 56
    (2, 8, 16, 2, 128, 131, 257),      # R = 64
    (2, 16, 16, 2, 128, 97, 65),       # R = 128: two row parts
    (2, 5, 12, 4, 128, 64, 95),        # R = 15
    (3, 1, 8, 8, 128, 50, 40),         # G = 1, r = 1
    (1, 2, 32, 2, 128, 40, 33),        # r = 16
    (2, 4, 8, 2, 64, 77, 91),          # d = 64: simple kernel under AUTO
    (5, 7, 6, 3, 128, 31, 1),          # one-row suffix buffers
    (2, 32, 14, 2, 128, 150, 60),      # R = 224: four row parts
    (2, 2, 64, 2, 128, 60, 50),        # r = 32: outside the matrix-core path, simple kernel under AUTO
]


def kv8_case(seed, P, G, Hq, Hkv, d, Lp_cap, Ls_cap, **kw):
    return wl.kv_to_e4m3(util.random_case(seed, P, G, Hq, Hkv, d, Lp_cap, Ls_cap, "bf16", **kw))


@pytest.mark.parametrize("algo", ["auto", "simple"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "P{}G{}H{}-{}d{}Lp{}Ls{}".format(*c))
def test_reduced_sizes(case, algo, B):
    import torch
    P, G, Hq, Hkv, d, Lp_cap, Ls_cap = case
    x = kv8_case(300 + CASES.index(case), *case)
    t = util.to_device(x)
    scale = 1.0 / math.sqrt(d)
    ds = B.desc_from_tensors(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], t["k_suffix"], t["v_suffix"],
                             t["suffix_lens"], scale, G, torch.empty((P * G, Hq, d), device="cuda"), None, None,
                             ALGOS[algo], t["k_scale"], t["v_scale"])
    want = 1 if algo == "simple" or d != 128 or Hq // Hkv > 16 else 2
    assert B.rl_decode_attn_plan(ds) == want
    out, lse = util.gpu_run(t, scale, G, algo=ALGOS[algo])
    ro, rl = util.oracle(x, scale, G)
    util.compare(out, lse, ro, rl, "bf16", str(case))


def test_scales_may_be_null(B):
    x = kv8_case(7, 2, 4, 8, 2, 128, 90, 70)
    # rescale the bytes' meaning: without factors the stored values (up to 448) are the keys themselves
    x.pop("k_scale"); x.pop("v_scale")
    t = util.to_device(x)
    out, lse = util.gpu_run(t, 1e-3, 4)
    ro, rl = util.oracle(x, 1e-3, 4)
    o = out.cpu().numpy().astype(np.float64)
    # |v| reaches 448 here; the 1e-2 bar is derived for |v| <= 4 and every error term is linear in V
    assert np.abs(o - ro).max() <= 1e-2 * 448 / 4
    assert np.abs(lse.cpu().numpy() - rl).max() <= 1e-3


def test_empty_full_and_clamped_lengths_with_nan_padding(B):
    P, G, Hq, Hkv, d, Lp_cap, Ls_cap = 3, 4, 8, 2, 128, 70, 45
    B_ = P * G
    sl = np.array([0, 45, 1, 32, 33, 0, 999, -4, 31, 45, 2, 44], np.int32)
    x = kv8_case(11, P, G, Hq, Hkv, d, Lp_cap, Ls_cap, plens=[0, 70, 1000], slens=sl)
    for b in range(B_):                                     # rows beyond the lengths hold NaN bytes
        x["k_suffix"][b, :, int(np.clip(sl[b], 0, Ls_cap)):] = 0x7F
        x["v_suffix"][b, :, int(np.clip(sl[b], 0, Ls_cap)):] = 0xFF
    x["k_prefix"][0] = 0x7F
    x["v_prefix"][0] = 0x7F
    for algo in ("auto", "simple"):
        t = util.to_device(x)
        out, lse = util.gpu_run(t, 0.09, G, algo=ALGOS[algo])
        ro, rl = util.oracle(x, 0.09, G)
        util.compare(out, lse, ro, rl, "bf16", algo)
    assert np.isneginf(rl[0]).all() and np.isfinite(rl[1]).all()        # sequence 0: no prefix, no suffix


@pytest.mark.parametrize("page_size", [32, 128])
def test_paged_store_with_finished_sequences(page_size, B):
    import torch
    P, G, Hq, Hkv, d = 3, 8, 28, 4, 128
    x = kv8_case(21, P, G, Hq, Hkv, d, 150, 400)
    y = wl.to_pages(x, page_size, seed=3)                   # NaN bytes in every row without a live key
    assert y["k_pages"].dtype == np.uint8 and (y["k_pages"] == 0x7F).any()
    act = (np.arange(P * G) % 3 != 1).astype(np.uint8)
    act[8:16] = 0                                           # a whole group finished: its prefix is skipped
    t = util.to_device(y)
    for a in (None, act):
        out, lse = util.gpu_run_paged(t, 0.088, G, active=None if a is None else torch.from_numpy(a).cuda())
        ro, rl = util.oracle_paged(y, 0.088, G, active=a)
        util.compare(out, lse, ro, rl, "bf16", f"paged {page_size} {a is not None}")


@pytest.mark.parametrize("G,Hq,Hkv", [(16, 16, 2), (32, 14, 2)])
def test_paged_store_with_several_row_parts(G, Hq, Hkv, B):
    """KV groups of 128 and 224 rows (two and four row parts) on a paged e4m3 store with finished sequences:
    the kernel variant that keeps the prefix tiles cached between the parts, in its extended e4m3 form."""
    import torch
    P, d = 3, 128
    x = kv8_case(23 + G, P, G, Hq, Hkv, d, 170, 260)
    y = wl.to_pages(x, 64, seed=5)
    act = (np.arange(P * G) % 4 != 2).astype(np.uint8)
    t = util.to_device(y)
    for a in (None, act):
        out, lse = util.gpu_run_paged(t, 0.088, G, active=None if a is None else torch.from_numpy(a).cuda())
        ro, rl = util.oracle_paged(y, 0.088, G, active=a)
        util.compare(out, lse, ro, rl, "bf16", f"paged G{G} {a is not None}")


def test_bitwise_determinism_and_store_independence(B):
    import torch
    x = kv8_case(31, 4, 8, 28, 4, 128, 300, 500)
    t = util.to_device(x)
    o1, l1 = util.gpu_run(t, 0.088, 8)
    o2, l2 = util.gpu_run(t, 0.088, 8)
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    # the same values held in a bf16 store (dequantised with power-of-two factors, hence exactly) give the same bits:
    # both stores feed identical bf16 tiles to the same arithmetic
    x2 = dict(x)
    ks = np.array([0.0078125, 0.015625, 0.0078125, 0.03125], np.float32)
    vs = np.array([0.015625, 0.0078125, 0.0078125, 0.0625], np.float32)
    x2["k_scale"], x2["v_scale"] = ks, vs
    t2 = util.to_device(x2)
    o8, l8 = util.gpu_run(t2, 0.088, 8)
    y = {k: v for k, v in x2.items() if k not in ("k_scale", "v_scale")}
    for name, sc in (("k", ks), ("v", vs)):
        for st in ("prefix", "suffix"):
            f = (ref.e4m3_to_f64(np.where((x[f"{name}_{st}"] & 0x7F) == 0x7F, 0, x[f"{name}_{st}"])) *
                 sc[None, :, None, None]).astype(np.float32)
            y[f"{name}_{st}"] = wl.f32_to_bf16_bits(f)
            assert np.array_equal(wl.bf16_bits_to_f32(y[f"{name}_{st}"]), f)       # exact in bf16
    ty = util.to_device(y)
    ob, lb = util.gpu_run(ty, 0.088, 8)
    ro, rl = util.oracle(x2, 0.088, 8)
    util.compare(o8, l8, ro, rl, "bf16", "kv8 pow2")
    do = np.abs(o8.cpu().numpy() - ob.cpu().numpy()).max()
    dl = np.abs(l8.cpu().numpy() - lb.cpu().numpy()).max()
    print(f"\ne4m3 store vs bf16 store of the same values: max |d out| {do:.2e}, max |d lse| {dl:.2e}")
    assert torch.equal(o8, ob) and torch.equal(l8, lb), (do, dl)      # bit for bit


def test_vlm7b_full_size_on_sampled_rows(B):
    import torch
    w = wl.WORKLOADS["vlm7b"]
    x = wl.kv_to_e4m3(wl.make_inputs(w))
    t = util.to_device(x)
    out, lse = util.gpu_run(t, w.scale, w.G)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    rows = np.stack([rng.integers(0, w.B, 300), rng.integers(0, w.Hq, 300)], 1).astype(np.int32)
    ro, rl = util.oracle(x, w.scale, w.G, rows=rows)
    o, l = out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(o).all() and np.isfinite(l).all()
    eo = max(np.abs(o[b, h] - ro[b, h]).max() for b, h in rows)
    el = max(abs(l[b, h] - rl[b, h]) for b, h in rows)
    print(f"\nvlm7b e4m3 store: max|out err| {eo:.2e}  max|lse err| {el:.2e}")
    assert eo <= 1e-2 and el <= 1e-3
