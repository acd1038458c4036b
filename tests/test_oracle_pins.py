"""Pins for the fp64 CPU oracle (no GPU).

The paper prints no worked numerical example of decode attention, so the
oracle is pinned to what the mathematics fixes: a pure-Python brute force,
closed forms, structural identities, and torch's CPU fp64 softmax routines.
Each check is chosen so that a plausible slip in the C code (wrong KV-head or
prompt index, scale in the wrong place, log base, a dropped prefix/suffix
term, a transposed operand, reading past a length) fails at least one of them.
"""
import math

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2512_21450_amd import workloads as wl


def rand_case(seed, P=2, G=3, Hq=4, Hkv=2, d=8, Lp_cap=7, Ls_cap=6, dtype="f32",
              plens=None, slens=None):
    rng = np.random.default_rng(seed)
    B = P * G

    def t(shape):
        x = rng.standard_normal(shape).astype(np.float32)
        return x if dtype == "f32" else wl.f32_to_bf16_bits(x)

    x = dict(q=t((B, Hq, d)), k_prefix=t((P, Hkv, Lp_cap, d)), v_prefix=t((P, Hkv, Lp_cap, d)),
             k_suffix=t((B, Hkv, Ls_cap, d)), v_suffix=t((B, Hkv, Ls_cap, d)))
    x["prefix_lens"] = (rng.integers(0, Lp_cap + 1, P) if plens is None else np.asarray(plens)).astype(np.int32)
    x["suffix_lens"] = (rng.integers(0, Ls_cap + 1, B) if slens is None else np.asarray(slens)).astype(np.int32)
    x["G"] = G
    return x


def run(x, scale, **kw):
    return ref.decode_attn_ref(x["q"], x["k_prefix"], x["v_prefix"], x["prefix_lens"],
                               x["k_suffix"], x["v_suffix"], x["suffix_lens"], scale, x["G"], **kw)


def as_f64(a):
    return (wl.bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64)


# ---------------------------------------------------------------- brute force
def brute_force(x, scale):
    """Pure-Python loops over Python floats, straight from the definition."""
    q, kp, vp, ks, vs = (as_f64(x[k]).tolist() for k in ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix"))
    B, Hq, d = x["q"].shape
    Hkv = x["k_prefix"].shape[1]
    G = x["G"]
    out = [[[0.0] * d for _ in range(Hq)] for _ in range(B)]
    lse = [[-math.inf] * Hq for _ in range(B)]
    for b in range(B):
        p = b // G
        for h in range(Hq):
            j = h // (Hq // Hkv)
            keys = [kp[p][j][n] for n in range(int(x["prefix_lens"][p]))] + \
                   [ks[b][j][n] for n in range(int(x["suffix_lens"][b]))]
            vals = [vp[p][j][n] for n in range(int(x["prefix_lens"][p]))] + \
                   [vs[b][j][n] for n in range(int(x["suffix_lens"][b]))]
            if not keys:
                continue
            s = [scale * sum(qc * kc for qc, kc in zip(q[b][h], k)) for k in keys]
            z = sum(math.exp(v) for v in s)          # small scores: no max shift needed
            lse[b][h] = math.log(z)
            for n, v in enumerate(vals):
                wgt = math.exp(s[n]) / z
                for c in range(d):
                    out[b][h][c] += wgt * v[c]
    return np.array(out), np.array(lse)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_tiny(seed, dtype):
    x = rand_case(seed, dtype=dtype)
    out, lse = run(x, 0.37)
    bo, bl = brute_force(x, 0.37)
    np.testing.assert_allclose(out, bo, rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse, bl, rtol=0, atol=1e-13)


def test_brute_force_one_to_three_keys_small_d():
    for d in (1, 2, 4):
        for n in (1, 2, 3):
            x = rand_case(10 * d + n, P=1, G=2, Hq=2, Hkv=1, d=d, Lp_cap=n, Ls_cap=2,
                          plens=[n], slens=[0, 2])
            out, lse = run(x, 1.3)
            bo, bl = brute_force(x, 1.3)
            np.testing.assert_allclose(out, bo, rtol=0, atol=1e-14)
            np.testing.assert_allclose(lse, bl, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- closed forms
def test_bf16_widening_exact():
    # 0x3F80 = 1.0, 0xC000 = -2.0, 0x3FC0 = 1.5, 0x4049 = 3.140625
    x = rand_case(3, P=1, G=1, Hq=1, Hkv=1, d=4, Lp_cap=1, Ls_cap=1, dtype="bf16", plens=[1], slens=[0])
    x["q"][...] = np.array([0x3F80, 0xC000, 0x3FC0, 0x4049], dtype=np.uint16)
    x["k_prefix"][...] = np.array([0x3F80, 0x3F80, 0x3F80, 0x3F80], dtype=np.uint16)
    x["v_prefix"][...] = np.array([0x4049, 0x3FC0, 0xC000, 0x3F80], dtype=np.uint16)
    out, lse = run(x, 2.0)
    assert lse[0, 0] == 2.0 * (1.0 - 2.0 + 1.5 + 3.140625)   # one key: lse = its score
    np.testing.assert_array_equal(out[0, 0], [3.140625, 1.5, -2.0, 1.0])


def test_single_key_gives_its_value_and_score():
    x = rand_case(4, plens=[1, 0], slens=[0, 0, 0, 1, 1, 1])
    out, lse = run(x, 0.5)
    q, kp, vp, ks, vs = (as_f64(x[k]) for k in ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix"))
    for b in range(6):
        for h in range(4):
            j = h // 2
            k, v = (kp[0, j, 0], vp[0, j, 0]) if b < 3 else (ks[b, j, 0], vs[b, j, 0])
            assert lse[b, h] == pytest.approx(0.5 * float(q[b, h] @ k), abs=1e-14)
            np.testing.assert_allclose(out[b, h], v, atol=1e-15)


def test_constant_v_returns_v():
    x = rand_case(5, dtype="bf16")
    c = wl.f32_to_bf16_bits(np.linspace(-2, 2, 8).astype(np.float32))
    x["v_prefix"][...] = c
    x["v_suffix"][...] = c
    x["prefix_lens"][:] = [3, 5]
    out, _ = run(x, 0.9)
    np.testing.assert_allclose(out, np.broadcast_to(as_f64(c), out.shape), atol=1e-14)


def test_zero_query_gives_mean_and_log_count():
    x = rand_case(6)
    x["q"][...] = 0
    out, lse = run(x, 0.7)
    vp, vs = as_f64(x["v_prefix"]), as_f64(x["v_suffix"])
    for b in range(6):
        p, Lp, Ls = b // 3, int(x["prefix_lens"][b // 3]), int(x["suffix_lens"][b])
        for h in range(4):
            j = h // 2
            if Lp + Ls == 0:
                assert lse[b, h] == -math.inf and not out[b, h].any()
                continue
            vals = np.concatenate([vp[p, j, :Lp], vs[b, j, :Ls]])
            assert lse[b, h] == pytest.approx(math.log(Lp + Ls), abs=1e-14)   # natural log
            np.testing.assert_allclose(out[b, h], vals.mean(0), atol=1e-14)


def test_identical_keys_and_duplicated_key_set():
    x = rand_case(7, P=1, G=1, Hq=2, Hkv=1, d=8, Lp_cap=5, Ls_cap=5, plens=[5], slens=[5])
    base_out, base_lse = run(x, 0.6)
    # duplicate the prefix keys into the suffix: out unchanged vs prefix-only, lse grows by ln 2
    x2 = dict(x)
    x2["k_suffix"] = x["k_prefix"].copy()
    x2["v_suffix"] = x["v_prefix"].copy()
    dup_out, dup_lse = run(x2, 0.6)
    x3 = dict(x, suffix_lens=np.array([0], dtype=np.int32))
    p_out, p_lse = run(x3, 0.6)
    np.testing.assert_allclose(dup_out, p_out, atol=1e-14)
    np.testing.assert_allclose(dup_lse, p_lse + math.log(2.0), atol=1e-14)
    assert np.abs(base_out - p_out).max() > 1e-3
    # all keys identical: out = mean(V), lse = s + ln n
    x4 = dict(x)
    x4["k_prefix"] = np.broadcast_to(x["k_prefix"][:, :, :1], x["k_prefix"].shape).copy()
    x4["k_suffix"] = np.broadcast_to(x["k_prefix"][:, :, :1], x["k_suffix"].shape).copy()
    o4, l4 = run(x4, 0.6)
    vals = np.concatenate([x["v_prefix"][0, 0], x["v_suffix"][0, 0]]).astype(np.float64)
    for h in range(2):
        s = 0.6 * float(x["q"][0, h].astype(np.float64) @ x["k_prefix"][0, 0, 0].astype(np.float64))
        assert l4[0, h] == pytest.approx(s + math.log(10), abs=1e-13)
        np.testing.assert_allclose(o4[0, h], vals.mean(0), atol=1e-14)


def test_large_scores_do_not_overflow():
    x = rand_case(8, P=1, G=1, Hq=1, Hkv=1, d=4, Lp_cap=2, Ls_cap=1, plens=[2], slens=[0])
    x["q"][...] = 100.0
    x["k_prefix"][0, 0, 0] = 10.0
    x["k_prefix"][0, 0, 1] = 10.0
    out, lse = run(x, 1.0)
    assert lse[0, 0] == pytest.approx(4000.0 + math.log(2.0), abs=1e-9)
    np.testing.assert_allclose(out[0, 0], as_f64(x["v_prefix"])[0, 0, :2].mean(0), atol=1e-14)


# ---------------------------------------------------------------- structure
def test_empty_suffix_empty_prefix_empty_both():
    x = rand_case(9, plens=[4, 0], slens=[0, 3, 6, 0, 2, 0])
    out, lse = run(x, 0.8)
    bo, bl = brute_force(x, 0.8)
    np.testing.assert_allclose(out, bo, atol=1e-13)
    np.testing.assert_allclose(lse, bl, atol=1e-13)
    # sequences 3 and 5 have no key at all
    for b in (3, 5):
        assert np.all(lse[b] == -math.inf) and not out[b].any() and not np.isnan(out[b]).any()
    # prefix-only (b=0) does not depend on the suffix buffers
    x2 = dict(x, k_suffix=x["k_suffix"] * 0 + 7, v_suffix=x["v_suffix"] * 0 - 3)
    o2, l2 = run(x2, 0.8)
    np.testing.assert_array_equal(o2[0], out[0])
    np.testing.assert_array_equal(l2[0], lse[0])


def test_lse_merge_of_prefix_and_suffix_equals_concatenation():
    x = rand_case(11, dtype="bf16", plens=[7, 2], slens=[6, 0, 3, 1, 5, 2])
    full_o, full_l = run(x, 0.45)
    po, pl = run(dict(x, suffix_lens=np.zeros(6, np.int32)), 0.45)
    so, sl = run(dict(x, prefix_lens=np.zeros(2, np.int32)), 0.45)
    for b in range(6):
        for h in range(4):
            o, l = ref.lse_combine_ref(np.stack([po[b, h], so[b, h]]), [pl[b, h], sl[b, h]])
            np.testing.assert_allclose(o, full_o[b, h], atol=1e-14)
            assert l == pytest.approx(full_l[b, h], abs=1e-14)


def test_lse_combine_closed_forms():
    o = np.array([[1.0, 2.0], [3.0, -4.0], [10.0, 10.0]])
    # weights proportional to exp(lse_i): ln1, ln3 -> 1/4, 3/4 ; third part empty
    out, l = ref.lse_combine_ref(o, [0.0, math.log(3.0), -math.inf])
    np.testing.assert_allclose(out, 0.25 * o[0] + 0.75 * o[1], atol=1e-15)
    assert l == pytest.approx(math.log(4.0), abs=1e-15)
    out, l = ref.lse_combine_ref(o, [-math.inf] * 3)
    assert l == -math.inf and not out.any()
    out, l = ref.lse_combine_ref(o[:1], [5.5])
    np.testing.assert_array_equal(out, o[0])
    assert l == 5.5
    # shift invariance, large magnitudes
    out, l = ref.lse_combine_ref(o[:2], [1000.0, 1000.0 + math.log(3.0)])
    np.testing.assert_allclose(out, 0.25 * o[0] + 0.75 * o[1], atol=1e-12)
    assert l == pytest.approx(1000.0 + math.log(4.0), abs=1e-12)


def test_key_permutation_invariance_within_and_across_boundary():
    x = rand_case(12, P=1, G=2, Hq=4, Hkv=2, d=8, Lp_cap=6, Ls_cap=6, plens=[6], slens=[6, 6])
    out, lse = run(x, 0.5)
    rng = np.random.default_rng(0)
    perm = rng.permutation(6)
    xp = dict(x, k_prefix=x["k_prefix"][:, :, perm], v_prefix=x["v_prefix"][:, :, perm],
              k_suffix=x["k_suffix"][:, :, perm[::-1]], v_suffix=x["v_suffix"][:, :, perm[::-1]])
    o2, l2 = run(xp, 0.5)
    np.testing.assert_allclose(o2, out, atol=1e-14)
    np.testing.assert_allclose(l2, lse, atol=1e-14)
    # across the boundary (G = 1 so that the prefix belongs to one sequence only):
    # exchange prefix rows 0..2 with suffix rows 0..2
    y = rand_case(13, P=2, G=1, Hq=4, Hkv=2, d=8, Lp_cap=6, Ls_cap=6, plens=[6, 5], slens=[6, 4])
    o, l = run(y, 0.5)
    y2 = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in y.items()}
    for a, bname in (("k_prefix", "k_suffix"), ("v_prefix", "v_suffix")):
        y2[a][:, :, :3] = y[bname][:, :, :3]
        y2[bname][:, :, :3] = y[a][:, :, :3]
    o2, l2 = run(y2, 0.5)
    np.testing.assert_allclose(o2, o, atol=1e-14)
    np.testing.assert_allclose(l2, l, atol=1e-14)


def test_replicated_prefix_equals_shared_prefix():
    x = rand_case(14, P=2, G=3, Hq=4, Hkv=2, d=8, Lp_cap=5, Ls_cap=4, plens=[5, 3])
    out, lse = run(x, 0.6)
    # physically copy each prompt's prefix in front of every sequence's own keys
    B, Hkv, d = 6, 2, 8
    ks = np.zeros((B, Hkv, 9, d), np.float32)
    vs = np.zeros_like(ks)
    sl = np.zeros(B, np.int32)
    for b in range(B):
        p, Lp, Ls = b // 3, int(x["prefix_lens"][b // 3]), int(x["suffix_lens"][b])
        ks[b, :, :Lp] = x["k_prefix"][p, :, :Lp]
        vs[b, :, :Lp] = x["v_prefix"][p, :, :Lp]
        ks[b, :, Lp:Lp + Ls] = x["k_suffix"][b, :, :Ls]
        vs[b, :, Lp:Lp + Ls] = x["v_suffix"][b, :, :Ls]
        sl[b] = Lp + Ls
    y = dict(x, k_suffix=ks, v_suffix=vs, suffix_lens=sl, prefix_lens=np.zeros(2, np.int32))
    o2, l2 = run(y, 0.6)
    np.testing.assert_allclose(o2, out, atol=1e-14)
    np.testing.assert_allclose(l2, lse, atol=1e-14)


def test_gqa_head_blocks_and_kv_head_swap():
    x = rand_case(15, P=1, G=2, Hq=6, Hkv=2, d=8, Lp_cap=5, Ls_cap=4, plens=[5], slens=[4, 2])
    # identical queries in all heads: outputs equal inside a KV block, differ across blocks
    x["q"][:] = x["q"][:, :1]
    out, lse = run(x, 0.5)
    for h in (1, 2):
        np.testing.assert_array_equal(out[:, h], out[:, 0])
    for h in (4, 5):
        np.testing.assert_array_equal(out[:, h], out[:, 3])
    assert np.abs(out[:, 0] - out[:, 3]).max() > 1e-3
    # swapping the two KV heads' data swaps the two output blocks
    sw = {k: x[k][:, ::-1].copy() for k in ("k_prefix", "v_prefix", "k_suffix", "v_suffix")}
    o2, l2 = run(dict(x, **sw), 0.5)
    np.testing.assert_array_equal(o2[:, :3], out[:, 3:])
    np.testing.assert_array_equal(o2[:, 3:], out[:, :3])
    np.testing.assert_array_equal(l2[:, :3], lse[:, 3:])


def test_rows_beyond_length_are_never_read_and_lengths_are_clamped():
    x = rand_case(16, plens=[4, 2], slens=[3, 0, 6, 1, 2, 5])
    out, lse = run(x, 0.5)
    y = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in x.items()}
    for p in range(2):
        y["k_prefix"][p, :, x["prefix_lens"][p]:] = np.nan
        y["v_prefix"][p, :, x["prefix_lens"][p]:] = np.nan
    for b in range(6):
        y["k_suffix"][b, :, x["suffix_lens"][b]:] = np.nan
        y["v_suffix"][b, :, x["suffix_lens"][b]:] = np.nan
    o2, l2 = run(y, 0.5)
    np.testing.assert_array_equal(o2, out)
    np.testing.assert_array_equal(l2, lse)
    # out-of-range lengths clamp to [0, cap]
    z = dict(x, prefix_lens=np.array([100, -5], np.int32), suffix_lens=np.array([-1, 99, 6, 0, 7, 6], np.int32))
    zc = dict(x, prefix_lens=np.array([7, 0], np.int32), suffix_lens=np.array([0, 6, 6, 0, 6, 6], np.int32))
    o3, l3 = run(z, 0.5)
    o4, l4 = run(zc, 0.5)
    np.testing.assert_array_equal(o3, o4)
    np.testing.assert_array_equal(l3, l4)


def test_row_subset_and_thread_count_do_not_change_values():
    x = rand_case(17, P=3, G=2, Hq=4, Hkv=2, d=16, Lp_cap=9, Ls_cap=11, dtype="bf16")
    out, lse = run(x, 0.3, n_threads=1)
    o8, l8, used = run(x, 0.3, n_threads=4, return_threads=True)
    assert used >= 1
    np.testing.assert_array_equal(o8, out)
    np.testing.assert_array_equal(l8, lse)
    rows = np.array([[5, 3], [0, 0], [2, 1]], np.int32)
    orr, lr = run(x, 0.3, rows=rows)
    for b, h in rows:
        np.testing.assert_array_equal(orr[b, h], out[b, h])
        assert lr[b, h] == lse[b, h]
    assert np.isnan(orr[1, 1]).all()
    # a row listed several times is computed several times, with the same result
    dup = np.array([[5, 3]] * 6 + [[0, 0]] * 6, np.int32)
    od, ld = run(x, 0.3, rows=dup, n_threads=4)
    np.testing.assert_array_equal(od[5, 3], out[5, 3])
    np.testing.assert_array_equal(od[0, 0], out[0, 0])


def test_invalid_arguments_rejected():
    x = rand_case(18)
    with pytest.raises(ValueError):
        run(x, 0.5, rows=np.array([[99, 0]], np.int32))
    bad = dict(x, q=x["q"][:, :3].copy())       # Hq=3 not divisible by Hkv=2
    with pytest.raises(ValueError):
        run(bad, 0.5)


# ---------------------------------------------------------------- library cross-check
def torch_reference(x, scale):
    """torch CPU fp64: repeat K/V per query head and per sample, mask by length."""
    q = torch.from_numpy(as_f64(x["q"]))
    B, Hq, d = q.shape
    P, Hkv, Lp_cap, _ = x["k_prefix"].shape
    Ls_cap = x["k_suffix"].shape[2]
    G, r = x["G"], Hq // Hkv
    kp, vp, ks, vs = (torch.from_numpy(as_f64(x[k])) for k in ("k_prefix", "v_prefix", "k_suffix", "v_suffix"))
    k = torch.cat([kp.repeat_interleave(G, 0), ks], 2).repeat_interleave(r, 1)   # [B,Hq,L,d]
    v = torch.cat([vp.repeat_interleave(G, 0), vs], 2).repeat_interleave(r, 1)
    pl = torch.from_numpy(x["prefix_lens"].astype(np.int64)).repeat_interleave(G)
    sl = torch.from_numpy(x["suffix_lens"].astype(np.int64))
    pos = torch.arange(Lp_cap + Ls_cap)
    valid = torch.where(pos[None] < Lp_cap, pos[None] < pl[:, None], (pos[None] - Lp_cap) < sl[:, None])
    mask = valid[:, None, None, :]                                               # [B,1,1,L]
    out = torch.nn.functional.scaled_dot_product_attention(q[:, :, None], k, v, attn_mask=mask, scale=scale)
    s = scale * torch.einsum("bhd,bhld->bhl", q, k)
    s = s.masked_fill(~valid[:, None, :], -math.inf)
    return out[:, :, 0].numpy(), torch.logsumexp(s, -1).numpy()


@pytest.mark.parametrize("name,shrink", [
    ("tiny", {}),
    ("vlm3b", dict(P=2, G=3, Lp_cap=37, Ls_cap=29, prefix=("const", 37), suffix=("uniform", 29))),
    ("vlm7b", dict(P=2, G=2, Lp_cap=40, Ls_cap=50, prefix=("const", 40), suffix=("uniform", 50))),
    ("agentic", dict(P=2, G=2, Lp_cap=60, Ls_cap=80, prefix=("agentic", 3, 8, 2, 12), suffix=("lognormal", 20.0, 1.0))),
    ("highbatch", dict(P=3, G=4, Lp_cap=33, Ls_cap=40, prefix=("const", 33), suffix=("lognormal", 10.0, 1.0))),
])
def test_against_torch_fp64_on_every_config_shape(name, shrink):
    w = wl.scaled(wl.WORKLOADS[name], **shrink)
    x = wl.make_inputs(w)
    x["G"] = w.G
    # keep at least one key everywhere: SDPA with a fully masked row is NaN by definition
    x["suffix_lens"] = np.maximum(x["suffix_lens"], 1).astype(np.int32)
    out, lse = run(x, w.scale)
    to, tl = torch_reference(x, w.scale)
    np.testing.assert_allclose(out, to, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, tl, rtol=0, atol=1e-12)


def test_golden_tiny_regression():
    """The stored file was written by tests/golden/make_golden.py from the oracle."""
    import os
    w = wl.WORKLOADS["tiny"]
    x = wl.make_inputs(w)
    x["G"] = w.G
    out, lse = run(x, w.scale)
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "tiny_oracle.txt")
    rows = [l.split() for l in open(path) if not l.startswith("#")]
    assert len(rows) == w.B * w.Hq
    for r in rows:
        b, h = int(r[0]), int(r[1])
        assert lse[b, h] == pytest.approx(float(r[2]), abs=1e-13)
        for c, v in zip((0, 21, 42, 63), r[3:]):
            assert out[b, h, c] == pytest.approx(float(v), abs=1e-13)
