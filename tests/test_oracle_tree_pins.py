"""Pins of the prefix-tree oracle (CPU only): the attention of a sequence over the segments it shares
on every level of the tree plus its own suffix is, by definition, the attention over the concatenated
keys.  What is new next to the decode oracle is the concatenation helper, so that is what is pinned:
against a pure-Python walk over every key of every level, against the single-level oracle, and through
identities a wrong segment map, a wrong order of copies or a wrong length would break."""
import math

import numpy as np
import pytest

from oracle import ref
from paper_2512_21450_amd import workloads as wl


def make_tree(rng, B, Hq, Hkv, d, groups, caps, Ls_cap, dtype="f32", empty=0.2):
    def t(shape):
        v = rng.standard_normal(shape).astype(np.float32)
        return v if dtype == "f32" else wl.f32_to_bf16_bits(v)
    levels = []
    for g, cap in zip(groups, caps):
        n = B // g
        lens = rng.integers(0, cap + 1, n) * (rng.random(n) >= empty)
        levels.append((t((n, Hkv, cap, d)), t((n, Hkv, cap, d)), lens.astype(np.int32), g))
    x = dict(q=t((B, Hq, d)), k_suffix=t((B, Hkv, Ls_cap, d)), v_suffix=t((B, Hkv, Ls_cap, d)),
             suffix_lens=(rng.integers(0, Ls_cap + 1, B) * (rng.random(B) >= empty)).astype(np.int32))
    return levels, x


def brute(q, levels, ks, vs, sl, scale):
    """every (b, h): walk the levels in order, key by key, in Python floats"""
    B, Hq, d = q.shape
    Hkv = ks.shape[1]
    r = Hq // Hkv
    out = np.zeros((B, Hq, d)); lse = np.full((B, Hq), -np.inf)
    for b in range(B):
        for h in range(Hq):
            j = h // r
            keys, vals = [], []
            for k, v, lens, group in levels:
                s = b // group
                for n in range(int(lens[s])):
                    keys.append(k[s, j, n]); vals.append(v[s, j, n])
            for n in range(int(sl[b])):
                keys.append(ks[b, j, n]); vals.append(vs[b, j, n])
            if not keys:
                continue
            sc = [scale * sum(float(a) * float(c) for a, c in zip(q[b, h], kk)) for kk in keys]
            m = max(sc)
            z = sum(math.exp(s_ - m) for s_ in sc)
            lse[b, h] = m + math.log(z)
            for s_, vv in zip(sc, vals):
                wgt = math.exp(s_ - lse[b, h])
                for c in range(d):
                    out[b, h, c] += wgt * float(vv[c])
    return out, lse


@pytest.mark.parametrize("groups", [(4,), (4, 2), (8, 4, 2), (4, 1), (2, 4)])
def test_tree_oracle_against_a_python_walk(groups):
    rng = np.random.default_rng(len(groups) * 7 + groups[0])
    levels, x = make_tree(rng, 8, 4, 2, 3, groups, [5, 4, 3][:len(groups)], 4)
    o, l = ref.decode_attn_tree_ref(x["q"], levels, x["k_suffix"], x["v_suffix"], x["suffix_lens"], 0.7)
    bo, bl = brute(x["q"], levels, x["k_suffix"], x["v_suffix"], x["suffix_lens"], 0.7)
    assert np.array_equal(np.isneginf(l), np.isneginf(bl))
    fin = np.isfinite(bl)
    assert np.abs(o - bo).max() < 1e-12 and np.abs(l[fin] - bl[fin]).max() < 1e-12


def test_concatenation_helper_puts_the_rows_where_the_definition_says():
    rng = np.random.default_rng(3)
    B, Hkv, d = 6, 2, 2
    levels, _ = make_tree(rng, B, 2, Hkv, d, (6, 3, 2), (4, 3, 5), 2, empty=0.3)
    kc, vc, cl = ref.concat_levels(levels, B)
    assert kc.shape == (B, Hkv, 12, d)
    for b in range(B):
        pos = 0
        for k, v, lens, g in levels:
            s = b // g
            for n in range(int(lens[s])):
                assert np.array_equal(kc[b, :, pos], k[s, :, n]) and np.array_equal(vc[b, :, pos], v[s, :, n])
                pos += 1
        assert cl[b] == pos
        assert not kc[b, :, pos:].any() and not vc[b, :, pos:].any()


def test_one_level_is_the_shared_prefix_oracle_bit_for_bit():
    rng = np.random.default_rng(5)
    levels, x = make_tree(rng, 12, 6, 2, 8, (4,), (20,), 9, dtype="bf16")
    k, v, lens, g = levels[0]
    o1, l1 = ref.decode_attn_tree_ref(x["q"], levels, x["k_suffix"], x["v_suffix"], x["suffix_lens"], 0.3)
    o2, l2 = ref.decode_attn_ref(x["q"], k, v, lens, x["k_suffix"], x["v_suffix"], x["suffix_lens"], 0.3, g)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    # no shared level at all: the suffix alone
    o3, l3 = ref.decode_attn_tree_ref(x["q"], [], x["k_suffix"], x["v_suffix"], x["suffix_lens"], 0.3)
    o4, l4 = ref.decode_attn_ref(x["q"], k, v, np.zeros_like(lens), x["k_suffix"], x["v_suffix"], x["suffix_lens"], 0.3, g)
    assert np.array_equal(o3, o4) and np.array_equal(l3, l4)


def test_cutting_a_segment_into_two_levels_changes_nothing():
    # keys [0, a) of every prompt as level 0 and keys [a, L) as level 1 of the same groups: the same key list
    rng = np.random.default_rng(6)
    levels, x = make_tree(rng, 8, 4, 2, 4, (4,), (16,), 5, empty=0.0)
    k, v, lens, g = levels[0]
    a = 6
    first = (k[:, :, :a].copy(), v[:, :, :a].copy(), np.minimum(lens, a).astype(np.int32), g)
    second = (k[:, :, a:].copy(), v[:, :, a:].copy(), np.maximum(lens - a, 0).astype(np.int32), g)
    o1, l1 = ref.decode_attn_tree_ref(x["q"], [levels[0]], x["k_suffix"], x["v_suffix"], x["suffix_lens"], 0.5)
    o2, l2 = ref.decode_attn_tree_ref(x["q"], [first, second], x["k_suffix"], x["v_suffix"], x["suffix_lens"], 0.5)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_order_of_levels_and_sharing_width_only_matter_through_the_key_sets():
    rng = np.random.default_rng(7)
    levels, x = make_tree(rng, 8, 4, 2, 4, (8, 2), (7, 6), 5)
    args = (x["k_suffix"], x["v_suffix"], x["suffix_lens"], 0.4)
    o1, l1 = ref.decode_attn_tree_ref(x["q"], levels, *args)
    o2, l2 = ref.decode_attn_tree_ref(x["q"], levels[::-1], *args)          # softmax over a set: order is rounding only
    fin = np.isfinite(l1)
    assert np.abs(o1 - o2).max() < 1e-12 and np.abs(l1[fin] - l2[fin]).max() < 1e-12
    # a level shared by 2 is the same as that level replicated and "shared" by 1
    k, v, lens, g = levels[1]
    rep = (np.repeat(k, g, axis=0), np.repeat(v, g, axis=0), np.repeat(lens, g), 1)
    o3, l3 = ref.decode_attn_tree_ref(x["q"], [levels[0], rep], *args)
    assert np.array_equal(o1, o3) and np.array_equal(l1, l3)
    # a wrong segment map would show here: giving sequence b the segment of another group changes the result
    wrong = (k[::-1].copy(), v[::-1].copy(), lens[::-1].copy(), g)
    o4, _ = ref.decode_attn_tree_ref(x["q"], [levels[0], wrong], *args)
    assert np.abs(o1 - o4).max() > 1e-3


def test_lengths_clamp_and_rows_beyond_them_are_never_read():
    rng = np.random.default_rng(8)
    levels, x = make_tree(rng, 4, 2, 1, 4, (4, 2), (6, 5), 3, empty=0.0)
    k, v, lens, g = levels[1]
    k2, v2 = k.copy(), v.copy()
    for s in range(k.shape[0]):
        k2[s, :, int(lens[s]):] = np.nan
        v2[s, :, int(lens[s]):] = np.nan
    args = (x["k_suffix"], x["v_suffix"], x["suffix_lens"], 0.4)
    o1, l1 = ref.decode_attn_tree_ref(x["q"], levels, *args)
    o2, l2 = ref.decode_attn_tree_ref(x["q"], [levels[0], (k2, v2, lens, g)], *args)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    big = (levels[0][0], levels[0][1], np.full_like(levels[0][2], 99), levels[0][3])
    full = (levels[0][0], levels[0][1], np.full_like(levels[0][2], 6), levels[0][3])
    o3, l3 = ref.decode_attn_tree_ref(x["q"], [big, levels[1]], *args)
    o4, l4 = ref.decode_attn_tree_ref(x["q"], [full, levels[1]], *args)
    assert np.array_equal(o3, o4) and np.array_equal(l3, l4)
