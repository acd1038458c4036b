"""Pins for the paged-suffix form of the oracle (no GPU).

The paged call is defined as the contiguous one on the gathered suffix, so the
pins are: a brute force that walks the block table key by key (no gather),
agreement with the contiguous oracle on layouts produced by an independently
written scatter, the inverse property gather(scatter(x)) = x, and the
finished-sequence rule.
"""
import math

import numpy as np
import pytest

from oracle import ref
from paper_2512_21450_amd import workloads as wl
from tests.test_oracle_pins import as_f64, rand_case


def paged(y, scale, G, active=None, **kw):
    return ref.decode_attn_paged_ref(y["q"], y["k_prefix"], y["v_prefix"], y["prefix_lens"], y["k_pages"],
                                     y["v_pages"], y["block_table"], y["suffix_lens"], active, scale, G, **kw)


def brute_force_paged(y, scale, G, active=None):
    """Python loops straight through the block table: key n -> page table[b][n // ps], row n % ps."""
    q, kp, vp, kpg, vpg = (as_f64(y[k]).tolist() for k in ("q", "k_prefix", "v_prefix", "k_pages", "v_pages"))
    B, Hq, d = y["q"].shape
    Hkv, ps = y["k_pages"].shape[1], y["k_pages"].shape[2]
    tab = y["block_table"].tolist()
    out = np.zeros((B, Hq, d))
    lse = np.full((B, Hq), -math.inf)
    for b in range(B):
        if active is not None and not active[b]:
            continue
        p = b // G
        for h in range(Hq):
            j = h // (Hq // Hkv)
            keys, vals = [], []
            for n in range(int(y["prefix_lens"][p])):
                keys.append(kp[p][j][n]); vals.append(vp[p][j][n])
            for n in range(int(y["suffix_lens"][b])):
                pg = tab[b][n // ps]
                keys.append(kpg[pg][j][n % ps]); vals.append(vpg[pg][j][n % ps])
            if not keys:
                continue
            s = [scale * sum(a * c for a, c in zip(q[b][h], k)) for k in keys]
            m = max(s)
            z = sum(math.exp(v - m) for v in s)
            lse[b, h] = m + math.log(z)
            for c in range(d):
                out[b, h, c] = sum(math.exp(sv - m) / z * v[c] for sv, v in zip(s, vals))
    return out, lse


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("ps", [2, 4])
def test_brute_force_through_the_block_table(dtype, ps):
    x = rand_case(11, P=2, G=2, Hq=4, Hkv=2, d=8, Lp_cap=5, Ls_cap=9, dtype=dtype, slens=[9, 0, 4, 5])
    y = wl.to_pages(x, ps, seed=3)
    o, l = paged(y, 0.3, 2)
    bo, bl = brute_force_paged(y, 0.3, 2)
    assert np.abs(o - bo).max() < 1e-12
    assert np.array_equal(np.isneginf(l), np.isneginf(bl))
    fin = np.isfinite(bl)
    assert np.abs(l[fin] - bl[fin]).max() < 1e-12


@pytest.mark.parametrize("ps,seed", [(32, 1), (64, 2), (128, 3)])
def test_paged_equals_contiguous_on_a_shuffled_pool(ps, seed):
    w = wl.scaled(wl.WORKLOADS["vlm3b"], P=2)
    x = wl.make_inputs(w)
    y = wl.to_pages(x, ps, seed=seed)
    assert sorted(y["block_table"][y["block_table"] >= 0].tolist()) == sorted(set(y["block_table"][y["block_table"] >= 0].tolist()))
    o1, l1 = ref.decode_attn_ref(x["q"], x["k_prefix"], x["v_prefix"], x["prefix_lens"], x["k_suffix"],
                                 x["v_suffix"], x["suffix_lens"], w.scale, w.G)
    o2, l2 = paged(y, w.scale, w.G)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_gather_inverts_scatter_and_zeroes_the_rest():
    x = rand_case(5, P=1, G=3, Hq=2, Hkv=2, d=4, Lp_cap=3, Ls_cap=21, dtype="f32", slens=[21, 7, 0])
    y = wl.to_pages(x, 4, seed=9)
    g = ref.gather_pages(y["k_pages"], y["block_table"], y["suffix_lens"], 21)
    for b, L in enumerate([21, 7, 0]):
        assert np.array_equal(g[b, :, :L], x["k_suffix"][b, :, :L])
        assert not g[b, :, L:].any()


def test_table_order_matters_only_through_the_layout():
    # two full pages swapped in the table AND in the pool leave the result unchanged; swapped in the
    # table alone they permute the keys, which attention does not see either (full pages); but a
    # table that names a wrong page changes the result
    x = rand_case(6, P=1, G=1, Hq=2, Hkv=1, d=4, Lp_cap=2, Ls_cap=12, dtype="f32", slens=[12])
    y = wl.to_pages(x, 4, seed=1, spare_pages=2, poison=False)
    o0, l0 = paged(y, 0.5, 1)
    z = dict(y); t = y["block_table"].copy(); t[0, 0], t[0, 1] = t[0, 1], t[0, 0]; z["block_table"] = t
    o1, l1 = paged(z, 0.5, 1)
    assert np.abs(o1 - o0).max() < 1e-12 and np.abs(l1 - l0).max() < 1e-12
    used = set(y["block_table"][0].tolist())
    spare = [p for p in range(y["k_pages"].shape[0]) if p not in used][0]
    y["k_pages"][spare] = 1.0
    t2 = y["block_table"].copy(); t2[0, 2] = spare; z["block_table"] = t2
    o2, _ = paged(z, 0.5, 1)
    assert np.abs(o2 - o0).max() > 1e-3


def test_finished_sequences_give_zero_and_minus_infinity_and_leave_the_others_alone():
    x = rand_case(8, P=2, G=2, Hq=4, Hkv=2, d=8, Lp_cap=6, Ls_cap=8, dtype="bf16", plens=[6, 3], slens=[8, 3, 0, 5])
    y = wl.to_pages(x, 4, seed=2)
    o_all, l_all = paged(y, 0.25, 2)
    act = np.array([1, 0, 0, 1], dtype=np.uint8)
    o, l = paged(y, 0.25, 2, active=act)
    assert not o[1].any() and not o[2].any()
    assert np.isneginf(l[1]).all() and np.isneginf(l[2]).all()
    assert np.array_equal(o[[0, 3]], o_all[[0, 3]]) and np.array_equal(l[[0, 3]], l_all[[0, 3]])
    bo, bl = brute_force_paged(y, 0.25, 2, active=act)
    assert np.abs(o - bo).max() < 1e-12


def test_lengths_are_clamped_to_the_table_capacity():
    x = rand_case(9, P=1, G=2, Hq=2, Hkv=1, d=4, Lp_cap=2, Ls_cap=8, dtype="f32", slens=[8, 5])
    y = wl.to_pages(x, 4, seed=4, poison=False)
    o0, l0 = paged(y, 1.0, 2)
    z = dict(y); z["suffix_lens"] = np.array([1000, 5], dtype=np.int32)
    o1, l1 = paged(z, 1.0, 2)
    assert np.array_equal(o0, o1) and np.array_equal(l0, l1)
    z["suffix_lens"] = np.array([-3, 5], dtype=np.int32)
    w = dict(y); w["suffix_lens"] = np.array([0, 5], dtype=np.int32)
    assert np.array_equal(paged(z, 1.0, 2)[0], paged(w, 1.0, 2)[0])
