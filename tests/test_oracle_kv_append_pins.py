"""Pins for the oracle of the decode-step state transition (RoPE + KV append), no GPU.

Pinned to what the rotary embedding's mathematics fixes: a pure-Python brute force with complex
multiplication (a rotation of the pair (x_i, x_{i+d/2}) is a multiplication by e^{i angle}),
identities (position 0, norm preservation, additivity of positions, the relative-position property
of the scores), the section -> component map, and the bookkeeping of the append.
"""
import cmath
import math

import numpy as np
import pytest

from oracle.kv_append_ref import kv_append_rope_ref, rope_tables, rotate
from paper_2512_21450_amd import workloads as wl


def case(seed, B=3, Hq=4, Hkv=2, d=8, cap=5, dtype="f32", lens=None):
    rng = np.random.default_rng(seed)
    t = lambda shape: (rng.standard_normal(shape).astype(np.float32) if dtype == "f32"
                       else wl.f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32)))
    return dict(q=t((B, Hq, d)), k_new=t((B, Hkv, d)), v_new=t((B, Hkv, d)),
                positions=rng.integers(0, 50, (3, B)).astype(np.int32), inv_freq=wl.rope_inv_freq(d, 100.0),
                sections=wl.mrope_sections(d), k_store=t((B, Hkv, cap, d)), v_store=t((B, Hkv, cap, d)),
                suffix_lens=(rng.integers(0, cap, B) if lens is None else np.asarray(lens)).astype(np.int32))


def run(x, **kw):
    return kv_append_rope_ref(x["q"], x["k_new"], x["v_new"], x["positions"], x["inv_freq"], x["sections"],
                              x["k_store"], x["v_store"], x["suffix_lens"], **kw)


def test_brute_force_complex_multiplication():
    x = case(1)
    q_rot, ks, vs, lens = run(x)
    B, Hq, d = x["q"].shape
    half = d // 2
    comp = [0] * x["sections"][0] + [1] * x["sections"][1] + [2] * x["sections"][2]
    for b in range(B):
        for h in range(Hq):
            for i in range(half):
                ang = float(x["positions"][comp[i], b]) * float(x["inv_freq"][i])
                z = complex(float(x["q"][b, h, i]), float(x["q"][b, h, i + half])) * cmath.exp(1j * ang)
                assert abs(q_rot[b, h, i] - z.real) < 2e-6 and abs(q_rot[b, h, i + half] - z.imag) < 2e-6
        n = int(x["suffix_lens"][b])
        for j in range(x["k_new"].shape[1]):
            for i in range(half):
                ang = float(x["positions"][comp[i], b]) * float(x["inv_freq"][i])
                z = complex(float(x["k_new"][b, j, i]), float(x["k_new"][b, j, i + half])) * cmath.exp(1j * ang)
                assert abs(ks[b, j, n, i] - z.real) < 2e-6 and abs(ks[b, j, n, i + half] - z.imag) < 2e-6
        assert np.array_equal(vs[b, :, n], x["v_new"][b]) and lens[b] == n + 1


def test_position_zero_is_identity_and_norms_are_kept():
    x = case(2)
    x["positions"][:] = 0
    q_rot, ks, _, _ = run(x)
    assert np.array_equal(q_rot, x["q"])
    x = case(3, d=16)
    q_rot, _, _, _ = run(x)
    half = 8
    n0 = x["q"][..., :half].astype(np.float64) ** 2 + x["q"][..., half:].astype(np.float64) ** 2
    n1 = q_rot[..., :half].astype(np.float64) ** 2 + q_rot[..., half:].astype(np.float64) ** 2
    assert np.allclose(n0, n1, rtol=1e-5)


def test_scores_depend_on_relative_position_only():
    # <R(m) q, R(n) k> = <R(m + s) q, R(n + s) k> for a common shift s of all three components
    rng = np.random.default_rng(4)
    d = 16
    inv = wl.rope_inv_freq(d, 50.0)
    sec = wl.mrope_sections(d)
    q = rng.standard_normal((1, 1, d)); k = rng.standard_normal((1, 1, d))
    def score(pq, pk):
        cq, sq = rope_tables(np.array(pq, np.int32).reshape(3, 1), inv, sec)
        ck, sk = rope_tables(np.array(pk, np.int32).reshape(3, 1), inv, sec)
        return float((rotate(q, cq, sq) * rotate(k, ck, sk)).sum())
    a = score([7, 3, 9], [2, 8, 4])
    b = score([7 + 11, 3 + 11, 9 + 11], [2 + 11, 8 + 11, 4 + 11])
    c = score([7, 3, 9], [3, 8, 4])
    assert abs(a - b) < 1e-5 and abs(a - c) > 1e-3


def test_sections_pick_the_component_and_pairing_is_rotate_half():
    d = 8                                     # sections (1, 1, 2): index 0 temporal, 1 height, 2..3 width
    inv = np.array([1.0, 1.0, 1.0, 1.0], np.float32)
    pos = np.array([[1], [2], [3]], np.int32)
    cos, sin = rope_tables(pos, inv, (1, 1, 2))
    assert np.allclose(cos[0], np.cos([1, 2, 3, 3]).astype(np.float32)) and np.allclose(sin[0], np.sin([1, 2, 3, 3]).astype(np.float32))
    x = np.zeros((1, 1, d)); x[0, 0, 1] = 1.0                     # unit vector on index 1: its partner is index 1 + d/2
    y = rotate(x, cos, sin)
    want = np.zeros(d); want[1] = math.cos(2.0); want[5] = math.sin(2.0)
    assert np.allclose(y[0, 0], want, atol=1e-7)


def test_rotations_compose_additively():
    rng = np.random.default_rng(5)
    d, inv, sec = 8, wl.rope_inv_freq(8, 10.0), (4, 0, 0)
    x = rng.standard_normal((2, 3, d))
    t = lambda p: rope_tables(np.array([p, p, p], np.int32), inv, sec)
    a = rotate(rotate(x, *t([3, 5])), *t([4, 1]))
    b = rotate(x, *t([7, 6]))
    assert np.allclose(a, b, atol=1e-6)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_append_bookkeeping_contiguous(dtype):
    x = case(6, B=4, cap=3, dtype=dtype, lens=[0, 2, 3, -1])      # full store and a negative length: skipped
    act = np.array([1, 1, 1, 1], np.uint8)
    q_rot, ks, vs, lens = run(x, seq_active=act)
    assert lens.tolist() == [1, 3, 3, -1]
    assert np.array_equal(ks[2], x["k_store"][2]) and np.array_equal(vs[3], x["v_store"][3])
    assert np.array_equal(vs[0, :, 0], x["v_new"][0]) and np.array_equal(vs[1, :, 2], x["v_new"][1])
    # untouched rows stay bit-identical
    m = np.ones(ks.shape, bool); m[0, :, 0] = False; m[1, :, 2] = False
    assert np.array_equal(ks[m], x["k_store"][m]) and np.array_equal(vs[m], x["v_store"][m])
    # finished sequences are left alone
    _, ks2, vs2, lens2 = run(x, seq_active=np.array([0, 1, 1, 1], np.uint8))
    assert lens2.tolist() == [0, 3, 3, -1] and np.array_equal(ks2[0], x["k_store"][0])


def test_append_into_pages_lands_where_the_attention_oracle_reads():
    from oracle import ref
    w = wl.scaled(wl.WORKLOADS["vlm3b"], P=1, G=3, Ls_cap=96, suffix=("uniform", 60))
    x = wl.make_inputs(w)
    full = dict(x); full["suffix_lens"] = np.full(w.B, 96, np.int32)
    y = wl.to_pages(full, 32, seed=2, poison=False)
    y["suffix_lens"] = x["suffix_lens"].copy()
    nt = wl.make_new_token(w, x, seed=5)
    q_rot, kp, vp, lens = kv_append_rope_ref(nt["q"], nt["k_new"], nt["v_new"], nt["positions"], nt["inv_freq"],
                                             nt["sections"], y["k_pages"], y["v_pages"], y["suffix_lens"],
                                             block_table=y["block_table"])
    assert np.array_equal(lens, x["suffix_lens"] + 1)
    g = ref.gather_pages(kp, y["block_table"], lens, 96)
    gv = ref.gather_pages(vp, y["block_table"], lens, 96)
    for b in range(w.B):
        n = int(x["suffix_lens"][b])
        assert np.array_equal(gv[b, :, n], nt["v_new"][b])
        assert np.array_equal(g[b, :, :n], x["k_suffix"][b, :, :n])
        assert not np.array_equal(g[b, :, n], nt["k_new"][b])     # rotated (positions are > 0)


def test_bf16_rounding_is_nearest_even():
    from oracle.kv_append_ref import _narrow
    like = np.zeros(1, np.uint16)
    vals = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, -2.5])
    got = _narrow(vals, like)
    assert got.tolist() == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xC020]
    assert np.array_equal(got, wl.f32_to_bf16_bits(vals.astype(np.float32)))


# ---------------------------------------------------------------- e4m3 stores
def test_e4m3_quantiser_against_the_definition():
    from oracle import ref
    from oracle.kv_append_ref import e4m3_round
    codes = np.arange(256, dtype=np.uint8)
    vals = ref.e4m3_to_f64(codes)                      # the decoder pinned in test_oracle_kv8_pins.py
    ok = ~np.isnan(vals)
    assert np.array_equal(e4m3_round(vals[ok]), codes[ok])            # representable values (and -0) keep their code
    pos = vals[:0x7F]
    for i in range(0x7E):                                             # between neighbours: nearest, ties to the even code
        lo, hi = pos[i], pos[i + 1]
        mid = (lo + hi) / 2
        assert e4m3_round(mid) == (i if i % 2 == 0 else i + 1), i
        assert e4m3_round(-mid) == (i if i % 2 == 0 else i + 1) | 0x80
        assert e4m3_round(np.nextafter(np.float32(mid), np.float32(0))) == i or np.float32(mid) != mid
        assert e4m3_round(mid - (hi - lo) / 64) == i and e4m3_round(mid + (hi - lo) / 64) == i + 1
    assert e4m3_round(448.0) == 0x7E and e4m3_round(449.0) == 0x7E and e4m3_round(1e30) == 0x7E
    assert e4m3_round(np.inf) == 0x7E and e4m3_round(-np.inf) == 0xFE
    assert e4m3_round(np.nan) & 0x7F == 0x7F
    assert e4m3_round(2.0 ** -10) == 0 and e4m3_round(2.0 ** -10 * 1.01) == 1      # half of the smallest subnormal ties to 0
    assert e4m3_round(0.0) == 0 and e4m3_round(-0.0) == 0x80


def test_e4m3_quantiser_against_library_rounding():
    import torch
    from oracle.kv_append_ref import e4m3_round
    rng = np.random.default_rng(3)
    x = np.concatenate([(rng.standard_normal(200000) * s).astype(np.float32) for s in (0.01, 1.0, 100.0)])
    x = x[np.abs(x) <= 448]                                            # beyond the range the library does not saturate
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(e4m3_round(x), lib)


def test_append_quantises_with_the_head_factor_and_leaves_other_rows_alone():
    from oracle import ref
    from oracle.kv_append_ref import e4m3_round
    x = case(21, dtype="bf16", lens=[0, 4, 5])                         # the third sequence is full (capacity 5)
    rng = np.random.default_rng(5)
    x["k_store"] = rng.integers(0, 256, x["k_store"].shape).astype(np.uint8)
    x["v_store"] = rng.integers(0, 256, x["v_store"].shape).astype(np.uint8)
    ksc, vsc = np.array([0.01, 0.37], np.float32), np.array([0.02, 0.005], np.float32)
    q_rot, ks, vs, lens = run(x, k_scale=ksc, v_scale=vsc)
    assert lens.tolist() == [1, 5, 5] and ks.dtype == np.uint8
    touched = np.zeros(ks.shape, bool)
    touched[0, :, 0] = True; touched[1, :, 4] = True
    assert np.array_equal(ks[~touched], x["k_store"][~touched]) and np.array_equal(vs[~touched], x["v_store"][~touched])
    v = wl.bf16_bits_to_f32(x["v_new"])
    for b, n in ((0, 0), (1, 4)):
        for j in range(2):
            want = e4m3_round((v[b, j] / vsc[j]).astype(np.float32))
            assert np.array_equal(vs[b, j, n], want)
            # dequantised, the stored row is within half an e4m3 step of the value (relative 2^-4 for normal values)
            back = ref.e4m3_to_f64(vs[b, j, n]) * float(vsc[j])
            assert np.all(np.abs(back - v[b, j]) <= np.maximum(np.abs(v[b, j]) * 2.0 ** -4, float(vsc[j]) * 2.0 ** -10))
    # the key row is the rotated key: same rotation as the bf16-store form, quantised from fp32
    cos, sin = rope_tables(x["positions"], x["inv_freq"], list(x["sections"]))
    kr = rotate(wl.bf16_bits_to_f32(x["k_new"]).astype(np.float64), cos, sin).astype(np.float32)
    for j in range(2):
        assert np.array_equal(ks[0, j, 0], e4m3_round((kr[0, j] / ksc[j]).astype(np.float32)))
    # factors of one are the default
    a = run(x)
    b = run(x, k_scale=np.ones(2, np.float32), v_scale=np.ones(2, np.float32))
    assert all(np.array_equal(u, w) for u, w in zip(a, b))
