"""Pins for the oracle's 8-bit (e4m3) K/V store form (no GPU).

The attention itself is pinned in test_oracle_pins.py; what is new here is the
decode of a stored byte and where the per-head scales enter.  Pins: the value
of all 256 bytes against the format's definition (hand values, the structure
of the encoding, and torch's CPU conversion as a library check), equality
with the fp32-input oracle whenever scale * value is exact in fp32, the closed
forms for a single key, and the scale identities.
"""
import math

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2512_21450_amd import workloads as wl
from tests.test_oracle_pins import rand_case, run


def kv8_case(seed, **kw):
    """A random case whose K/V stores are random e4m3 bytes (NaN bytes excluded)."""
    x = rand_case(seed, **kw)
    rng = np.random.default_rng(seed + 77)
    for k in ("k_prefix", "v_prefix", "k_suffix", "v_suffix"):
        b = rng.integers(0, 256, x[k].shape).astype(np.uint8)
        b[(b & 0x7F) == 0x7F] = 0x3A
        x[k] = b
    return x


def run8(x, scale, k_scale=None, v_scale=None, **kw):
    return ref.decode_attn_ref(x["q"], x["k_prefix"], x["v_prefix"], x["prefix_lens"], x["k_suffix"],
                               x["v_suffix"], x["suffix_lens"], scale, x["G"], k_scale=k_scale, v_scale=v_scale, **kw)


def test_e4m3_hand_values():
    v = ref.e4m3_to_f64(np.arange(256))
    # values read off the format's definition: bias 7, 3 mantissa bits, subnormals below 2^-6
    hand = {0x00: 0.0, 0x01: 2.0 ** -9, 0x02: 2.0 ** -8, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x09: 1.125 * 2.0 ** -6,
            0x30: 0.5, 0x38: 1.0, 0x39: 1.125, 0x3C: 1.5, 0x3F: 1.875, 0x40: 2.0, 0x48: 4.0, 0x77: 240.0,
            0x78: 256.0, 0x7E: 448.0}
    for b, val in hand.items():
        assert v[b] == val, hex(b)
        assert v[b | 0x80] == -val and math.copysign(1.0, v[b | 0x80]) == -1.0, hex(b | 0x80)
    assert math.isnan(v[0x7F]) and math.isnan(v[0xFF])
    assert np.isfinite(np.delete(v, [0x7F, 0xFF])).all()          # no infinities in this format


def test_e4m3_structure_of_the_encoding():
    v = ref.e4m3_to_f64(np.arange(0x7F))
    assert (np.diff(v) > 0).all()                                  # the positive bytes are ordered by value
    # inside a binade the 8 mantissa steps are equal, and the step doubles from one binade to the next
    for e in range(1, 16):
        blk = v[8 * e:8 * e + 8]                                   # the top binade has 7 values (0x7f is NaN)
        steps = np.diff(blk)
        assert (steps == 2.0 ** (e - 10)).all(), e
    assert (np.diff(v[:9]) == 2.0 ** -9).all()                     # subnormals continue the first binade's step
    # every value is an integer multiple of 2^-9 with at most 4 significant bits: exact in bf16 and fp32
    m, _ = np.frexp(v[1:])
    assert (m * 16 == np.round(m * 16)).all()


def test_e4m3_against_library_conversion():
    b = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(b).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = ref.e4m3_to_f64(b)
    assert np.array_equal(np.isnan(lib), np.isnan(mine))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], mine[ok]) and np.array_equal(np.signbit(lib[ok]), np.signbit(mine[ok]))


@pytest.mark.parametrize("seed,qdtype", [(1, "f32"), (2, "bf16"), (3, "f32")])
def test_equals_the_fp32_store_oracle_when_dequantisation_is_exact(seed, qdtype):
    # power-of-two scales: scale * e4m3 value is exact in fp32, so the same attention can be
    # stated on fp32 stores and must give the same numbers
    x = kv8_case(seed, dtype=qdtype, P=2, G=3, Hq=4, Hkv=2, d=8, Lp_cap=9, Ls_cap=7)
    ksc, vsc = np.array([0.25, 2.0], np.float32), np.array([0.5, 0.0625], np.float32)
    o8, l8 = run8(x, 0.3, ksc, vsc)
    y = dict(x)
    for k, sc in (("k_prefix", ksc), ("k_suffix", ksc), ("v_prefix", vsc), ("v_suffix", vsc)):
        y[k] = (ref.e4m3_to_f64(x[k]) * sc[None, :, None, None]).astype(np.float32)
    if qdtype == "bf16":                                           # the fp32-store form wants one element type
        y["q"] = wl.bf16_bits_to_f32(x["q"])
    o, l = run(y, 0.3)
    assert np.allclose(o8, o, rtol=0, atol=1e-14) and np.allclose(l8, l, rtol=0, atol=1e-13)


def test_single_key_returns_scaled_value_and_score():
    x = kv8_case(5, P=1, G=2, Hq=4, Hkv=2, d=8, Lp_cap=0, Ls_cap=3, slens=[1, 1])
    ksc, vsc = np.array([0.37, 1.9], np.float32), np.array([0.011, 3.3], np.float32)
    o, l = run8(x, 0.7, ksc, vsc)
    kf, vf = ref.e4m3_to_f64(x["k_suffix"]), ref.e4m3_to_f64(x["v_suffix"])
    for b in range(2):
        for h in range(4):
            j = h // 2
            assert np.allclose(o[b, h], float(vsc[j]) * vf[b, j, 0], rtol=1e-15, atol=0)
            s = 0.7 * float(ksc[j]) * float(np.dot(x["q"][b, h].astype(np.float64), kf[b, j, 0]))
            assert abs(l[b, h] - s) <= 1e-12 * max(1.0, abs(s))


def test_scale_identities():
    x = kv8_case(9, P=2, G=2, Hq=6, Hkv=3, d=8, Lp_cap=6, Ls_cap=5)
    one = np.ones(3, np.float32)
    o0, l0 = run8(x, 0.4, None, None)
    o1, l1 = run8(x, 0.4, one, one)
    assert np.array_equal(o0, o1) and np.array_equal(l0, l1)      # no scales = scales of one
    # a uniform K scale is a softmax scale; a V scale multiplies the output of its own heads only
    o2, l2 = run8(x, 0.4, 4 * one, one)
    o3, l3 = run8(x, 1.6, one, one)
    assert np.allclose(o2, o3, rtol=1e-13, atol=1e-15)
    fin = np.isfinite(l3)
    assert np.array_equal(np.isfinite(l2), fin) and np.allclose(l2[fin], l3[fin], rtol=1e-13, atol=1e-13)
    vsc = np.array([1.0, 3.0, 0.5], np.float32)
    o4, l4 = run8(x, 0.4, one, vsc)
    assert np.array_equal(l4, l0)
    for h in range(6):
        assert np.allclose(o4[:, h], float(vsc[h // 2]) * o0[:, h], rtol=1e-14, atol=0)
    # per-head K scale: changing head 1's factor leaves the other KV groups untouched
    o5, l5 = run8(x, 0.4, np.array([1.0, 2.5, 1.0], np.float32), one)
    assert np.array_equal(o5[:, [0, 1, 4, 5]], o0[:, [0, 1, 4, 5]]) and np.array_equal(l5[:, [0, 1, 4, 5]], l0[:, [0, 1, 4, 5]])
    assert not np.array_equal(l5[:, 2:4], l0[:, 2:4])


def test_paged_form_takes_bytes_too():
    x = kv8_case(11, P=2, G=2, Hq=4, Hkv=2, d=8, Lp_cap=5, Ls_cap=96)
    sc = np.array([0.5, 0.3], np.float32)
    y = wl.to_pages(x, 32, seed=4)
    assert y["k_pages"].dtype == np.uint8
    o, l = ref.decode_attn_paged_ref(y["q"], y["k_prefix"], y["v_prefix"], y["prefix_lens"], y["k_pages"],
                                     y["v_pages"], y["block_table"], y["suffix_lens"], None, 0.4, x["G"],
                                     k_scale=sc, v_scale=sc)
    o0, l0 = run8(x, 0.4, sc, sc)
    assert np.array_equal(o, o0) and np.array_equal(l, l0)


def test_quantiser_of_the_workload_generator_rounds_to_nearest():
    # data preparation, not the method -- but the bench relies on it: stored byte = nearest e4m3 to value / scale
    w = wl.scaled(wl.WORKLOADS["vlm3b"], P=1, G=2, Lp_cap=40, Ls_cap=33, prefix=("const", 40), suffix=("uniform", 33))
    x = wl.make_inputs(w)
    y = wl.kv_to_e4m3(x)
    table = ref.e4m3_to_f64(np.arange(0x7F))
    for name in ("k", "v"):
        sc = y[f"{name}_scale"]
        assert sc.shape == (w.Hkv,) and sc.dtype == np.float32
        for store in ("prefix", "suffix"):
            f = wl.bf16_bits_to_f32(x[f"{name}_{store}"]).astype(np.float64) / sc[None, :, None, None].astype(np.float32)
            got = ref.e4m3_to_f64(y[f"{name}_{store}"])
            assert np.isfinite(got).all() and np.abs(got).max() <= 448.0
            # no table entry is closer than the chosen one (the division above is in fp32 like the generator's)
            f32 = (wl.bf16_bits_to_f32(x[f"{name}_{store}"]) / sc[None, :, None, None]).astype(np.float64)
            best = np.abs(np.abs(f32)[..., None] - table).min(axis=-1)
            assert np.allclose(np.abs(got - f32), best, rtol=0, atol=1e-12)
        assert np.abs(ref.e4m3_to_f64(y[f"{name}_prefix"])).max() == 448.0 or \
               np.abs(ref.e4m3_to_f64(y[f"{name}_suffix"])).max() == 448.0
