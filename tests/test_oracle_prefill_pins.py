"""Pins for the oracle of the causal prefill attention (no GPU).

Pinned to the decode-attention oracle (itself pinned in test_oracle_pins.py): position i of the
prefill is one decode query whose key set is the first i + 1 rows; plus the closed forms of the
first position, the irrelevance of future keys, and a brute force in pure Python.
"""
import math

import numpy as np
import pytest

from oracle import ref
from oracle.prefill_ref import prefill_attn_ref
from paper_2512_21450_amd import workloads as wl


def case(seed, P=2, L=9, Hq=4, Hkv=2, d=8, dtype="f32", lens=None):
    rng = np.random.default_rng(seed)
    t = lambda s: (rng.standard_normal(s).astype(np.float32) if dtype == "f32"
                   else wl.f32_to_bf16_bits(rng.standard_normal(s).astype(np.float32)))
    return dict(q=t((P, L, Hq, d)), k=t((P, Hkv, L, d)), v=t((P, Hkv, L, d)),
                lens=(rng.integers(1, L + 1, P) if lens is None else np.asarray(lens)).astype(np.int32))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_every_position_is_a_decode_query_over_its_own_past(dtype):
    x = case(1, dtype=dtype, lens=[9, 5])
    out, lse = prefill_attn_ref(x["q"], x["k"], x["v"], x["lens"], 0.37)
    P, L, Hq, d = x["q"].shape
    none = np.zeros((1, x["k"].shape[1], 1, d), x["k"].dtype)
    for p in range(P):
        for i in range(int(x["lens"][p])):
            o, l = ref.decode_attn_ref(np.ascontiguousarray(x["q"][p:p + 1, i]), x["k"][p:p + 1], x["v"][p:p + 1],
                                       np.array([i + 1], np.int32), none, none, np.zeros(1, np.int32), 0.37, 1)
            assert np.allclose(out[p, i], o[0], rtol=1e-12, atol=1e-14) and np.allclose(lse[p, i], l[0], rtol=1e-13)
        assert np.isnan(out[p, int(x["lens"][p]):]).all() and np.isnan(lse[p, int(x["lens"][p]):]).all()


def test_brute_force_and_first_position():
    x = case(2, P=1, L=5, Hq=2, Hkv=1, d=3, lens=[5])
    out, lse = prefill_attn_ref(x["q"], x["k"], x["v"], x["lens"], 0.5)
    q, k, v = (a.astype(np.float64).tolist() for a in (x["q"], x["k"], x["v"]))
    for i in range(5):
        for h in range(2):
            s = [0.5 * sum(q[0][i][h][c] * k[0][0][n][c] for c in range(3)) for n in range(i + 1)]
            z = sum(math.exp(t) for t in s)
            assert math.isclose(lse[0, i, h], math.log(z), rel_tol=1e-12, abs_tol=1e-12)
            for c in range(3):
                want = sum(math.exp(s[n]) / z * v[0][0][n][c] for n in range(i + 1))
                assert math.isclose(out[0, i, h, c], want, rel_tol=1e-12, abs_tol=1e-14)
    # the first token sees only itself: its value comes back, its lse is its score
    assert np.allclose(out[0, 0, :, :], x["v"][0, 0, 0].astype(np.float64)[None, :])
    assert np.allclose(lse[0, 0], 0.5 * (x["q"][0, 0].astype(np.float64) @ x["k"][0, 0, 0].astype(np.float64)))


def test_the_future_and_the_padding_do_not_matter_and_heads_map_in_blocks():
    x = case(3, P=1, L=8, Hq=4, Hkv=2, lens=[6])
    out, lse = prefill_attn_ref(x["q"], x["k"], x["v"], x["lens"], 0.3)
    y = {a: b.copy() for a, b in x.items()}
    y["k"][0, :, 4:] = 77.0; y["v"][0, :, 4:] = -55.0; y["q"][0, 4:] = 9.0         # everything after position 3 changes
    o2, l2 = prefill_attn_ref(y["q"], y["k"], y["v"], y["lens"], 0.3)
    assert np.array_equal(o2[0, :4], out[0, :4]) and np.array_equal(l2[0, :4], lse[0, :4])
    assert not np.array_equal(o2[0, 4:6], out[0, 4:6])
    z = {a: b.copy() for a, b in x.items()}
    z["k"][0, :, 6:] = np.nan; z["v"][0, :, 6:] = np.nan                              # rows beyond the length are never read
    o3, l3 = prefill_attn_ref(z["q"], z["k"], z["v"], z["lens"], 0.3)
    assert np.array_equal(o3[0, :6], out[0, :6])
    w = {a: b.copy() for a, b in x.items()}
    w["k"][0, 1] += 1.0                                                                # KV head 1 serves query heads 2 and 3 only
    o4, _ = prefill_attn_ref(w["q"], w["k"], w["v"], w["lens"], 0.3)
    assert np.array_equal(o4[0, :6, :2], out[0, :6, :2]) and not np.array_equal(o4[0, :6, 2:], out[0, :6, 2:])
    e = prefill_attn_ref(x["q"], x["k"], x["v"], np.array([0], np.int32), 0.3)         # empty prompt: nothing defined
    assert np.isnan(e[0]).all()
