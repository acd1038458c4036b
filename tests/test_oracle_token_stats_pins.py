"""Pins for the fp64 oracle of the per-token policy statistics (no GPU).

Pinned to closed forms, a pure-Python brute force, invariances, and to library
routines written by others (scipy.special, scipy.stats, torch CPU fp64), so
that a dropped term, a wrong sign, KL taken in the wrong direction, a
temperature applied to one side only or a wrong gather index fails a check.
"""
import math

import numpy as np
import pytest
import scipy.special
import scipy.stats
import torch

from oracle.token_stats_ref import token_stats_ref
from paper_2512_21450_amd import workloads as wl


def test_uniform_logits_closed_form():
    for V in (1, 2, 7, 1000):
        lg = np.full((3, V), 1.75, np.float32)
        r = token_stats_ref(lg, [0, V - 1, V // 2], ref_logits=lg + 4.0)
        assert np.allclose(r["logprob"], -math.log(V), atol=1e-13)
        assert np.allclose(r["lse"], 1.75 + math.log(V), atol=1e-13)
        assert np.allclose(r["entropy"], math.log(V), atol=1e-13)
        assert np.allclose(r["kl"], 0.0, atol=1e-13)            # a shifted copy is the same distribution
        assert np.allclose(r["ref_logprob"], -math.log(V), atol=1e-13)


def test_two_token_closed_form_and_kl_direction():
    a, b = 0.3, -1.1           # p = sigmoid(a - b) on token 0
    c, d = -0.4, 0.9           # reference
    lg = np.array([[a, b]], np.float32)
    rf = np.array([[c, d]], np.float32)
    a, b, c, d = (float(np.float32(v)) for v in (a, b, c, d))   # the values the oracle sees
    p0 = 1 / (1 + math.exp(b - a)); p1 = 1 - p0
    r0 = 1 / (1 + math.exp(d - c)); r1 = 1 - r0
    r = token_stats_ref(lg, [1], ref_logits=rf)
    assert abs(r["logprob"][0] - math.log(p1)) < 1e-13
    assert abs(r["ref_logprob"][0] - math.log(r1)) < 1e-13
    assert abs(r["entropy"][0] + p0 * math.log(p0) + p1 * math.log(p1)) < 1e-13
    kl_pr = p0 * math.log(p0 / r0) + p1 * math.log(p1 / r1)
    kl_rp = r0 * math.log(r0 / p0) + r1 * math.log(r1 / p1)
    assert abs(kl_pr - kl_rp) > 1e-3
    assert abs(r["kl"][0] - kl_pr) < 1e-13                      # KL(policy || reference), not the reverse


def brute(lg, y, invT, rf=None):
    z = [float(v) * invT for v in lg]
    Z = sum(math.exp(v) for v in z)
    p = [math.exp(v) / Z for v in z]
    res = dict(logprob=math.log(p[y]), lse=math.log(Z), entropy=-sum(q * math.log(q) for q in p))
    if rf is not None:
        w = [float(v) * invT for v in rf]
        W = sum(math.exp(v) for v in w)
        r = [math.exp(v) / W for v in w]
        res["kl"] = sum(q * math.log(q / s) for q, s in zip(p, r))
        res["ref_logprob"] = math.log(r[y])
    return res


@pytest.mark.parametrize("invT", [1.0, 0.5, 1.7])
def test_pure_python_brute_force(invT):
    rng = np.random.default_rng(3)
    lg = rng.standard_normal((5, 11)).astype(np.float32) * 2
    rf = rng.standard_normal((5, 11)).astype(np.float32) * 2
    ids = rng.integers(0, 11, 5)
    r = token_stats_ref(lg, ids, invT, ref_logits=rf)
    for b in range(5):
        e = brute(lg[b], int(ids[b]), invT, rf[b])
        for k, v in e.items():
            assert abs(r[k][b] - v) < 1e-12, (k, b)


def test_against_scipy_and_torch_routines():
    x = wl.make_logits(6, 5003, seed=21, dtype="f32", with_ref=True)
    invT = 0.8
    r = token_stats_ref(x["logits"], x["token_ids"], invT, ref_logits=x["ref_logits"])
    z = x["logits"].astype(np.float64) * invT
    w = x["ref_logits"].astype(np.float64) * invT
    ls = scipy.special.log_softmax(z, axis=1)
    assert np.allclose(r["lse"], scipy.special.logsumexp(z, axis=1), atol=1e-12)
    assert np.allclose(r["logprob"], ls[np.arange(6), x["token_ids"]], atol=1e-12)
    p, q = scipy.special.softmax(z, axis=1), scipy.special.softmax(w, axis=1)
    assert np.allclose(r["entropy"], scipy.stats.entropy(p, axis=1), atol=1e-12)
    assert np.allclose(r["kl"], scipy.stats.entropy(p, q, axis=1), atol=1e-12)
    tz, tw = torch.from_numpy(z), torch.from_numpy(w)
    ids = torch.from_numpy(x["token_ids"].astype(np.int64))
    ce = torch.nn.functional.cross_entropy(tz, ids, reduction="none")
    assert np.allclose(r["logprob"], -ce.numpy(), atol=1e-12)
    kl = torch.nn.functional.kl_div(torch.log_softmax(tw, 1), torch.log_softmax(tz, 1), reduction="none",
                                    log_target=True).sum(1)     # kl_div(input=log r, target=log p) = sum p (log p - log r)
    assert np.allclose(r["kl"], kl.numpy(), atol=1e-12)
    assert np.allclose(r["ref_logprob"], torch.log_softmax(tw, 1)[torch.arange(6), ids].numpy(), atol=1e-12)


def test_shift_invariance_peaked_rows_and_large_values():
    rng = np.random.default_rng(5)
    lg = rng.standard_normal((4, 300)).astype(np.float32)
    ids = rng.integers(0, 300, 4)
    r0 = token_stats_ref(lg, ids)
    r1 = token_stats_ref(lg + np.float32(64.0), ids)            # exact in fp32 for these magnitudes? compare loosely
    assert np.allclose(r0["logprob"], r1["logprob"], atol=1e-4) and np.allclose(r1["lse"] - 64.0, r0["lse"], atol=1e-4)
    big = np.full((1, 50), -1e4, np.float32); big[0, 17] = 1e4  # one-hot: no overflow, entropy 0
    r = token_stats_ref(big, [17], ref_logits=big)
    assert r["logprob"][0] == 0.0 and r["entropy"][0] == 0.0 and r["kl"][0] == 0.0 and r["lse"][0] == 1e4
    r = token_stats_ref(big, [3])
    assert r["logprob"][0] == -2e4


def test_temperature_is_a_scale_on_both_tensors_and_ids_are_rowwise():
    x = wl.make_logits(3, 97, seed=8, dtype="f32", with_ref=True)
    a = token_stats_ref(x["logits"], x["token_ids"], 0.5, ref_logits=x["ref_logits"])
    b = token_stats_ref(x["logits"] * np.float32(0.5), x["token_ids"], 1.0, ref_logits=x["ref_logits"] * np.float32(0.5))
    for k in a:
        assert np.allclose(a[k], b[k], atol=1e-12), k
    # swapping two rows swaps the results (the id of row b indexes row b)
    perm = [1, 0, 2]
    c = token_stats_ref(x["logits"][perm], x["token_ids"][perm], 0.5, ref_logits=x["ref_logits"][perm])
    for k in a:
        assert np.allclose(c[k], a[k][perm], atol=0), k


def test_ignored_and_out_of_range_ids_and_bf16_widening():
    lg = np.array([[0.0, 1.0, 2.0]], np.float32)
    assert token_stats_ref(lg, [-100])["logprob"][0] == 0.0
    assert np.isnan(token_stats_ref(lg, [3])["logprob"][0])
    bits = wl.f32_to_bf16_bits(np.array([[0.5, -1.25, 3.0]], np.float32))
    r1 = token_stats_ref(bits, [2])
    r2 = token_stats_ref(np.array([[0.5, -1.25, 3.0]], np.float32), [2])
    assert r1["logprob"][0] == r2["logprob"][0]


def test_kl_is_nonnegative_and_zero_only_for_equal_distributions():
    x = wl.make_logits(8, 400, seed=9, dtype="bf16", with_ref=True)
    r = token_stats_ref(x["logits"], x["token_ids"], ref_logits=x["ref_logits"])
    assert (r["kl"] > 0).all() and (r["entropy"] > 0).all() and (r["entropy"] <= math.log(400)).all()
    r = token_stats_ref(x["logits"], x["token_ids"], ref_logits=x["logits"])
    assert np.abs(r["kl"]).max() < 1e-15 and np.array_equal(r["logprob"], r["ref_logprob"])


def test_generator_is_seeded_and_ids_in_range():
    a = wl.make_logits(16, 1000, seed=4, with_ref=True)
    b = wl.make_logits(16, 1000, seed=4, with_ref=True)
    assert all(np.array_equal(a[k], b[k]) for k in a)
    assert a["logits"].dtype == np.uint16 and a["token_ids"].dtype == np.int32
    assert (a["token_ids"] >= 0).all() and (a["token_ids"] < 1000).all()


def test_masked_logits_are_the_distribution_over_the_rest():
    rng = np.random.default_rng(12)
    lg = rng.standard_normal((2, 40)).astype(np.float32)
    rf = rng.standard_normal((2, 40)).astype(np.float32)
    keep = np.ones(40, bool); keep[[3, 17, 18, 39]] = False
    m, mr = lg.copy(), rf.copy()
    m[:, ~keep] = -np.inf
    ids_full = np.array([5, 20])
    ids_kept = np.array([int(keep[:5].sum()), int(keep[:20].sum())])
    a = token_stats_ref(m, ids_full, ref_logits=rf)
    b = token_stats_ref(lg[:, keep], ids_kept, ref_logits=rf[:, keep])
    assert np.allclose(a["logprob"], b["logprob"], atol=1e-13) and np.allclose(a["entropy"], b["entropy"], atol=1e-13)
    # KL against a reference that keeps its mass on the masked tokens differs; against one masked alike it matches
    mr[:, ~keep] = -np.inf
    c = token_stats_ref(m, ids_full, ref_logits=mr)
    assert np.allclose(c["kl"], b["kl"], atol=1e-13) and np.allclose(c["ref_logprob"], b["ref_logprob"], atol=1e-13)
    assert np.isneginf(token_stats_ref(m, [3, 3])["logprob"]).all()


def test_nan_logits_are_read_as_masked_tokens():
    # the reading the header states: a NaN logit is a masked token; the rest of the row keeps its distribution
    rng = np.random.default_rng(13)
    lg = rng.standard_normal((3, 30)).astype(np.float32)
    rf = rng.standard_normal((3, 30)).astype(np.float32)
    bad, ref_bad = lg.copy(), rf.copy()
    bad[:, [2, 11, 29]] = np.nan
    ref_bad[:, [2, 11, 29]] = np.nan
    inf, ref_inf = lg.copy(), rf.copy()
    inf[:, [2, 11, 29]] = -np.inf
    ref_inf[:, [2, 11, 29]] = -np.inf
    ids = np.array([0, 11, 12])
    a = token_stats_ref(bad, ids, 0.7, ref_logits=ref_bad)
    b = token_stats_ref(inf, ids, 0.7, ref_logits=ref_inf)
    for k in a:
        assert np.array_equal(a[k], b[k], equal_nan=True), k
    assert np.isfinite(a["lse"]).all() and np.isfinite(a["entropy"]).all() and np.isfinite(a["kl"]).all()
    assert np.isneginf(a["logprob"][1]) and np.isfinite(a["logprob"][[0, 2]]).all()   # the sampled token itself masked
