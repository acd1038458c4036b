"""Pins for the oracle of the advantage estimators and the clipped policy loss (no GPU).

Pinned to what the definitions fix: hand-computed cases of every branch of the clipped
surrogate, the on-policy point (ratio 1), finite differences of the loss for the gradient,
the two aggregations on ragged lengths by hand, linearity in the regulariser weights, and
for the estimators their defining identities.
"""
import math

import numpy as np
import pytest

from oracle.policy_loss_ref import (ADV_GROUP_CENTER, ADV_GROUP_NORM, ADV_LEAVE_ONE_OUT, AGG_SEQ_MEAN,
                                    AGG_TOKEN_MEAN, FORM_PPO, FORM_PRINTED, group_advantage_ref, policy_loss_ref)


def case(seed, B=6, T=9, spread=0.3):
    rng = np.random.default_rng(seed)
    old = -np.abs(rng.standard_normal((B, T))).astype(np.float32) - 0.1
    lp = (old + spread * rng.standard_normal((B, T))).astype(np.float32)
    return dict(logprob=lp, old_logprob=old, advantages=rng.standard_normal(B).astype(np.float32),
                lens=rng.integers(0, T + 1, B).astype(np.int32),
                kl=np.abs(rng.standard_normal((B, T))).astype(np.float32),
                entropy=np.abs(rng.standard_normal((B, T))).astype(np.float32))


def test_every_branch_of_the_clipped_surrogate_by_hand():
    # one token per sequence; eps_low = 0.2, eps_high = 0.3: ratio clipped to [0.8, 1.3]
    rho = np.array([1.0, 1.5, 1.5, 0.5, 0.5, 1.25, 0.875])        # the last two: inside the range
    A = np.array([2.0, 2.0, -2.0, 2.0, -2.0, 1.0, -1.0])
    want = np.array([2.0, 2.6, -3.0, 1.0, -1.6, 1.25, -0.875])   # min(rho A, clip(rho) A)
    dwant = np.array([2.0, 0.0, -3.0, 1.0, 0.0, 1.25, -0.875])   # rho A where the unclipped branch is the minimum
    lp = np.log(rho)[:, None].astype(np.float32)
    r = policy_loss_ref(lp, np.zeros_like(lp), A, np.ones(7, np.int32), 0.2, 0.3)
    rho32 = np.exp(lp.astype(np.float64))[:, 0]
    assert np.allclose(r["ratio"][:, 0], rho32)
    assert math.isclose(r["pg"], want.mean(), rel_tol=1e-6) and math.isclose(r["loss"], -want.mean(), rel_tol=1e-6)
    assert np.allclose(r["grad"][:, 0], -dwant / 7, rtol=1e-6)
    assert math.isclose(r["clip_frac"], 2 / 7) and r["n_tokens"] == 7
    # the expression as printed under Eq. 6, min(rho, clip(rho)) A, differs exactly where A < 0 and rho leaves the range
    p = policy_loss_ref(lp, np.zeros_like(lp), A, np.ones(7, np.int32), 0.2, 0.3, form=FORM_PRINTED)
    wantp = np.minimum(rho, 1.3) * A
    assert math.isclose(p["pg"], wantp.mean(), rel_tol=1e-6)
    differs = ~np.isclose(wantp, want)
    assert differs.tolist() == [False, False, True, False, True, False, False]
    assert np.allclose(p["grad"][:, 0], -np.where(rho > 1.3, 0.0, rho * A) / 7, rtol=1e-6)


def test_on_policy_point():
    x = case(1)
    r = policy_loss_ref(x["old_logprob"], x["old_logprob"], x["advantages"], x["lens"], 0.2, 0.2)
    L = x["lens"].astype(np.float64)
    assert math.isclose(r["pg"], (x["advantages"].astype(np.float64) * L).sum() / L.sum(), rel_tol=1e-12)
    assert r["clip_frac"] == 0.0 and math.isclose(r["ratio_mean"], 1.0) and r["approx_kl"] == 0.0
    valid = np.arange(9)[None, :] < x["lens"][:, None]
    assert np.allclose(r["grad"], np.where(valid, -x["advantages"].astype(np.float64)[:, None] / L.sum(), 0.0))


@pytest.mark.parametrize("form", [FORM_PPO, FORM_PRINTED])
@pytest.mark.parametrize("agg", [AGG_TOKEN_MEAN, AGG_SEQ_MEAN])
def test_gradient_by_finite_differences(form, agg):
    x = case(2, spread=0.4)
    args = (x["advantages"], x["lens"], 0.2, 0.28)
    kw = dict(kl=x["kl"], entropy=x["entropy"], beta_kl=0.05, beta_ent=0.01, form=form, agg=agg)
    lp = x["logprob"].astype(np.float64)
    r = policy_loss_ref(lp, x["old_logprob"], *args, **kw)
    h = 1e-6
    near_kink = (np.abs(r["ratio"] - 0.8) < 1e-4) | (np.abs(r["ratio"] - 1.28) < 1e-4)
    checked = 0
    for b in range(lp.shape[0]):
        for t in range(lp.shape[1]):
            if near_kink[b, t]:
                continue
            up, dn = lp.copy(), lp.copy()
            up[b, t] += h; dn[b, t] -= h
            fd = (policy_loss_ref(up, x["old_logprob"], *args, **kw)["loss"] -
                  policy_loss_ref(dn, x["old_logprob"], *args, **kw)["loss"]) / (2 * h)
            assert abs(fd - r["grad"][b, t]) <= 1e-7 + 1e-5 * abs(fd), (b, t)
            checked += 1
    assert checked > 40 and (r["grad"][np.arange(9)[None, :] >= x["lens"][:, None]] == 0).all()


def test_aggregations_by_hand_and_padding_is_ignored():
    lp = np.log(np.array([[1.1, 0.9, 7.0], [1.0, 5.0, 5.0], [3.0, 3.0, 3.0]])).astype(np.float32)
    old = np.zeros_like(lp)
    A = np.array([1.0, -1.0, 4.0], np.float32)
    lens = np.array([2, 1, 0], np.int32)                           # third sequence: no tokens at all
    rho = np.exp(lp.astype(np.float64))
    t = policy_loss_ref(lp, old, A, lens, 0.5, 0.5)
    assert math.isclose(t["pg"], (rho[0, 0] + rho[0, 1] - rho[1, 0]) / 3, rel_tol=1e-12) and t["n_tokens"] == 3
    s = policy_loss_ref(lp, old, A, lens, 0.5, 0.5, agg=AGG_SEQ_MEAN)
    assert math.isclose(s["pg"], ((rho[0, 0] + rho[0, 1]) / 2 - rho[1, 0]) / 2, rel_tol=1e-12)
    assert (t["grad"][2] == 0).all() and t["grad"][0, 2] == 0 and (t["grad"][1, 1:] == 0).all()
    lp2 = lp.copy(); lp2[0, 2] = np.nan; lp2[2] = np.inf            # garbage in the padding changes nothing
    with np.errstate(all="ignore"):
        t2 = policy_loss_ref(lp2, old, A, lens, 0.5, 0.5)
    assert t2["loss"] == t["loss"] and np.array_equal(t2["grad"], t["grad"])
    e = policy_loss_ref(lp, old, A, np.zeros(3, np.int32), 0.5, 0.5)   # no token anywhere: everything 0, nothing NaN
    assert e["loss"] == 0 and e["n_tokens"] == 0 and (e["grad"] == 0).all()
    c = policy_loss_ref(lp, old, A, np.array([9, -3, 1], np.int32), 0.5, 0.5)   # lengths clamp to [0, T]
    assert c["n_tokens"] == 4


def test_regulariser_terms_are_linear_and_signed_as_in_the_objective():
    x = case(3)
    base = policy_loss_ref(x["logprob"], x["old_logprob"], x["advantages"], x["lens"], 0.2, 0.2)
    r = policy_loss_ref(x["logprob"], x["old_logprob"], x["advantages"], x["lens"], 0.2, 0.2,
                        kl=x["kl"], entropy=x["entropy"], beta_kl=0.3, beta_ent=0.07)
    valid = np.arange(9)[None, :] < x["lens"][:, None]
    n = valid.sum()
    assert math.isclose(r["kl"], x["kl"].astype(np.float64)[valid].sum() / n, rel_tol=1e-12)
    assert math.isclose(r["entropy"], x["entropy"].astype(np.float64)[valid].sum() / n, rel_tol=1e-12)
    # maximise sum L - Omega with Omega = beta_KL KL - beta_ent H  <=>  loss = -L + beta_KL KL - beta_ent H
    assert math.isclose(r["loss"], base["loss"] + 0.3 * r["kl"] - 0.07 * r["entropy"], rel_tol=1e-12)
    assert np.array_equal(r["grad"], base["grad"])                  # the regularisers do not depend on the sampled token's logprob


def test_group_estimators():
    rng = np.random.default_rng(4)
    P, G, M = 5, 8, 3
    m = rng.standard_normal((M, P * G)).astype(np.float32)
    a = np.array([1.0, 0.5, -2.0], np.float32)
    r, adv = group_advantage_ref(m, a, G)
    assert np.allclose(r, (a[:, None].astype(np.float64) * m).sum(0))              # scoring stage: weighted sum of metrics
    g, A = r.reshape(P, G), adv.reshape(P, G)
    assert np.allclose(A.mean(1), 0, atol=1e-12)
    assert np.allclose(A.std(1, ddof=1), 1, atol=1e-4)                              # eps = 1e-6 keeps it just below 1
    assert np.allclose(A * (g.std(1, ddof=1, keepdims=True) + 1e-6), g - g.mean(1, keepdims=True))
    _, Ab = group_advantage_ref(m, a, G, unbiased=False)
    assert np.allclose(Ab.reshape(P, G) * (g.std(1, keepdims=True) + 1e-6), g - g.mean(1, keepdims=True))
    _, C = group_advantage_ref(m, a, G, mode=ADV_GROUP_CENTER)
    assert np.allclose(C.reshape(P, G), g - g.mean(1, keepdims=True))
    _, Lo = group_advantage_ref(m, a, G, mode=ADV_LEAVE_ONE_OUT)
    brute = np.array([[g[p, i] - np.delete(g[p], i).mean() for i in range(G)] for p in range(P)])
    assert np.allclose(Lo.reshape(P, G), brute)
    assert np.allclose(Lo.reshape(P, G), (g - g.mean(1, keepdims=True)) * G / (G - 1))   # the known closed form
    # a group whose samples all earned the same reward carries no signal, and nothing divides by zero
    same = np.ones((1, 8), np.float32)
    for mode in (ADV_GROUP_NORM, ADV_GROUP_CENTER, ADV_LEAVE_ONE_OUT):
        assert (group_advantage_ref(same, np.ones(1), 4, mode=mode)[1] == 0).all()
        assert (group_advantage_ref(same, np.ones(1), 1, mode=mode)[1] == 0).all()   # groups of one sample
    # shift invariance, and scale invariance of the normalised estimator
    _, A2 = group_advantage_ref(3 * m + 0.0, a, G, eps=0.0)
    _, A1 = group_advantage_ref(m, a, G, eps=0.0)
    assert np.allclose(A1, A2)
    m2 = m.copy(); m2[0] += 5
    assert np.allclose(group_advantage_ref(m2, a, G)[1], adv)
