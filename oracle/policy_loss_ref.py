"""fp64 CPU oracle of the scoring, advantage-estimation and policy-loss arithmetic
(TEST INFRASTRUCTURE ONLY: tests, the smoke check and the benchmark's CPU leg may import this
module; the product path never does).

What the paper fixes (Sec. 2.2 "Adaptation for Off-Policy" and "Regularization"; Sec. 3.1 "The
Objective of RLLaVA", Eq. 6 and the text under it; Sec. 3.2.2 scoring, advantage estimation and
policy update stages; Algorithm 1):

  scoring       r_b = sum_m alpha_m R_m(b)                  one scalar per trajectory
  advantages    A   = AdvEstimator(r)                        critic-free: from the K rewards of a group
  ratio         rho_t = pi_theta(y_t | .) / pi_old(y_t | .) = exp(logprob_t - old_logprob_t)
  policy term   L_t = min(rho_t A, clip(rho_t, 1 - eps_low, 1 + eps_high) A)       (PPO's clipped surrogate)
  regulariser   Omega = beta_KL sum_t KL_t  (and the entropy bonus beta_ent sum_t H_t)
  objective     maximise  sum_t L_t - Omega ; the loss is its negative, aggregated over tokens

Readings where the paper is silent or loose (also listed in the design notes):
  * The text under Eq. 6 prints the clipped term as min[rho, clip(rho)] * A.  For A >= 0 that is
    the same number as PPO's min(rho A, clip(rho) A); for A < 0 it is not (it would reward pushing
    rho up without bound).  The paper names PPO's clipped surrogate as what it means, so `form`
    0 is PPO's; `form` 1 evaluates the expression exactly as printed.
  * Two clip widths (eps_low, eps_high): the "decoupled clip ratios" the paper lists among its
    integrated variants (Sec. 4.2); equal widths give plain PPO.
  * Group estimators (named in Sec. 4.2, formulas from their publications): group normalisation
    A_i = (r_i - mean) / (std + eps) over the G samples of a prompt (std with divisor G - 1 when
    `unbiased`, else G; a group of one sample gets std 0), centring A_i = r_i - mean, and the
    leave-one-out baseline A_i = r_i - mean_{j != i} r_j (0 for a group of one).
  * Aggregation: token mean (every valid token of the batch weighs 1/N) or sequence mean of
    per-sequence token means (sequences without tokens do not count).  Tokens at t >= lens[b]
    are padding.

Everything is numpy fp64 over the given fp32 inputs.
"""
from __future__ import annotations

import numpy as np

ADV_GROUP_NORM, ADV_GROUP_CENTER, ADV_LEAVE_ONE_OUT = 0, 1, 2
FORM_PPO, FORM_PRINTED = 0, 1
AGG_TOKEN_MEAN, AGG_SEQ_MEAN = 0, 1


def group_advantage_ref(metrics, weights, G, mode=ADV_GROUP_NORM, eps=1e-6, unbiased=True):
    """metrics [M, B] (fp32), weights [M] -> (rewards [B], advantages [B]) in fp64; B = P * G,
    the G samples of a prompt adjacent."""
    R = np.asarray(metrics, dtype=np.float64)
    a = np.asarray(weights, dtype=np.float64)
    r = (a[:, None] * R).sum(axis=0)
    g = r.reshape(-1, G)
    mean = g.mean(axis=1, keepdims=True)
    if mode == ADV_GROUP_CENTER:
        adv = g - mean
    elif mode == ADV_LEAVE_ONE_OUT:
        adv = np.zeros_like(g) if G == 1 else g - (g.sum(axis=1, keepdims=True) - g) / (G - 1)
    elif mode == ADV_GROUP_NORM:
        div = G - 1 if unbiased else G
        var = ((g - mean) ** 2).sum(axis=1, keepdims=True) / div if div > 0 else np.zeros_like(mean)
        adv = (g - mean) / (np.sqrt(var) + eps)
    else:
        raise ValueError(mode)
    return r, adv.reshape(-1)


def policy_loss_ref(logprob, old_logprob, advantages, lens, clip_low, clip_high, kl=None, entropy=None,
                    beta_kl=0.0, beta_ent=0.0, form=FORM_PPO, agg=AGG_TOKEN_MEAN):
    """Returns dict(loss, pg, kl, entropy, clip_frac, ratio_mean, approx_kl, n_tokens, grad [B, T],
    ratio [B, T]) in fp64.  logprob / old_logprob / kl / entropy are [B, T]; advantages [B]."""
    lp = np.asarray(logprob, dtype=np.float64)
    old = np.asarray(old_logprob, dtype=np.float64)
    A = np.asarray(advantages, dtype=np.float64)[:, None]
    B, T = lp.shape
    L = np.clip(np.asarray(lens, dtype=np.int64), 0, T)
    valid = np.arange(T)[None, :] < L[:, None]
    n_tok = int(valid.sum())
    # weight of a token in the aggregate
    if agg == AGG_TOKEN_MEAN:
        w = np.where(valid, 1.0 / max(n_tok, 1), 0.0)
    elif agg == AGG_SEQ_MEAN:
        n_seq = int((L > 0).sum())
        w = np.where(valid, 1.0 / (np.maximum(L, 1)[:, None] * max(n_seq, 1)), 0.0)
    else:
        raise ValueError(agg)
    lp, old = np.where(valid, lp, 0.0), np.where(valid, old, 0.0)      # padding may hold anything: never looked at
    rho = np.exp(lp - old)
    lo, hi = 1.0 - clip_low, 1.0 + clip_high
    clipped = np.clip(rho, lo, hi)
    if form == FORM_PPO:
        s1, s2 = rho * A, clipped * A
        term = np.minimum(s1, s2)
        # inside [lo, hi] both branches are rho A; outside, the clipped branch is flat.  d(rho A)/d logprob = rho A
        active = s1 <= s2
        dterm = np.where(active, rho * A, 0.0)
        is_clipped = ~active
    elif form == FORM_PRINTED:
        m = np.minimum(rho, clipped)                   # = min(rho, hi)
        term = m * A
        flat = rho > hi
        dterm = np.where(flat, 0.0, rho * A)
        is_clipped = flat
    else:
        raise ValueError(form)
    zero = np.zeros_like(lp)
    klt = zero if kl is None else np.where(valid, np.asarray(kl, dtype=np.float64), 0.0)
    ent = zero if entropy is None else np.where(valid, np.asarray(entropy, dtype=np.float64), 0.0)
    pg = float((w * term).sum())
    klm = float((w * klt).sum())
    enm = float((w * ent).sum())
    tokmean = np.where(valid, 1.0 / max(n_tok, 1), 0.0)
    return dict(loss=-pg + beta_kl * klm - beta_ent * enm, pg=pg, kl=klm, entropy=enm,
                clip_frac=float((tokmean * is_clipped).sum()), ratio_mean=float((tokmean * rho).sum()),
                approx_kl=float((tokmean * (old - lp)).sum()), n_tokens=float(n_tok),
                grad=np.where(valid, -w * dterm, 0.0), ratio=rho)
