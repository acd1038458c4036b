"""fp64 CPU oracle of the per-token policy statistics (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module; the product path never does.

What it defines.  The policy's distribution over the next token is the softmax
of the vocabulary logits (optionally divided by a sampling temperature).  The
later stages of the RL loop consume, per generated token y_t:

  * log pi(y_t | s_0, y_<t): numerator and denominator of the importance ratio
    r_t(theta) (paper Sec. 2.2, "Adaptation for Off-Policy"; Eq. 6 through
    L^PG; Sec. 3.2.2, policy-update stage);
  * the entropy H(pi(. | s_0, y_<t)) of the entropy bonus (Sec. 2.2,
    "Regularization");
  * KL(pi_theta(.|s) || pi_ref(.|s)) over the whole vocabulary, the
    KL-to-reference regulariser (Sec. 2.2 "Regularization" item (1); the
    Omega term under Eq. 6; Sec. 3.2.2 KL_t).

With z = logits / T and w = ref_logits / T (both widened to fp64):
  lse      = ln sum_i exp(z_i)
  logprob  = z_y - lse                      (0 for a negative id: ignored position)
  entropy  = - sum_i p_i ln p_i             with p_i = exp(z_i - lse)
  ref_logprob = w_y - ln sum_i exp(w_i)
  kl       = sum_i p_i (ln p_i - ln r_i)    with r_i = exp(w_i - lse_w)
A logit of -inf (a masked token) has p_i = 0 and contributes nothing to the
entropy and KL sums (the limit p ln p -> 0); a row must keep at least one
finite logit.  A NaN logit is read as a masked token as well (a reading: the
paper says nothing about invalid logits; a mask is the one meaning under which
the other tokens of the row still have a distribution).  Everything is written out as these definitions, in numpy fp64,
one row at a time; nothing is fused or reordered.
"""
from __future__ import annotations

import numpy as np


def _widen(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:                       # bf16 bit patterns: exact widening
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def token_stats_ref(logits, token_ids, inv_temperature=1.0, ref_logits=None):
    """Returns a dict of fp64 arrays [n_rows]: logprob, lse, entropy and, with
    ``ref_logits``, ref_logprob and kl.  ``logits`` [n_rows, V] float32 or
    uint16 (bf16 bits)."""
    n, V = logits.shape
    ids = np.asarray(token_ids).astype(np.int64)
    out = {k: np.zeros(n) for k in ("logprob", "lse", "entropy")}
    if ref_logits is not None:
        out["ref_logprob"] = np.zeros(n)
        out["kl"] = np.zeros(n)
    for b in range(n):
        z = _widen(logits[b]) * float(inv_temperature)
        z = np.where(np.isnan(z), -np.inf, z)       # NaN: a masked token
        m = z.max()
        lse = m + np.log(np.exp(z - m).sum())
        logp = z - lse                              # ln p_i
        p = np.exp(logp)
        out["lse"][b] = lse
        live = p > 0
        out["entropy"][b] = -(p[live] * logp[live]).sum()
        y = int(ids[b])
        if y >= V:
            out["logprob"][b] = np.nan
        elif y >= 0:
            out["logprob"][b] = logp[y]
        if ref_logits is not None:
            w = _widen(ref_logits[b]) * float(inv_temperature)
            w = np.where(np.isnan(w), -np.inf, w)
            mw = w.max()
            logr = w - (mw + np.log(np.exp(w - mw).sum()))
            out["kl"][b] = (p[live] * (logp[live] - logr[live])).sum()
            out["ref_logprob"][b] = np.nan if y >= V else (logr[y] if y >= 0 else 0.0)
    return out
