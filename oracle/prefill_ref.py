"""fp64 CPU oracle of the shared-prefix prefill attention (TEST INFRASTRUCTURE ONLY: tests, the
smoke check and the benchmark's CPU leg may import this module; the product path never does).

Before the rollout of Algorithm 1 can sample its K trajectories, the prompt s_0 = (x_0, y_0)
(Sec. 3.1) has to be run through the policy once; because the K samples of a group share s_0
(Sec. 3.2.2 "Sampling stage"), that pass is needed once per prompt, not once per trajectory, and its
keys and values become the shared prefix store of the decode step.  For one attention layer it is
causal scaled dot-product attention with grouped-query heads over the prompt's own tokens (the
paper prints no formula; this is the definition the policy models of Sec. 5.1 use):

    j = h / (Hq/Hkv)
    s_in      = scale * <q[p,i,h,:], k[p,j,n,:]>             n <= i < L_p
    lse[p,i,h] = ln sum_{n<=i} exp(s_in)
    out[p,i,h,:] = sum_{n<=i} exp(s_in - lse) v[p,j,n,:]

Positions i >= L_p are padding: their rows are returned as NaN (the GPU call does not write them).
Inputs are widened exactly to fp64; one matrix product per (prompt, head) for the scores, a
masked two-pass softmax, one for the values: numpy library steps, nothing blocked or fused.
"""
from __future__ import annotations

import numpy as np


def _widen(a):
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def prefill_attn_ref(q, k, v, lens, scale):
    """q [P, L_cap, Hq, d]; k, v [P, Hkv, L_cap, d]; lens [P] -> out [P, L_cap, Hq, d], lse [P, L_cap, Hq] (fp64)."""
    P, Lc, Hq, d = q.shape
    Hkv = k.shape[1]
    r = Hq // Hkv
    out = np.full((P, Lc, Hq, d), np.nan)
    lse = np.full((P, Lc, Hq), np.nan)
    for p in range(P):
        L = int(min(max(int(lens[p]), 0), Lc))
        if L == 0:
            continue
        causal = np.tril(np.ones((L, L), bool))
        for h in range(Hq):
            j = h // r
            Q, K, V = _widen(q[p, :L, h]), _widen(k[p, j, :L]), _widen(v[p, j, :L])
            S = np.where(causal, scale * (Q @ K.T), -np.inf)
            m = S.max(axis=1, keepdims=True)
            E = np.exp(S - m)
            z = E.sum(axis=1, keepdims=True)
            out[p, :L, h] = (E / z) @ V
            lse[p, :L, h] = (m + np.log(z))[:, 0]
    return out, lse
