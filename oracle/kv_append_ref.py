"""fp64 CPU oracle of the decode-step state transition (TEST INFRASTRUCTURE ONLY).

Only tests and the smoke check may import this module; the product path never
does.

The transition appends the chosen token to the state (paper Sec. 2.2; Sec. 3.1
"The MDP of RLLaVA", item (3)); for one attention layer: rotate the new token's
query and key by its position, append the rotated key and the value to the
sequence's suffix store, count it.  The paper prints no rotary formula; this is
the RoFormer rotary embedding in the rotate-half pairing with three position
components assigned to consecutive sections of the frequency index (the public
definition of the multimodal variant used by the policy models of Sec. 5.1):

    angle(b, i) = positions[c(i), b] * inv_freq[i]          (fp64 product of the given values)
    y[i]        = x[i] cos - x[i + d/2] sin
    y[i + d/2]  = x[i + d/2] cos + x[i] sin

cos and sin are rounded to fp32 before use (the precision the definition's
tables are kept in); everything else is fp64; outputs are rounded to the
element type (bf16: nearest even) at the end.  Written as plain loops over
sequences with numpy row arithmetic.
"""
from __future__ import annotations

import numpy as np


def _widen(a):
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _narrow(x64, like):
    x = x64.astype(np.float32)
    if like.dtype == np.uint16:                   # fp32 -> bf16, round to nearest even (finite values)
        u = x.view(np.uint32)
        return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    return x


def rope_tables(positions, inv_freq, sections):
    """cos, sin [B, d/2] as fp32 values (held in fp64 arrays)."""
    half = inv_freq.shape[0]
    assert sum(sections) == half
    comp = np.repeat(np.arange(3), sections)                      # position component of each frequency index
    ang = positions[comp, :].T.astype(np.float64) * inv_freq.astype(np.float64)[None, :]
    return np.cos(ang).astype(np.float32).astype(np.float64), np.sin(ang).astype(np.float32).astype(np.float64)


def rotate(x, cos, sin):
    """x [B, H, d] (fp64), cos/sin [B, d/2] -> rotated copy."""
    half = x.shape[2] // 2
    lo, hi = x[:, :, :half], x[:, :, half:]
    c, s = cos[:, None, :], sin[:, None, :]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=2)


def kv_append_rope_ref(q, k_new, v_new, positions, inv_freq, sections, k_store, v_store, suffix_lens,
                       block_table=None, seq_active=None):
    """Returns (q_rot, k_store', v_store', suffix_lens') as new arrays of the input element types.

    Contiguous stores are [B, Hkv, Ls_cap, d]; with ``block_table`` they are page pools
    [n_pages, Hkv, page_size, d]."""
    B, Hq, d = q.shape
    cos, sin = rope_tables(np.asarray(positions), np.asarray(inv_freq, dtype=np.float32), list(sections))
    q_rot = _narrow(rotate(_widen(q), cos, sin), q)
    k_rot = _narrow(rotate(_widen(k_new), cos, sin), k_new)
    ks, vs, lens = k_store.copy(), v_store.copy(), np.asarray(suffix_lens).astype(np.int32).copy()
    for b in range(B):
        if seq_active is not None and not seq_active[b]:
            continue
        n = int(lens[b])
        if block_table is None:
            if not 0 <= n < ks.shape[2]:
                continue
            ks[b, :, n, :] = k_rot[b]
            vs[b, :, n, :] = v_new[b]
        else:
            ps = ks.shape[2]
            if not 0 <= n < block_table.shape[1] * ps:
                continue
            pg = int(min(max(int(block_table[b, n // ps]), 0), ks.shape[0] - 1))
            ks[pg, :, n % ps, :] = k_rot[b]
            vs[pg, :, n % ps, :] = v_new[b]
        lens[b] = n + 1
    return q_rot, ks, vs, lens
