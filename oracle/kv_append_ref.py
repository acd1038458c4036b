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

8-bit stores: with uint8 stores and per-KV-head factors the appended rows are
quantised to e4m3 bytes (the encoding rl_decode_attn_ref.h describes):

    byte = the e4m3 value nearest to  fp32(x) / factor[j]   (the quotient rounded to fp32),
           ties to the even code, magnitudes above 448 saturate to 448, NaN -> 0x7f

where x is the rotated key (rounded once to fp32) or the value as given.  The
quantiser is the definition written out: a search over the sorted table of
the 127 non-negative e4m3 values.
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


def _e4m3_table():
    """The non-negative e4m3 values in code order (0x00 .. 0x7e), from the format's definition."""
    vals = []
    for code in range(0x7F):
        e, m = code >> 3, code & 7
        vals.append(m * 2.0 ** -9 if e == 0 else (1 + m / 8.0) * 2.0 ** (e - 7))
    return np.array(vals, dtype=np.float64)


def e4m3_round(y):
    """Bytes of the e4m3 values nearest to y (any shape, float): ties to the even code,
    saturation at 448, NaN -> 0x7f, the sign bit kept (also of zeros)."""
    y = np.asarray(y, dtype=np.float64)
    tab = _e4m3_table()
    a = np.minimum(np.abs(y), tab[-1])
    hi = np.clip(np.searchsorted(tab, a, side="left"), 1, len(tab) - 1)      # tab[hi-1] <= a <= tab[hi] (a > 0)
    lo = hi - 1
    dl, dh = a - tab[lo], tab[hi] - a
    code = np.where(dl < dh, lo, np.where(dh < dl, hi, np.where(lo % 2 == 0, lo, hi)))
    code = np.where(np.isnan(y), 0x7F, code).astype(np.uint8)
    return (code | (np.signbit(y).astype(np.uint8) << 7)).astype(np.uint8)


def _quantise(x64, factor):
    """x [B, Hkv, d] -> e4m3 bytes of fp32(x) / factor[j], the quotient taken in fp32."""
    x32 = x64.astype(np.float32)
    f32 = np.ones(x32.shape[1], np.float32) if factor is None else np.asarray(factor, dtype=np.float32)
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        y = x32 / f32[None, :, None]
    assert y.dtype == np.float32
    return e4m3_round(y)


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
                       block_table=None, seq_active=None, k_scale=None, v_scale=None):
    """Returns (q_rot, k_store', v_store', suffix_lens') as new arrays of the input element types.

    Contiguous stores are [B, Hkv, Ls_cap, d]; with ``block_table`` they are page pools
    [n_pages, Hkv, page_size, d].  uint8 stores take e4m3 bytes (factors ``k_scale`` / ``v_scale``
    [Hkv], None = 1)."""
    B, Hq, d = q.shape
    cos, sin = rope_tables(np.asarray(positions), np.asarray(inv_freq, dtype=np.float32), list(sections))
    q_rot = _narrow(rotate(_widen(q), cos, sin), q)
    if k_store.dtype == np.uint8:
        k_rot = _quantise(rotate(_widen(k_new), cos, sin), k_scale)
        v_new = _quantise(_widen(v_new), v_scale)
    else:
        assert k_scale is None and v_scale is None
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
