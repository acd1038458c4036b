"""ctypes front end of the fp64 CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this module; the product path never does.  It compiles
``rl_decode_attn_ref.c`` with gcc on demand and calls it on numpy arrays.
bf16 tensors are passed as ``uint16`` bit patterns.

The definition the C code follows (paper Sec. 2.2, Sec. 3.1 "The MDP of
RLLaVA", Algorithm 1, Sec. 3.2.2 "Sampling stage") is stated in
``rl_decode_attn_ref.h``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "rl_decode_attn_ref.c")
_HDR = os.path.join(_HERE, "rl_decode_attn_ref.h")
_LIB = os.path.join(_HERE, "librl_decode_attn_ref.so")

F32, BF16 = 0, 1
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle shared object with gcc (plain C, OpenMP)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < max(os.path.getmtime(_SRC), os.path.getmtime(_HDR)))
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp, ip = ctypes.c_void_p, ctypes.c_int
        lib.rl_decode_attn_ref_f64.restype = ip
        lib.rl_decode_attn_ref_f64.argtypes = [ip] * 8 + [ctypes.c_double] + [vp] * 9 + [
            vp, ctypes.c_int64, ip, ctypes.POINTER(ip)]
        lib.rl_decode_attn_ref_kv8_f64.restype = ip
        lib.rl_decode_attn_ref_kv8_f64.argtypes = [ip, vp, vp] + [ip] * 7 + [ctypes.c_double] + [vp] * 9 + [
            vp, ctypes.c_int64, ip, ctypes.POINTER(ip)]
        lib.rl_e4m3_to_f64_ref.restype = ctypes.c_double
        lib.rl_e4m3_to_f64_ref.argtypes = [ctypes.c_uint8]
        lib.rl_lse_combine_ref_f64.restype = None
        lib.rl_lse_combine_ref_f64.argtypes = [ip, ip, vp, vp, vp, vp]
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _elem(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    raise TypeError(f"oracle takes float32 or uint16 (bf16 bits), got {a.dtype}")


def e4m3_to_f64(bits) -> np.ndarray:
    """Values of e4m3 bytes (any shape), by the C oracle's decoder."""
    lib = _load()
    b = np.asarray(bits, dtype=np.uint8)
    return np.array([lib.rl_e4m3_to_f64_ref(int(x)) for x in b.ravel()], dtype=np.float64).reshape(b.shape)


def decode_attn_ref(q, k_prefix, v_prefix, prefix_lens, k_suffix, v_suffix, suffix_lens,
                    scale, G, rows=None, n_threads=0, return_threads=False, k_scale=None, v_scale=None):
    """out[B,Hq,d], lse[B,Hq] in fp64.  Shapes as in rl_decode_attn_ref.h.

    ``rows``: optional int array [n,2] of (b, h) pairs; then only those entries
    are computed and the rest of the returned arrays is NaN.

    K/V stores of dtype uint8 hold e4m3 bytes; ``k_scale`` / ``v_scale`` ([Hkv]
    float32 or None) are then the per-KV-head dequantisation factors.
    """
    lib = _load()
    q = np.ascontiguousarray(q)
    et = _elem(q)
    B, Hq, d = q.shape
    P, Hkv, Lp_cap, _ = k_prefix.shape
    Ls_cap = k_suffix.shape[2]
    assert B == P * G and k_suffix.shape[0] == B and k_suffix.shape[1] == Hkv
    arrs = [np.ascontiguousarray(a) for a in (k_prefix, v_prefix, k_suffix, v_suffix)]
    kv8 = arrs[0].dtype == np.uint8
    for a in arrs:
        assert (a.dtype == np.uint8) if kv8 else (_elem(a) == et)
    if not kv8:
        assert k_scale is None and v_scale is None, "scales belong to e4m3 stores"
    ksc = None if k_scale is None else np.ascontiguousarray(k_scale, dtype=np.float32)
    vsc = None if v_scale is None else np.ascontiguousarray(v_scale, dtype=np.float32)
    assert ksc is None or ksc.shape == (Hkv,)
    assert vsc is None or vsc.shape == (Hkv,)
    pl = np.ascontiguousarray(prefix_lens, dtype=np.int32)
    sl = np.ascontiguousarray(suffix_lens, dtype=np.int32)
    assert pl.shape == (P,) and sl.shape == (B,)
    fill = np.nan if rows is not None else 0.0
    out = np.full((B, Hq, d), fill, dtype=np.float64)
    lse = np.full((B, Hq), fill, dtype=np.float64)
    r = None
    n_rows = 0
    if rows is not None:
        r = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 2)
        n_rows = r.shape[0]
    used = ctypes.c_int(0)
    tail = (P, G, Hq, Hkv, d, Lp_cap, Ls_cap, float(scale),
            _ptr(q), _ptr(arrs[0]), _ptr(arrs[1]), _ptr(pl), _ptr(arrs[2]), _ptr(arrs[3]), _ptr(sl),
            _ptr(out), _ptr(lse), _ptr(r), n_rows, int(n_threads), ctypes.byref(used))
    if kv8:
        rc = lib.rl_decode_attn_ref_kv8_f64(et, _ptr(ksc), _ptr(vsc), *tail)
    else:
        rc = lib.rl_decode_attn_ref_f64(et, *tail)
    if rc != 0:
        raise ValueError(f"oracle returned {rc}")
    if return_threads:
        return out, lse, used.value
    return out, lse


def lse_combine_ref(o_parts, lse_parts):
    """Merge n partials (o_parts [n,d], lse_parts [n]) -> (out [d], lse)."""
    lib = _load()
    o = np.ascontiguousarray(o_parts, dtype=np.float64)
    l = np.ascontiguousarray(lse_parts, dtype=np.float64)
    n, d = o.shape
    out = np.zeros(d, dtype=np.float64)
    res = np.zeros(1, dtype=np.float64)
    lib.rl_lse_combine_ref_f64(n, d, _ptr(o), _ptr(l), _ptr(out), _ptr(res))
    return out, float(res[0])


def gather_pages(pages, block_table, suffix_lens, Ls_cap):
    """Contiguous suffix store [B, Hkv, Ls_cap, d] from a paged one.

    ``pages`` [n_pages, Hkv, page_size, d]; key n of sequence b is row
    n % page_size of page block_table[b, n // page_size].  Rows at or beyond
    suffix_lens[b] are left zero.  Plain indexing, no arithmetic on values.
    """
    n_pages, Hkv, ps, d = pages.shape
    B = block_table.shape[0]
    out = np.zeros((B, Hkv, Ls_cap, d), dtype=pages.dtype)
    for b in range(B):
        L = int(min(max(int(suffix_lens[b]), 0), block_table.shape[1] * ps, Ls_cap))
        for i in range((L + ps - 1) // ps):
            rows = min(ps, L - i * ps)
            out[b, :, i * ps:i * ps + rows, :] = pages[int(block_table[b, i]), :, :rows, :]
    return out


def decode_attn_paged_ref(q, k_prefix, v_prefix, prefix_lens, k_pages, v_pages, block_table, suffix_lens,
                          seq_active, scale, G, rows=None, n_threads=0, k_scale=None, v_scale=None):
    """The paged-suffix call by its definition: gather every sequence's pages
    in table order and evaluate the attention of the contiguous layout;
    sequences marked finished (seq_active[b] == 0) get out = 0, lse = -inf."""
    ps = k_pages.shape[2]
    sl = np.clip(np.asarray(suffix_lens, dtype=np.int64), 0, block_table.shape[1] * ps).astype(np.int32)
    cap = max(int(sl.max(initial=0)), 1)
    ks = gather_pages(k_pages, block_table, sl, cap)
    vs = gather_pages(v_pages, block_table, sl, cap)
    out, lse = decode_attn_ref(q, k_prefix, v_prefix, prefix_lens, ks, vs, sl, scale, G, rows=rows,
                               n_threads=n_threads, k_scale=k_scale, v_scale=v_scale)
    if seq_active is not None:
        dead = np.asarray(seq_active) == 0
        out[dead] = 0.0
        lse[dead] = -np.inf
    return out, lse


def concat_levels(levels, B):
    """Per-sequence key lists of a tree of shared segments, written out.

    ``levels``: list of (k, v, lens, group): stores [n_seg, Hkv, cap, d], lengths [n_seg], and the number
    of consecutive sequences that share one segment (n_seg * group == B): sequence b attends to segment
    b // group of every level.  Returns (k_cat, v_cat, cat_lens): [B, Hkv, cap_total, d] stores that hold,
    for each sequence, the live rows of its segment of level 0, then of level 1, ... one after the other
    (lengths clamped to [0, cap]), and the number of rows per sequence.  Plain indexing, no arithmetic on
    values.  With these as a "prefix" of its own per sequence (group size 1) the attention over a tree of
    shared prefixes is, by definition, the attention over the concatenated keys.
    """
    assert len(levels) >= 1
    k0 = levels[0][0]
    Hkv, d = k0.shape[1], k0.shape[3]
    cap_total = max(sum(int(k.shape[2]) for k, _, _, _ in levels), 1)
    k_cat = np.zeros((B, Hkv, cap_total, d), dtype=k0.dtype)
    v_cat = np.zeros((B, Hkv, cap_total, d), dtype=k0.dtype)
    cat_lens = np.zeros(B, dtype=np.int32)
    for b in range(B):
        pos = 0
        for k, v, lens, group in levels:
            assert k.shape[0] * group == B and k.shape == v.shape
            s = b // group
            L = int(min(max(int(lens[s]), 0), k.shape[2]))
            k_cat[b, :, pos:pos + L, :] = k[s, :, :L, :]
            v_cat[b, :, pos:pos + L, :] = v[s, :, :L, :]
            pos += L
        cat_lens[b] = pos
    return k_cat, v_cat, cat_lens


def decode_attn_tree_ref(q, levels, k_suffix, v_suffix, suffix_lens, scale, rows=None, n_threads=0):
    """Attention of every sequence over the segments it shares on each level of a prefix tree
    (see concat_levels) followed by its own suffix: the two-pass fp64 attention over the concatenated keys."""
    B = q.shape[0]
    if not levels:
        Hkv, d = k_suffix.shape[1], k_suffix.shape[3]
        kc = np.zeros((B, Hkv, 1, d), dtype=k_suffix.dtype)
        return decode_attn_ref(q, kc, kc, np.zeros(B, np.int32), k_suffix, v_suffix, suffix_lens, scale, 1,
                               rows=rows, n_threads=n_threads)
    k_cat, v_cat, cat_lens = concat_levels(levels, B)
    return decode_attn_ref(q, k_cat, v_cat, cat_lens, k_suffix, v_suffix, suffix_lens, scale, 1,
                           rows=rows, n_threads=n_threads)
