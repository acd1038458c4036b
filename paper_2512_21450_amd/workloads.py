"""Seeded synthetic rollout workloads (input generation only).

This module draws lengths and tensor values; it holds none of the attention
arithmetic.  Both the GPU path's tests/benchmark and the CPU oracle's tests
take their inputs from here, as numpy arrays (bf16 tensors are ``uint16`` bit
patterns, rounded to nearest-even from fp32 draws).

The shapes stand in for the rollouts the paper runs (Sec. 5.1: GRPO with 4-8
responses per prompt on 2B-7B Qwen-VL policies; Sec. 3.1: the prompt
s_0 = (x_0, y_0) is an image part plus a text part, every sampled trajectory of
a group starts from it).  The paper states no token counts; the ones below are
typical visual-token and response budgets for those models.
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    dtype: str            # "f32" or "bf16": element type of q, k, v
    P: int                # prompts
    G: int                # sampled responses per prompt (the GRPO group)
    Hq: int
    Hkv: int
    d: int
    Lp_cap: int           # row capacity of the prefix KV buffers
    Ls_cap: int           # row capacity of the per-sequence suffix KV buffers
    prefix: tuple         # ("const", L) | ("agentic", n_img, img_tokens, lo, hi)
    suffix: tuple         # ("uniform", hi) | ("lognormal", median, sigma) | ("const", L)
    q_gain: float = 1.0   # q ~ q_gain * N(0,1)
    note: str = ""

    @property
    def B(self) -> int:
        return self.P * self.G

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.d)

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


# The five configurations the throughput metric and the parity bar are stated on.
WORKLOADS = {
    "tiny": Workload("tiny", 1001, "f32", 1, 4, 2, 1, 64, 64, 32,
                     ("const", 64), ("uniform", 32),
                     note="1 prompt x G=4, 2/1 heads, d=64, prefix 48 image + 16 text"),
    "vlm3b": Workload("vlm3b", 1002, "bf16", 8, 8, 16, 2, 128, 452, 512,
                      ("const", 452), ("uniform", 512),
                      note="8 prompts x G=8, 16/2 heads, prefix 324 visual + 128 text"),
    "vlm7b": Workload("vlm7b", 1003, "bf16", 32, 8, 28, 4, 128, 1280, 2048,
                      ("const", 1280), ("uniform", 2048), q_gain=2.0,
                      note="32 prompts x G=8, 28/4 heads, prefix 1024 visual + 256 text"),
    "agentic": Workload("agentic", 1004, "bf16", 16, 8, 28, 4, 128, 1344, 4096,
                        ("agentic", 3, 256, 64, 192), ("lognormal", 300.0, 1.0),
                        note="16 prompts x G=8, 28/4 heads, 3 x (256 image + 64..192 text)"),
    "highbatch": Workload("highbatch", 1005, "bf16", 128, 16, 16, 2, 128, 640, 1024,
                          ("const", 640), ("lognormal", 200.0, 1.0),
                          note="128 prompts x G=16, 16/2 heads, prefix 576 visual + 64 text"),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of ``w`` with some fields replaced (reduced-size parity cases)."""
    return replace(w, **kw)


def _draw_lens(rng: np.random.Generator, kind: tuple, n: int, cap: int) -> np.ndarray:
    if kind[0] == "const":
        lens = np.full(n, kind[1], dtype=np.int64)
    elif kind[0] == "uniform":                      # integers, both ends inclusive
        lens = rng.integers(0, kind[1] + 1, size=n)
    elif kind[0] == "lognormal":                    # median * exp(sigma z), rounded, clipped
        z = rng.standard_normal(n)
        lens = np.rint(np.exp(math.log(kind[1]) + kind[2] * z)).astype(np.int64)
    elif kind[0] == "agentic":                      # n_img x (img_tokens + U{lo..hi} text)
        _, n_img, img, lo, hi = kind
        lens = n_img * img + rng.integers(lo, hi + 1, size=(n, n_img)).sum(axis=1)
    else:
        raise ValueError(kind)
    return np.clip(lens, 0, cap).astype(np.int32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


_CHUNK = 1 << 23  # elements per independently seeded chunk


def _normal_tensor(seed: int, tensor_id: int, shape, dtype: str, gain: float, threads: int):
    """N(0,1)*gain tensor; each 8M-element chunk has its own child seed so the
    values do not depend on how many threads filled it."""
    n = int(np.prod(shape, dtype=np.int64))
    out = np.empty(n, dtype=np.float32 if dtype == "f32" else np.uint16)

    def fill(ci: int):
        lo, hi = ci * _CHUNK, min(n, (ci + 1) * _CHUNK)
        g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tensor_id, ci])))
        x = g.standard_normal(hi - lo, dtype=np.float32)
        if gain != 1.0:
            x *= np.float32(gain)
        out[lo:hi] = x if dtype == "f32" else f32_to_bf16_bits(x)

    n_chunks = (n + _CHUNK - 1) // _CHUNK
    if n_chunks <= 1 or threads <= 1:
        for ci in range(n_chunks):
            fill(ci)
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out.reshape(shape)


def make_inputs(w: Workload, threads: int = 8) -> dict:
    """Draw one batch: lengths first, then q, k_prefix, v_prefix, k_suffix, v_suffix.

    Every row of the KV buffers is filled (also rows beyond the drawn lengths)
    so that a kernel that reads past a length is caught by the parity check.
    """
    rng = np.random.default_rng(w.seed)
    prefix_lens = _draw_lens(rng, w.prefix, w.P, w.Lp_cap)
    suffix_lens = _draw_lens(rng, w.suffix, w.B, w.Ls_cap)
    t = lambda i, shape, gain=1.0: _normal_tensor(w.seed, i, shape, w.dtype, gain, threads)
    return {
        "prefix_lens": prefix_lens,
        "suffix_lens": suffix_lens,
        "q": t(0, (w.B, w.Hq, w.d), w.q_gain),
        "k_prefix": t(1, (w.P, w.Hkv, w.Lp_cap, w.d)),
        "v_prefix": t(2, (w.P, w.Hkv, w.Lp_cap, w.d)),
        "k_suffix": t(3, (w.B, w.Hkv, w.Ls_cap, w.d)),
        "v_suffix": t(4, (w.B, w.Hkv, w.Ls_cap, w.d)),
    }


def make_tree_inputs(seed: int, B: int, Hq: int, Hkv: int, d: int, levels, Ls_cap: int, suffix: tuple,
                     q_gain: float = 1.0, empty: float = 0.0, threads: int = 8) -> dict:
    """One batch for the tree form: shared segments on several levels plus the own suffixes (bf16).

    ``levels``: list of (group, cap, length kind as in Workload.prefix / suffix); level l has B // group
    segments.  ``empty``: fraction of segments and suffixes whose length is forced to zero.  Returns
    ``q``, ``k_suffix``, ``v_suffix``, ``suffix_lens`` and ``levels`` = [(k, v, lens, group)].
    Stands in for a multi-turn rollout (Sec. 5.1, tasks (4)-(5)): the prompt shared by the whole group,
    a first turn (tool call and observation) shared by a sub-group, then each trajectory's own tokens.
    """
    rng = np.random.default_rng(seed)
    lens = []
    for group, cap, kind in levels:
        n = B // group
        lens.append((_draw_lens(rng, kind, n, cap) * (rng.random(n) >= empty)).astype(np.int32))
    suffix_lens = (_draw_lens(rng, suffix, B, Ls_cap) * (rng.random(B) >= empty)).astype(np.int32)
    t = lambda i, shape, gain=1.0: _normal_tensor(seed, i, shape, "bf16", gain, threads)
    out = {"q": t(0, (B, Hq, d), q_gain), "k_suffix": t(1, (B, Hkv, Ls_cap, d)), "v_suffix": t(2, (B, Hkv, Ls_cap, d)),
           "suffix_lens": suffix_lens, "levels": []}
    for i, ((group, cap, _), ln) in enumerate(zip(levels, lens)):
        n = B // group
        out["levels"].append((t(3 + 2 * i, (n, Hkv, cap, d)), t(4 + 2 * i, (n, Hkv, cap, d)), ln, group))
    return out


E4M3_MAX = 448.0          # largest finite e4m3 value


def kv_to_e4m3(x: dict, chunk_rows: int = 8) -> dict:
    """Re-store the K/V buffers of a bf16 batch as e4m3 bytes with one scale per KV head.

    Data preparation only (the quantiser a serving engine runs when it fills an 8-bit KV cache):
    ``k_scale[j]`` = largest |k| of KV head j over prefix and suffix stores / 448, likewise
    ``v_scale``; every element is divided by its head's scale and rounded to the nearest e4m3
    value (ties to even) by torch's CPU conversion.  The attention operates on the stored bytes
    and scales; what they were rounded from plays no further role.
    """
    import torch
    y = dict(x)
    for name in ("k", "v"):
        stores = [x[f"{name}_prefix"], x[f"{name}_suffix"]]
        Hkv = stores[0].shape[1]
        amax = np.zeros(Hkv, np.float32)
        for a in stores:
            for i in range(0, a.shape[0], chunk_rows):
                f = bf16_bits_to_f32(a[i:i + chunk_rows]) if a.dtype == np.uint16 else a[i:i + chunk_rows]
                if f.size:
                    amax = np.maximum(amax, np.abs(f).max(axis=(0, 2, 3)))
        sc = np.where(amax > 0, amax / np.float32(E4M3_MAX), np.float32(1.0)).astype(np.float32)
        for a, key in zip(stores, (f"{name}_prefix", f"{name}_suffix")):
            out = np.empty(a.shape, np.uint8)
            for i in range(0, a.shape[0], chunk_rows):
                f = bf16_bits_to_f32(a[i:i + chunk_rows]) if a.dtype == np.uint16 else a[i:i + chunk_rows]
                t = torch.from_numpy(np.ascontiguousarray(f / sc[None, :, None, None]))
                out[i:i + chunk_rows] = t.clamp_(-E4M3_MAX, E4M3_MAX).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
            y[key] = out
        y[f"{name}_scale"] = sc
    return y


def algorithmic_bytes(w: Workload, prefix_lens, suffix_lens, kv_elem_bytes: int = 0) -> dict:
    """Bytes one decode step has to move, from the realised lengths: each
    prompt's prefix K/V once, each sequence's own suffix K/V once, q in,
    out (fp32) and lse (fp32) out, and the two length arrays.
    ``kv_elem_bytes``: bytes per stored K/V element when it differs from q's (1 for e4m3)."""
    row = w.Hkv * 2 * w.d * (kv_elem_bytes or w.elem_bytes)   # K+V bytes per token, all KV heads
    prefix = int(np.sum(prefix_lens, dtype=np.int64)) * row
    suffix = int(np.sum(suffix_lens, dtype=np.int64)) * row
    io = w.B * w.Hq * w.d * w.elem_bytes + w.B * w.Hq * w.d * 4 + w.B * w.Hq * 4 + 4 * (w.P + w.B)
    return {"prefix": prefix, "suffix": suffix, "io": io, "total": prefix + suffix + io}


def to_pages(x: dict, page_size: int, seed: int, spare_pages: int = 3, poison: bool = True) -> dict:
    """Re-house the suffix K/V of a batch in a shuffled page pool (layout only).

    Returns a copy of ``x`` without k_suffix / v_suffix and with
    ``k_pages`` / ``v_pages`` [n_pages, Hkv, page_size, d], ``block_table``
    [B, max_pages] (int32) and ``page_size``.  Every sequence gets
    ceil(len / page_size) pages, assigned in a seeded random order over the
    pool, which also holds ``spare_pages`` unused pages.  With ``poison`` all
    rows that hold no live key (tails of last pages, spare pages) are NaN and
    unused table entries are -1, so that a reader that strays is caught.
    """
    ks, vs, sl = x["k_suffix"], x["v_suffix"], np.asarray(x["suffix_lens"])
    B, Hkv, Ls_cap, d = ks.shape
    L = np.clip(sl, 0, Ls_cap)
    need = (L + page_size - 1) // page_size
    n_pages = int(need.sum()) + spare_pages
    max_pages = max((Ls_cap + page_size - 1) // page_size, 1)
    order = np.random.default_rng(seed).permutation(n_pages)
    nan_bits = {np.dtype(np.uint16): np.uint16(0x7FC0), np.dtype(np.uint8): np.uint8(0x7F)}.get(
        ks.dtype, np.float32(np.nan))
    fill = nan_bits if poison else ks.dtype.type(0)
    kp = np.full((n_pages, Hkv, page_size, d), fill, dtype=ks.dtype)
    vp = np.full((n_pages, Hkv, page_size, d), fill, dtype=vs.dtype)
    table = np.full((B, max_pages), -1 if poison else 0, dtype=np.int32)
    nxt = 0
    for b in range(B):
        for i in range(int(need[b])):
            pg = int(order[nxt]); nxt += 1
            rows = min(page_size, int(L[b]) - i * page_size)
            kp[pg, :, :rows] = ks[b, :, i * page_size:i * page_size + rows]
            vp[pg, :, :rows] = vs[b, :, i * page_size:i * page_size + rows]
            table[b, i] = pg
    y = {k: v for k, v in x.items() if k not in ("k_suffix", "v_suffix")}
    y.update(k_pages=kp, v_pages=vp, block_table=table, page_size=page_size)
    return y


# ---- vocabulary logits of one decode step (for the per-token policy statistics) ----------
QWEN2_VOCAB = 151936      # vocabulary size in the public configs of the Qwen2 / Qwen2.5 (-VL) models


def make_logits(n_rows: int, vocab: int, seed: int, dtype: str = "bf16", spread: float = 3.0,
                with_ref: bool = False, threads: int = 8) -> dict:
    """Seeded logits ~ spread * N(0,1) [n_rows, vocab], token ids (nine in ten uniform, one in ten
    the row's largest logit, as sampled tokens tend to be likely ones) and, on request, reference
    logits = logits + 0.3 * N(0,1) (a nearby policy)."""
    lg = _normal_tensor(seed, 10, (n_rows, vocab), "f32", spread, threads)
    rng = np.random.default_rng(seed)
    ids = rng.integers(0, vocab, n_rows).astype(np.int32)
    top = rng.random(n_rows) < 0.1
    ids[top] = lg[top].argmax(axis=1).astype(np.int32)
    out = {"token_ids": ids}
    if with_ref:
        ref = lg + _normal_tensor(seed, 11, (n_rows, vocab), "f32", 0.3, threads)
        out["ref_logits"] = ref if dtype == "f32" else f32_to_bf16_bits(ref)
    out["logits"] = lg if dtype == "f32" else f32_to_bf16_bits(lg)
    return out


# ---- rotary embedding inputs of a decode step ----------------------------------------------
def rope_inv_freq(d: int, base: float = 1.0e6) -> np.ndarray:
    """inv_freq[i] = base^(-2i/d), i < d/2, as fp32 (base 1e6 as in the public Qwen2-VL configs)."""
    return (1.0 / (base ** (np.arange(0, d, 2, dtype=np.float64) / d))).astype(np.float32)


def mrope_sections(d: int) -> tuple:
    """Frequency indices per (temporal, height, width) component: 16/24/24 at d = 128, scaled otherwise."""
    half = d // 2
    t = half // 4
    h = (half - t) // 2
    return (t, h, half - t - h)


def make_new_token(w: Workload, x: dict, seed: int) -> dict:
    """The projections of one new token per sequence (q, k_new, v_new ~ N(0,1)) and its three position
    components: text tokens (all equal: prompt length + suffix length) for most sequences, and for
    every fifth sequence an image-patch-like triple (different height / width indices)."""
    t = lambda i, shape: _normal_tensor(seed, i, shape, w.dtype, 1.0, 1)
    pos = (np.repeat(np.asarray(x["prefix_lens"]), w.G) + np.asarray(x["suffix_lens"])).astype(np.int32)
    p3 = np.stack([pos, pos, pos]).astype(np.int32)
    rng = np.random.default_rng(seed)
    img = np.arange(w.B) % 5 == 4
    p3[1, img] = rng.integers(0, 48, int(img.sum()))
    p3[2, img] = rng.integers(0, 48, int(img.sum()))
    return {"q": t(20, (w.B, w.Hq, w.d)), "k_new": t(21, (w.B, w.Hkv, w.d)), "v_new": t(22, (w.B, w.Hkv, w.d)),
            "positions": p3, "inv_freq": rope_inv_freq(w.d), "sections": mrope_sections(w.d)}


# ---- per-token tensors of a finished rollout batch (for the advantage / policy-loss arithmetic) ----------
def make_rollout_tokens(B: int, T: int, G: int, seed: int, n_metrics: int = 2, drift: float = 0.15,
                        lens: tuple = ("lognormal", 300.0, 1.0)) -> dict:
    """Seeded stand-in for what a rollout hands to the policy update: response lengths, the behaviour
    policy's log-prob of every sampled token (negative, a few nats), the target policy's (the former plus a
    small drift, as after a few optimiser steps), per-token KL and entropy (positive), and per-trajectory
    reward metrics (a 0/1 accuracy-like metric and a format-like one in [0, 1])."""
    rng = np.random.default_rng(seed)
    old = -np.abs(rng.standard_normal((B, T), dtype=np.float32)) * 1.5 - 0.01
    lp = (old + drift * rng.standard_normal((B, T), dtype=np.float32)).astype(np.float32)
    metrics = np.empty((n_metrics, B), np.float32)
    metrics[0] = (rng.random(B) < 0.4).astype(np.float32)
    for m in range(1, n_metrics):
        metrics[m] = rng.random(B).astype(np.float32)
    return dict(logprob=lp, old_logprob=old, lens=_draw_lens(rng, lens, B, T),
                kl=np.abs(rng.standard_normal((B, T), dtype=np.float32)) * 0.05,
                entropy=np.abs(rng.standard_normal((B, T), dtype=np.float32)) + 0.1,
                metrics=metrics, weights=np.array([1.0] + [0.5] * (n_metrics - 1), np.float32), G=G)
