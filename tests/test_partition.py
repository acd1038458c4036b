"""The static work partition of the shared-prefix path, checked on the host:
every tile is processed exactly once, partial slots are unique, and the
combine step reads exactly the partials the walk produces, in line order."""
import ctypes

import numpy as np
import pytest

from paper_2512_21450_amd import binding as B
from paper_2512_21450_amd import workloads as wl

TK = 32
_f = B._lib.rl_decode_attn_debug_partition
_f.restype = ctypes.c_int64
_f.argtypes = [ctypes.c_int32] * 6 + [ctypes.c_void_p] * 2 + [ctypes.c_void_p, ctypes.c_int64,
                                                               ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]


_g = B._lib.rl_decode_attn_debug_partition_on
_g.restype = ctypes.c_int64
_g.argtypes = [ctypes.c_int32] * 7 + [ctypes.c_void_p] * 2 + [ctypes.c_void_p, ctypes.c_int64,
                                                               ctypes.c_void_p, ctypes.c_int64, ctypes.c_void_p]
_pairs = B._lib.rl_decode_attn_debug_pairs
_pairs.restype = ctypes.c_int32
_pairs.argtypes = [ctypes.c_int32]


def partition(P, G, Hkv, Lp_cap, Ls_cap, plens, slens, R=8, cus=256):
    plens = np.ascontiguousarray(plens, np.int32)
    slens = np.ascontiguousarray(slens, np.int32)
    cap = 4 * (P * (G + 2) * Hkv + 8 * 512) + 16
    runs = np.zeros((cap, 8), np.int32)
    parts = np.zeros((cap, 6), np.int32)
    npart = ctypes.c_int64(0)
    if cus == 256:
        nr = _f(P, G, Hkv, R, Lp_cap, Ls_cap, plens.ctypes.data, slens.ctypes.data, runs.ctypes.data, cap,
                parts.ctypes.data, cap, ctypes.byref(npart))
    else:
        nr = _g(cus, P, G, Hkv, R, Lp_cap, Ls_cap, plens.ctypes.data, slens.ctypes.data, runs.ctypes.data, cap,
                parts.ctypes.data, cap, ctypes.byref(npart))
    assert 0 <= nr <= cap and npart.value <= cap
    return runs[:nr], parts[:npart.value]


def check(P, G, Hkv, Lp_cap, Ls_cap, plens, slens, R=8, cus=256):
    """R: query rows per KV group; above 64 the prefix units are (prompt, KV head, row half), and twin pairs
    (c and c ^ 8, on one die) walk the same tiles, one for the even row half and one for the odd one.
    cus: compute units of the device the partition is made for."""
    runs, parts = partition(P, G, Hkv, Lp_cap, Ls_cap, plens, slens, R, cus)
    NC = _pairs(cus)                              # workgroup pairs
    HkvP = Hkv * (4 if R > 128 else 2 if R > 64 else 1)
    tp = -(-np.clip(plens, 0, Lp_cap) // TK)
    ts = -(-np.clip(slens, 0, Ls_cap) // TK)
    # coverage: each unit's tiles [0, T) are tiled by its runs without gap or overlap
    for kind, counts, heads in ((0, tp, HkvP), (1, ts, Hkv)):
        rk = runs[runs[:, 0] == kind]
        seen = {}
        for _, major, j, t0, n, w, v, slot in rk:
            assert n > 0
            seen.setdefault((major, j), []).append((t0, n))
        for major, T in enumerate(counts):
            for j in range(heads):
                segs = sorted(seen.pop((major, j), []))
                pos = 0
                for t0, n in segs:
                    assert t0 == pos, (kind, major, j, segs)
                    pos += n
                assert pos == T, (kind, major, j, segs, T)
        assert not seen
    # slots: unique per kind, inside the workspace the library sizes
    for kind, nslots in ((0, P * HkvP + 512), (1, P * G * Hkv + 8 * 256)):
        sl = runs[runs[:, 0] == kind][:, 7]
        assert len(set(sl.tolist())) == len(sl)
        assert sl.size == 0 or (sl.min() >= 0 and sl.max() < nslots)
    assert runs.shape[0] == 0 or (runs[:, 5].min() >= 0 and runs[:, 5].max() < 2 * NC)
    # the combine enumeration == the set of runs, and per unit in increasing line order
    key_r = sorted((int(k), int(m), int(j), int(w), int(v), int(s)) for k, m, j, _, _, w, v, s in runs)
    key_p = sorted(tuple(int(x) for x in row) for row in parts)
    assert key_r == key_p
    # balance: the two workgroups of a pair (w and 256 + w share a compute unit) together hold
    # an equal share of the prefix tiles and of the suffix tiles, up to rounding
    npt, nst = int(tp.sum()) * HkvP, int(ts.sum()) * Hkv
    dual = R > 64 and NC > 1
    # a batch of fewer than 2048 tiles works with half the pairs (down to 32), the first workgroups of the grid;
    # the others stay idle
    NC = NC // 2 if npt + nst < 2048 and NC >= 64 and not dual else NC
    assert runs.shape[0] == 0 or runs[:, 5].max() < 2 * NC
    for kind, total in ((0, npt), (1, nst)):
        load = np.zeros(NC, np.int64)
        rk = runs[runs[:, 0] == kind]
        np.add.at(load, rk[:, 5] % NC, rk[:, 4])
        assert load.sum() == total
        if dual and kind == 0:                    # twins hold equal shares of the line of half the units
            assert (total // 2) // (NC // 2) <= load.min() and load.max() <= -(-(total // 2) // (NC // 2))
        else:
            assert load.max() <= -(-total // NC) and load.min() >= total // NC
    if dual:
        # twin pairs walk the same prefix tiles (the split inside a pair may differ by the pairs' suffix shares),
        # for row halves 2k (the pair without the twin bit) and 2k + 1
        tb = min(3, NC.bit_length() - 2)
        pre = runs[runs[:, 0] == 0]
        tiles = {0: {}, 1: {}}
        for _, major, j, t0, n, w, _, _ in pre:
            side = ((w % NC) >> tb) & 1
            assert j % 2 == side
            share = (w % NC) & ~(1 << tb)
            tiles[side].setdefault(share, set()).update((major, j - side, t) for t in range(t0, t0 + n))
        assert tiles[0] == tiles[1]
    # inside a pair the heavier line is shared: the second workgroup has prefix tiles only if the first
    # has no suffix tiles, and the two then differ by less than two tiles' weight
    WP, WS = (14 if npt + nst < 16384 and 6 * npt <= 4 * nst else 6), 4   # small suffix-heavy batches weigh prefix tiles more
    wa, wb = np.zeros(NC, np.int64), np.zeros(NC, np.int64)
    a_suffix, b_prefix = np.zeros(NC, np.int64), np.zeros(NC, np.int64)
    for kind, _, _, _, n, w, _, _ in runs:
        wt = n * (WP if kind == 0 else WS)
        if w < NC:
            wa[w] += wt
            a_suffix[w] += n if kind == 1 else 0
        else:
            wb[w - NC] += wt
            b_prefix[w - NC] += n if kind == 0 else 0
    assert not ((a_suffix > 0) & (b_prefix > 0)).any()
    shared = (a_suffix > 0) | (b_prefix > 0)
    assert (np.abs(wa - wb)[shared] <= 2 * max(WP, WS)).all()
    return runs


@pytest.mark.parametrize("name", ["vlm3b", "vlm7b", "agentic", "highbatch"])
def test_partition_of_the_benchmark_workloads(name):
    w = wl.WORKLOADS[name]
    rng = np.random.default_rng(w.seed)
    pl = wl._draw_lens(rng, w.prefix, w.P, w.Lp_cap)
    sl = wl._draw_lens(rng, w.suffix, w.B, w.Ls_cap)
    runs = check(w.P, w.G, w.Hkv, w.Lp_cap, w.Ls_cap, pl, sl, R=w.G * w.Hq // w.Hkv)
    assert len(runs) > 0
    if name == "vlm3b":                           # 1264 tiles: half the pairs, the first 256 workgroups; the others idle
        assert runs[:, 5].max() == 255
    else:
        assert runs[:, 5].max() == 511
    if name == "highbatch":                       # 128 rows per KV group: twice the prefix units
        assert runs[runs[:, 0] == 0][:, 2].max() == 2 * w.Hkv - 1


def test_prefix_heavy_batches_put_prefix_tiles_on_both_workgroups():
    # long prompts, a few generated tokens: the first steps of a rollout, or short answers
    w = wl.WORKLOADS["vlm7b"]
    runs = check(w.P, w.G, w.Hkv, w.Lp_cap, w.Ls_cap, [w.Lp_cap] * w.P, [5] * w.B)
    pre = runs[runs[:, 0] == 0]
    on_b = pre[pre[:, 5] >= 256][:, 4].sum()
    assert 0.35 * pre[:, 4].sum() < on_b < 0.5 * pre[:, 4].sum()
    runs = check(w.P, w.G, w.Hkv, w.Lp_cap, w.Ls_cap, [w.Lp_cap] * w.P, [0] * w.B)     # no suffix at all: halves
    pre = runs[runs[:, 0] == 0]
    assert abs(int(pre[pre[:, 5] >= 256][:, 4].sum()) * 2 - int(pre[:, 4].sum())) <= 256
    # suffix-heavy: every prefix tile on the first workgroup of a pair
    rng = np.random.default_rng(w.seed)
    pl = wl._draw_lens(rng, w.prefix, w.P, w.Lp_cap)
    sl = wl._draw_lens(rng, w.suffix, w.B, w.Ls_cap)
    runs = check(w.P, w.G, w.Hkv, w.Lp_cap, w.Ls_cap, pl, sl)
    assert not (runs[runs[:, 0] == 0][:, 5] >= 256).any()


def test_partition_edge_cases():
    rng = np.random.default_rng(0)
    # nothing at all, prefix only, suffix only, single tile, fewer tiles than workgroups
    check(2, 3, 2, 64, 64, [0, 0], [0] * 6)
    check(2, 3, 2, 64, 64, [64, 1], [0] * 6)
    check(2, 3, 2, 64, 64, [0, 0], [5, 0, 64, 0, 0, 33])
    check(1, 1, 1, 40, 40, [1], [0])
    check(3, 2, 4, 100, 100, [100, 0, 31], [0, 100, 1, 32, 33, 0])
    # zero-length prompts/sequences at the start, in the middle and at the end
    check(5, 2, 2, 500, 500, [0, 300, 0, 0, 77], [0, 0, 400, 0, 12, 0, 0, 500, 0, 0])
    # lengths outside [0, cap] clamp
    check(2, 2, 2, 100, 50, [-5, 1000], [999, -1, 50, 3])
    for _ in range(20):
        P, G, Hkv = int(rng.integers(1, 40)), int(rng.integers(1, 9)), int(rng.integers(1, 5))
        Lp_cap, Ls_cap = int(rng.integers(0, 3000)), int(rng.integers(0, 5000))
        pl = rng.integers(0, Lp_cap + 1, P) * (rng.random(P) < 0.8)
        sl = rng.integers(0, Ls_cap + 1, P * G) * (rng.random(P * G) < 0.7)
        check(P, G, Hkv, Lp_cap, Ls_cap, pl, sl, R=int(rng.choice([7, 56, 64, 65, 128, 129, 256])))


def test_partition_of_long_lines():
    """Millions of tiles on a line: the owner of a line position comes from a float quotient settled by exact
    steps, which has to hold where the quotient's rounding is coarsest."""
    rng = np.random.default_rng(5)
    P, G, Hkv = 512, 8, 4
    pl = rng.integers(7000, 8193, P)
    sl = rng.integers(0, 8193, P * G)
    check(P, G, Hkv, 8192, 8192, pl, sl, R=56)
    check(64, 16, 2, 100000, 60000, rng.integers(90000, 100001, 64), rng.integers(0, 60001, 64 * 16), R=128, cus=128)


def test_pairs_follow_the_compute_unit_count():
    # the largest power of two that is at most the device's compute units and at most 256
    assert [_pairs(c) for c in (256, 304, 255, 128, 100, 64, 33, 32, 2, 1)] == [256, 256, 128, 128, 64, 64, 32, 32, 2, 1]
    assert _pairs(0) < 0 and _pairs(-3) < 0


@pytest.mark.parametrize("cus", [128, 64, 32, 100, 1])
def test_partition_for_other_compute_unit_counts(cus):
    """A partition of the chip (128, 64 or 32 compute units) or any other count: every tile once, slots
    unique and inside the workspace, the combine reads what the walk writes, pairs evenly loaded."""
    w = wl.WORKLOADS["vlm7b"]
    rng = np.random.default_rng(w.seed)
    pl = wl._draw_lens(rng, w.prefix, w.P, w.Lp_cap)
    sl = wl._draw_lens(rng, w.suffix, w.B, w.Ls_cap)
    check(w.P, w.G, w.Hkv, w.Lp_cap, w.Ls_cap, pl, sl, R=w.G * w.Hq // w.Hkv, cus=cus)
    check(w.P, w.G, w.Hkv, w.Lp_cap, w.Ls_cap, [w.Lp_cap] * w.P, [5] * w.B, cus=cus)
    check(3, 2, 4, 100, 100, [100, 0, 31], [0, 100, 1, 32, 33, 0], cus=cus)
    rng = np.random.default_rng(cus)
    for _ in range(6):
        P, G, Hkv = int(rng.integers(1, 40)), int(rng.integers(1, 9)), int(rng.integers(1, 5))
        Lp_cap, Ls_cap = int(rng.integers(0, 3000)), int(rng.integers(0, 5000))
        pl = rng.integers(0, Lp_cap + 1, P) * (rng.random(P) < 0.8)
        sl = rng.integers(0, Ls_cap + 1, P * G) * (rng.random(P * G) < 0.7)
        check(P, G, Hkv, Lp_cap, Ls_cap, pl, sl, R=int(rng.choice([7, 56, 64, 65, 128, 129, 256])), cus=cus)
