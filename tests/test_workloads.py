"""Host-side checks of the seeded input recipes (no GPU)."""
import numpy as np

from paper_2512_21450_amd import workloads as wl


def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.1415927, 0.0], np.float32)
    b = wl.f32_to_bf16_bits(f)
    # 1.00390625 = 1 + 2^-8 is a tie between 1.0 (even mantissa) and 1.0078125 -> 1.0
    # 1.01171875 = 1 + 3*2^-8 is a tie between 1.0078125 (odd) and 1.015625 (even) -> up
    assert b.tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC020, 0x4049, 0x0000]
    back = wl.bf16_bits_to_f32(b)
    assert back.tolist() == [1.0, 1.0, 1.015625, -2.5, 3.140625, 0.0]
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    r = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(x))
    assert np.all(np.abs(r - x) <= np.abs(x) * 2.0 ** -8)


def test_presets_match_the_stated_shapes():
    W = wl.WORKLOADS
    assert (W["tiny"].B, W["tiny"].Hq, W["tiny"].Hkv, W["tiny"].d, W["tiny"].dtype) == (4, 2, 1, 64, "f32")
    assert W["tiny"].scale == 0.125
    assert (W["vlm3b"].B, W["vlm3b"].Hq, W["vlm3b"].Hkv, W["vlm3b"].Lp_cap) == (64, 16, 2, 452)
    assert (W["vlm7b"].B, W["vlm7b"].Hq, W["vlm7b"].Hkv, W["vlm7b"].Lp_cap, W["vlm7b"].Ls_cap) == (256, 28, 4, 1280, 2048)
    assert (W["agentic"].B, W["agentic"].Ls_cap) == (128, 4096)
    assert (W["highbatch"].B, W["highbatch"].Hq, W["highbatch"].Hkv) == (2048, 16, 2)


def test_lengths_follow_the_recipes():
    for name, w in wl.WORKLOADS.items():
        rng = np.random.default_rng(w.seed)
        pl = wl._draw_lens(rng, w.prefix, w.P, w.Lp_cap)
        sl = wl._draw_lens(rng, w.suffix, w.B, w.Ls_cap)
        assert pl.dtype == np.int32 and sl.dtype == np.int32
        assert pl.min() >= 0 and pl.max() <= w.Lp_cap and sl.min() >= 0 and sl.max() <= w.Ls_cap
        if w.prefix[0] == "const":
            assert np.all(pl == w.prefix[1])
    w = wl.WORKLOADS["agentic"]
    rng = np.random.default_rng(w.seed)
    pl = wl._draw_lens(rng, w.prefix, w.P, w.Lp_cap)
    assert np.all(pl >= 3 * 256 + 3 * 64) and np.all(pl <= 3 * 256 + 3 * 192)
    sl = wl._draw_lens(np.random.default_rng(1), ("lognormal", 300.0, 1.0), 20000, 4096)
    assert abs(np.median(sl) - 300) < 15 and sl.max() == 4096
    su = wl._draw_lens(np.random.default_rng(2), ("uniform", 32), 20000, 32)
    assert su.min() == 0 and su.max() == 32 and abs(su.mean() - 16) < 0.5


def test_make_inputs_is_deterministic_and_thread_independent():
    w = wl.scaled(wl.WORKLOADS["vlm7b"], P=2, G=2, Lp_cap=64, Ls_cap=9000)   # > one chunk
    a = wl.make_inputs(w, threads=1)
    b = wl.make_inputs(w, threads=4)
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    assert a["q"].dtype == np.uint16 and a["q"].shape == (4, 28, 128)
    q = wl.bf16_bits_to_f32(a["q"])
    k = wl.bf16_bits_to_f32(a["k_suffix"])
    assert abs(q.std() - 2.0) < 0.05 and abs(k.std() - 1.0) < 0.01 and abs(k.mean()) < 0.01
    t = wl.make_inputs(wl.WORKLOADS["tiny"])
    assert t["q"].dtype == np.float32 and t["prefix_lens"].tolist() == [64]


def test_algorithmic_bytes_formula():
    w = wl.WORKLOADS["vlm7b"]
    pl = np.full(w.P, 1280, np.int32)
    sl = np.full(w.B, 1024, np.int32)
    ab = wl.algorithmic_bytes(w, pl, sl)
    assert ab["prefix"] == 32 * 1280 * 2048            # 83.9 MB, once per prompt
    assert ab["suffix"] == 256 * 1024 * 2048           # 536.9 MB
    assert ab["io"] == 256 * 28 * 128 * 2 + 256 * 28 * 128 * 4 + 256 * 28 * 4 + 4 * (32 + 256)
    assert ab["total"] == ab["prefix"] + ab["suffix"] + ab["io"]
