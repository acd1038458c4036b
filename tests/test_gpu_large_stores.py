"""GPU parity on K/V stores, page pools and outputs larger than 4 GiB (more than 2^31 elements).

A serving engine sizes the stores of a layer for the whole batch at full capacity; on a 288 GB device
a single store passes 4 GiB easily.  These cases put live rows behind byte offset 2^32 (and element
offset 2^31) of every tensor the library indexes, so that an offset computed in 32 bits anywhere would
read or write the wrong rows.  The device tensors are allocated at full capacity and only the live rows
are filled; the fp64 oracle, whose result does not depend on a capacity, runs on compact host copies of
the same rows.  Tolerances are those of the other parity tests.
"""
import numpy as np
import pytest

from paper_2512_21450_amd import workloads as wl
from tests import util

pytestmark = pytest.mark.gpu
FOUR_GIB = 1 << 32


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2512_21450_amd import binding
    return binding


def bf(a):
    import torch
    return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)


def grow(compact, cap, axis=2):
    """Device tensor like `compact` (bf16 bits) with `axis` widened to `cap`, zero beyond the copy."""
    import torch
    shape = list(compact.shape)
    w = shape[axis]
    shape[axis] = cap
    big = torch.zeros(shape, dtype=torch.bfloat16, device="cuda")
    assert big.numel() * 2 > FOUR_GIB
    big.narrow(axis, 0, w).copy_(bf(compact))
    return big


@pytest.mark.parametrize("algo", ["auto", "simple"])
def test_suffix_stores_beyond_4gib(B, algo):
    import torch
    P, G, Hq, Hkv, d, W, cap = 2, 80, 8, 4, 128, 96, 33024
    rng = np.random.default_rng(5)
    sl = rng.integers(0, W + 1, P * G).astype(np.int32)
    sl[[3, 150]] = 0
    sl[[130, 159]] = W
    x = util.random_case(51, P, G, Hq, Hkv, d, 256, W, "bf16", slens=sl)
    t = util.to_device({k: v for k, v in x.items() if k not in ("k_suffix", "v_suffix")})
    t["k_suffix"], t["v_suffix"] = grow(x["k_suffix"], cap), grow(x["v_suffix"], cap)
    # sequences 128 .. 159 start behind 4 GiB
    assert 128 * Hkv * cap * d * 2 >= FOUR_GIB
    out, lse = util.gpu_run(t, 0.09, G, algo={"auto": B.RLDA_ALGO_AUTO, "simple": B.RLDA_ALGO_SIMPLE}[algo])
    torch.cuda.synchronize()
    ro, rl = util.oracle(x, 0.09, G)
    util.compare(out, lse, ro, rl, "bf16", f"suffix stores of {t['k_suffix'].numel() * 2 / 2**30:.1f} GiB, {algo}")


def test_prefix_stores_beyond_4gib(B):
    import torch
    P, G, Hq, Hkv, d, W, cap = 40, 2, 8, 4, 128, 200, 131072
    rng = np.random.default_rng(6)
    pl = rng.integers(1, W + 1, P).astype(np.int32)
    pl[[2, 39]] = W
    pl[35] = 0
    x = util.random_case(52, P, G, Hq, Hkv, d, W, 64, "bf16", plens=pl)
    t = util.to_device({k: v for k, v in x.items() if k not in ("k_prefix", "v_prefix")})
    t["k_prefix"], t["v_prefix"] = grow(x["k_prefix"], cap), grow(x["v_prefix"], cap)
    assert 32 * Hkv * cap * d * 2 >= FOUR_GIB                # prompts 32 .. 39 start behind 4 GiB
    for algo in (B.RLDA_ALGO_AUTO, B.RLDA_ALGO_SIMPLE):
        out, lse = util.gpu_run(t, 0.09, G, algo=algo)
        torch.cuda.synchronize()
        ro, rl = util.oracle(x, 0.09, G)
        util.compare(out, lse, ro, rl, "bf16", f"prefix stores of {t['k_prefix'].numel() * 2 / 2**30:.1f} GiB, algo {algo}")


def test_page_pool_beyond_4gib(B):
    import torch
    P, G, Hq, Hkv, d, ps, n_big = 4, 16, 28, 4, 128, 128, 40000
    x = util.random_case(53, P, G, Hq, Hkv, d, 180, 600, "bf16")
    y = wl.to_pages(x, ps, seed=9, poison=False)
    n_small = y["k_pages"].shape[0]
    # the same pages at the top of a 5 GiB pool, in reverse order
    remap = (n_big - 1 - np.arange(n_small)).astype(np.int64)
    assert int(remap.min()) * Hkv * ps * d * 2 >= FOUR_GIB
    t = util.to_device({k: v for k, v in y.items() if k not in ("k_pages", "v_pages", "block_table")})
    idx = torch.from_numpy(remap).cuda()
    for name in ("k_pages", "v_pages"):
        pool = torch.zeros((n_big, Hkv, ps, d), dtype=torch.bfloat16, device="cuda")
        pool[idx] = bf(y[name])
        t[name] = pool
    table = y["block_table"].astype(np.int64)
    t["block_table"] = torch.from_numpy(np.where(table >= 0, n_big - 1 - table, table).astype(np.int32)).cuda()
    for algo in (B.RLDA_ALGO_AUTO, B.RLDA_ALGO_SIMPLE):
        out, lse = util.gpu_run_paged(t, 0.09, G, algo=algo)
        torch.cuda.synchronize()
        ro, rl = util.oracle_paged(y, 0.09, G)
        util.compare(out, lse, ro, rl, "bf16", f"pool of {t['k_pages'].numel() * 2 / 2**30:.1f} GiB, algo {algo}")


def test_append_into_stores_beyond_4gib(B):
    """The appended rows land at the end of every sequence's region of a 5 GiB store; nothing else is written."""
    import torch
    from oracle.kv_append_ref import kv_append_rope_ref
    from tests.test_gpu_kv_append import close, host
    w = wl.scaled(wl.WORKLOADS["vlm7b"], P=20, Ls_cap=8, suffix=("uniform", 7))      # 160 sequences, 4 KV heads
    cap, shift = 33024, 33024 - 8
    x = wl.make_inputs(w)
    nt = wl.make_new_token(w, x, seed=91)
    lens = np.random.default_rng(7).integers(0, 8, w.B).astype(np.int32)
    lens[0] = 8                                               # full: skipped
    t = {k: (bf(v) if v.dtype == np.uint16 else torch.from_numpy(v).cuda()) for k, v in nt.items() if isinstance(v, np.ndarray)}
    stores = {}
    for name in ("k", "v"):
        big = torch.zeros((w.B, w.Hkv, cap, w.d), dtype=torch.bfloat16, device="cuda")
        big[:, :, shift:] = bf(x[f"{name}_suffix"])
        stores[name] = big
    assert 128 * w.Hkv * cap * w.d * 2 >= FOUR_GIB
    dl = torch.from_numpy(lens + shift).cuda()
    B.rl_kv_append_rope(t["q"], t["k_new"], t["v_new"], t["positions"], t["inv_freq"], nt["sections"],
                        stores["k"], stores["v"], dl)
    torch.cuda.synchronize()
    q_ref, k_ref, v_ref, l_ref = kv_append_rope_ref(nt["q"], nt["k_new"], nt["v_new"], nt["positions"], nt["inv_freq"],
                                                    nt["sections"], x["k_suffix"], x["v_suffix"], lens)
    assert np.array_equal(dl.cpu().numpy() - shift, l_ref)
    close(host(t["q"]), q_ref, "q")
    assert np.array_equal(host(stores["v"][:, :, shift:].contiguous()), v_ref)
    close(host(stores["k"][:, :, shift:].contiguous()), k_ref, "key store")
    for name in ("k", "v"):
        assert int(torch.count_nonzero(stores[name][:, :, :shift].view(torch.int16))) == 0, "a row outside the target was written"


def test_prefill_with_q_and_out_beyond_4gib(B):
    import torch
    from oracle.prefill_ref import prefill_attn_ref
    P, Hq, Hkv, d, W, cap = 9, 32, 8, 128, 320, 32768
    lens = np.zeros(P, np.int32)
    lens[8], lens[0], lens[5] = 300, 100, W
    rng = np.random.default_rng(8)
    tb = lambda shape, g=1.0: wl.f32_to_bf16_bits((rng.standard_normal(shape) * g).astype(np.float32))
    q, k, v = tb((P, W, Hq, d), 2.0), tb((P, Hkv, W, d)), tb((P, Hkv, W, d))
    # q [P, cap, Hq, d] is 2.3 GiB, out (fp32) 4.5 GiB: prompt 8's rows sit behind 4 GiB of out
    dq = torch.zeros((P, cap, Hq, d), dtype=torch.bfloat16, device="cuda")
    dq[:, :W] = bf(q)
    dk = torch.zeros((P, Hkv, cap, d), dtype=torch.bfloat16, device="cuda")
    dv = torch.zeros_like(dk)
    dk[:, :, :W], dv[:, :, :W] = bf(k), bf(v)
    out = torch.zeros((P, cap, Hq, d), dtype=torch.float32, device="cuda")
    assert 8 * cap * Hq * d * 4 >= FOUR_GIB
    lse = torch.zeros((P, cap, Hq), dtype=torch.float32, device="cuda")
    B.rl_prefill_attn(dq, dk, dv, torch.from_numpy(lens).cuda(), 0.088, out=out, lse=lse)
    torch.cuda.synchronize()
    ro, rl = prefill_attn_ref(q, k, v, lens, 0.088)
    for p in (0, 5, 8):
        n = int(lens[p])
        eo = np.abs(out[p, :n].cpu().numpy().astype(np.float64) - ro[p, :n]).max()
        el = np.abs(lse[p, :n].cpu().numpy().astype(np.float64) - rl[p, :n]).max()
        assert eo <= 1e-2 and el <= 1e-3, (p, eo, el)
    written = torch.count_nonzero(out.view(P, cap, -1).abs().sum(dim=2))
    assert int(written) == int(lens.sum()), "rows beyond a prompt's length must stay untouched"
