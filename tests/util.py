"""Shared helpers of the tests: tensors to the device, oracle call, comparison."""
import numpy as np

from paper_2512_21450_amd import workloads as wl

# acceptance tolerances (absolute, max over all elements): fp32 inputs 1e-5 on
# out and lse; bf16 inputs with fp32 accumulation 1e-2 on out, 1e-3 on lse
TOL = {"f32": (1e-5, 1e-5), "bf16": (1e-2, 1e-3)}


def to_device(x, device="cuda:0"):
    import torch
    out = {}
    for k, v in x.items():
        if not isinstance(v, np.ndarray):
            continue
        if v.dtype == np.uint16:
            out[k] = torch.from_numpy(v.view(np.int16)).to(device).view(torch.bfloat16)
        else:
            out[k] = torch.from_numpy(v).to(device)
    return out


def oracle(x, scale, G, **kw):
    from oracle import ref
    return ref.decode_attn_ref(x["q"], x["k_prefix"], x["v_prefix"], x["prefix_lens"],
                               x["k_suffix"], x["v_suffix"], x["suffix_lens"], scale, G,
                               k_scale=x.get("k_scale"), v_scale=x.get("v_scale"), **kw)


def gpu_run(t, scale, G, **kw):
    from paper_2512_21450_amd import binding
    return binding.rl_decode_attn(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"],
                                  t["k_suffix"], t["v_suffix"], t["suffix_lens"], scale, G,
                                  k_scale=t.get("k_scale"), v_scale=t.get("v_scale"), **kw)


def compare(out, lse, ref_out, ref_lse, dtype, what=""):
    """Element-by-element against the fp64 oracle; -inf must match exactly."""
    tol_o, tol_l = TOL[dtype]
    out = out.detach().cpu().numpy().astype(np.float64)
    lse = lse.detach().cpu().numpy().astype(np.float64)
    assert not np.isnan(out).any(), f"{what}: NaN in out"
    assert not np.isnan(lse).any(), f"{what}: NaN in lse"
    inf_ref = np.isneginf(ref_lse)
    assert np.array_equal(np.isneginf(lse), inf_ref), f"{what}: -inf pattern of lse differs"
    eo = np.abs(out - ref_out).max() if out.size else 0.0
    el = np.abs(np.where(inf_ref, 0.0, lse) - np.where(inf_ref, 0.0, ref_lse)).max() if lse.size else 0.0
    assert eo <= tol_o, f"{what}: max |out - oracle| = {eo:.3e} > {tol_o}"
    assert el <= tol_l, f"{what}: max |lse - oracle| = {el:.3e} > {tol_l}"
    return eo, el


def random_case(seed, P, G, Hq, Hkv, d, Lp_cap, Ls_cap, dtype="bf16", plens=None, slens=None, gain=1.0):
    """Seeded N(0,1) tensors with explicit or uniformly drawn lengths."""
    rng = np.random.default_rng(seed)
    B = P * G

    def t(shape, g=1.0):
        v = (rng.standard_normal(shape) * g).astype(np.float32)
        return v if dtype == "f32" else wl.f32_to_bf16_bits(v)

    x = dict(q=t((B, Hq, d), gain), k_prefix=t((P, Hkv, Lp_cap, d)), v_prefix=t((P, Hkv, Lp_cap, d)),
             k_suffix=t((B, Hkv, Ls_cap, d)), v_suffix=t((B, Hkv, Ls_cap, d)))
    x["prefix_lens"] = (rng.integers(0, Lp_cap + 1, P) if plens is None else np.asarray(plens)).astype(np.int32)
    x["suffix_lens"] = (rng.integers(0, Ls_cap + 1, B) if slens is None else np.asarray(slens)).astype(np.int32)
    return x


def oracle_paged(y, scale, G, active=None, **kw):
    from oracle import ref
    return ref.decode_attn_paged_ref(y["q"], y["k_prefix"], y["v_prefix"], y["prefix_lens"], y["k_pages"],
                                     y["v_pages"], y["block_table"], y["suffix_lens"], active, scale, G,
                                     k_scale=y.get("k_scale"), v_scale=y.get("v_scale"), **kw)


def gpu_run_paged(t, scale, G, active=None, **kw):
    from paper_2512_21450_amd import binding
    return binding.rl_decode_attn_paged(t["q"], t["k_prefix"], t["v_prefix"], t["prefix_lens"], t["k_pages"],
                                        t["v_pages"], t["block_table"], t["suffix_lens"], scale, G,
                                        seq_active=active, k_scale=t.get("k_scale"), v_scale=t.get("v_scale"), **kw)
