"""GPU parity of rl_group_advantage and rl_policy_loss with the fp64 oracle, through the C ABI.

Bar (the arithmetic is fp32 with fp32 per-sequence and fp64 cross-sequence sums): batch
statistics within 2e-5 relative (+1e-7 abs); per-token gradients within 2e-6 relative of the
oracle's, except tokens whose ratio lies within 1e-5 of a clip bound, where fp32 and fp64 may
sit on different branches: there either branch's value is accepted (and the clip fraction may
differ by those tokens).  Advantages within 1e-5 * (1 + |A|); combined rewards within 1e-6.
"""
import numpy as np
import pytest

from oracle.policy_loss_ref import group_advantage_ref, policy_loss_ref
from paper_2512_21450_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    import torch
    assert torch.cuda.is_available()
    from paper_2512_21450_amd import binding
    return binding


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def check_loss(B, x, adv, clip_low, clip_high, **kw):
    import torch
    beta_kl, beta_ent = kw.get("beta_kl", 0.0), kw.get("beta_ent", 0.0)
    use_reg = kw.pop("use_reg", True)
    kl = x["kl"] if use_reg else None
    ent = x["entropy"] if use_reg else None
    stats, grad = B.rl_policy_loss(dev(x["logprob"]), dev(x["old_logprob"]), dev(adv), dev(x["lens"]), clip_low, clip_high,
                                   kl=None if kl is None else dev(kl), entropy=None if ent is None else dev(ent), **kw)
    torch.cuda.synchronize()
    r = policy_loss_ref(x["logprob"], x["old_logprob"], adv, x["lens"], clip_low, clip_high, kl=kl, entropy=ent,
                        beta_kl=beta_kl, beta_ent=beta_ent, form=kw.get("form", 0), agg=kw.get("agg", 0))
    s = dict(zip(B.POLICY_LOSS_STATS, stats.cpu().numpy().astype(np.float64)))
    T = x["logprob"].shape[1]
    valid = np.arange(T)[None, :] < np.clip(x["lens"], 0, T)[:, None]
    lo, hi = 1 - clip_low, 1 + clip_high
    edge = valid & ((np.abs(r["ratio"] - lo) < 1e-5) | (np.abs(r["ratio"] - hi) < 1e-5))
    n = max(r["n_tokens"], 1)
    assert s["n_tokens"] == r["n_tokens"]
    for k in ("loss", "pg", "kl", "entropy", "ratio_mean", "approx_kl"):
        slack = edge.sum() / n * 4 * np.abs(adv).max() if k in ("loss", "pg") else 0.0
        assert abs(s[k] - r[k]) <= 2e-5 * abs(r[k]) + 1e-7 + slack, (k, s[k], r[k])
    assert abs(s["clip_frac"] - r["clip_frac"]) <= (edge.sum() + 0.5) / n
    g = grad.cpu().numpy().astype(np.float64)
    assert (g[~valid] == 0).all(), "padding must get zero gradient"
    ok = np.abs(g - r["grad"]) <= 2e-6 * np.abs(r["grad"]) + 1e-12
    # on a clip bound the other branch (zero, or the unclipped slope) is as good
    w = np.abs(r["grad"]).max() if r["grad"].size else 0.0
    other = edge & (np.abs(g) <= 2 * w + 1e-12)
    assert (ok | other).all(), f"{(~(ok | other)).sum()} gradient entries off"
    return s, r


@pytest.mark.parametrize("form", [0, 1])
@pytest.mark.parametrize("agg", [0, 1])
def test_policy_loss_reduced(B, form, agg):
    x = wl.make_rollout_tokens(48, 700, 8, seed=11 + form + 2 * agg, drift=0.25, lens=("uniform", 700))
    x["lens"][[0, 5, 17]] = 0
    x["lens"][3] = 700
    x["lens"][4] = 1
    _, adv = group_advantage_ref(x["metrics"], x["weights"], 8)
    s, r = check_loss(B, x, adv.astype(np.float32), 0.2, 0.28, beta_kl=0.04, beta_ent=0.01, form=form, agg=agg)
    assert 0.01 < r["clip_frac"] < 0.6                                   # the case does exercise both branches


def test_policy_loss_edge_cases(B):
    import torch
    x = wl.make_rollout_tokens(5, 33, 5, seed=3, lens=("uniform", 33))
    adv = np.array([1.0, -1.0, 0.0, 2.5, -0.5], np.float32)
    # lengths outside [0, T] clamp; garbage (NaN / inf) in the padding is never read
    x["lens"] = np.array([40, -3, 33, 1, 0], np.int32)
    for k in ("logprob", "old_logprob", "kl", "entropy"):
        x[k][3, 1:] = np.nan
        x[k][4, :] = np.inf
        x[k][1, :] = np.nan
    check_loss(B, x, adv, 0.2, 0.2, beta_kl=0.1, beta_ent=0.1)
    check_loss(B, x, adv, 0.0, 0.0)                                       # zero-width range: every off-policy token is clipped one way
    check_loss(B, x, adv, 0.2, 0.2, use_reg=False, beta_kl=0.3)          # no KL / entropy tensors: their terms are zero
    # nothing valid at all: all statistics zero, gradient zero
    x["lens"][:] = 0
    s, _ = check_loss(B, x, adv, 0.2, 0.2)
    assert all(v == 0 for v in s.values())
    # on-policy point: ratio exactly 1 everywhere
    y = wl.make_rollout_tokens(16, 64, 4, seed=5, lens=("uniform", 64))
    y["logprob"] = y["old_logprob"].copy()
    _, a = group_advantage_ref(y["metrics"], y["weights"], 4)
    s, r = check_loss(B, y, a.astype(np.float32), 0.2, 0.2)
    assert s["clip_frac"] == 0 and s["ratio_mean"] == 1.0 and s["approx_kl"] == 0
    # empty batch and T = 0
    st, g = B.rl_policy_loss(torch.empty((0, 8), device="cuda"), torch.empty((0, 8), device="cuda"),
                             torch.empty(0, device="cuda"), torch.empty(0, dtype=torch.int32, device="cuda"), 0.2, 0.2)
    assert (st.cpu().numpy() == 0).all()


def test_policy_loss_strided_rows_determinism_and_no_grad(B):
    import torch
    x = wl.make_rollout_tokens(32, 300, 8, seed=21, lens=("lognormal", 100.0, 1.0))
    _, adv = group_advantage_ref(x["metrics"], x["weights"], 8)
    adv = adv.astype(np.float32)
    pad = lambda a: torch.nn.functional.pad(dev(a), (0, 20), value=float("nan"))[:, :300]     # row stride 320
    lp, old, kl, en = pad(x["logprob"]), pad(x["old_logprob"]), pad(x["kl"]), pad(x["entropy"])
    assert lp.stride(0) == 320
    s1, g1 = B.rl_policy_loss(lp, old, dev(adv), dev(x["lens"]), 0.2, 0.2, kl=kl, entropy=en, beta_kl=0.05, want_grad=False)
    assert g1 is None
    s2, _ = B.rl_policy_loss(dev(x["logprob"]), dev(x["old_logprob"]), dev(adv), dev(x["lens"]), 0.2, 0.2, kl=dev(x["kl"]),
                             entropy=dev(x["entropy"]), beta_kl=0.05)
    s3, _ = B.rl_policy_loss(dev(x["logprob"]), dev(x["old_logprob"]), dev(adv), dev(x["lens"]), 0.2, 0.2, kl=dev(x["kl"]),
                             entropy=dev(x["entropy"]), beta_kl=0.05)
    assert torch.equal(s1, s2) and torch.equal(s2, s3)                   # the layout does not change the bits; nor does a rerun


def test_policy_loss_at_rollout_scale(B):
    # 2048 trajectories of up to 1024 generated tokens (the high-batch rollout), lognormal lengths
    x = wl.make_rollout_tokens(2048, 1024, 16, seed=31, lens=("lognormal", 200.0, 1.0))
    _, adv = group_advantage_ref(x["metrics"], x["weights"], 16)
    s, r = check_loss(B, x, adv.astype(np.float32), 0.2, 0.28, beta_kl=0.04, agg=1)
    print(f"\n{int(r['n_tokens'])} tokens: loss {s['loss']:.6f} (oracle {r['loss']:.6f}), clip fraction {s['clip_frac']:.4f}")


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("P,G,M", [(64, 8, 2), (5, 1, 1), (3, 1000, 3), (128, 16, 1), (7, 257, 2)])
def test_group_advantage(B, mode, P, G, M):
    import torch
    rng = np.random.default_rng(P * 1000 + G + mode)
    m = rng.standard_normal((M, P * G)).astype(np.float32)
    if G > 1:
        m[:, :G] = 0.7                                                   # a group without signal
    a = rng.standard_normal(M).astype(np.float32)
    for unbiased in (True, False):
        rew, adv = B.rl_group_advantage(dev(m), dev(a), G, mode=mode, eps=1e-6, unbiased=unbiased)
        torch.cuda.synchronize()
        r_ref, a_ref = group_advantage_ref(m, a, G, mode=mode, eps=1e-6, unbiased=unbiased)
        rew, adv = rew.cpu().numpy().astype(np.float64), adv.cpu().numpy().astype(np.float64)
        assert np.abs(rew - r_ref).max() <= 1e-6 * (1 + np.abs(r_ref).max())
        # the oracle normalises its fp64 rewards, the kernel its fp32 ones: compare on the kernel's rewards too
        _, a_own = group_advantage_ref(rew[None, :], np.ones(1), G, mode=mode, eps=1e-6, unbiased=unbiased)
        assert np.abs(adv - a_own).max() <= 1e-5 * (1 + np.abs(a_own).max())
        # against the oracle's own fp64 rewards the normalised estimator amplifies the fp32 rounding of the
        # rewards by 1 / std of the group, so that comparison is looser
        assert np.abs(adv - a_ref).max() <= 1e-4 * (1 + np.abs(a_ref).max())
        if G > 1:
            assert (adv[:G] == 0).all(), "equal rewards must give exactly zero advantages"
        else:
            assert (adv == 0).all()


def test_policy_loss_many_short_sequences(B):
    # more than 4096 sequences: the batch totals come from a launch of their own instead of from every workgroup
    x = wl.make_rollout_tokens(5000, 48, 8, seed=41, lens=("uniform", 48))
    x["lens"][::7] = 0
    _, adv = group_advantage_ref(x["metrics"], x["weights"], 8)
    for agg in (0, 1):
        check_loss(B, x, adv.astype(np.float32), 0.2, 0.25, beta_kl=0.03, beta_ent=0.01, agg=agg)
