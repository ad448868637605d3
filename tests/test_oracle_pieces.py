"""Pins for the oracle's building blocks: each is checked against an independent library routine,
a closed form or an invariant, so that a dropped term, a wrong sign or a transposed operand fails."""
import math

import numpy as np
import pytest
import scipy.special as sps
import torch
import torch.nn.functional as F

from oracle import decoder as O

f64 = np.float64


def rng(seed):
    return np.random.default_rng(seed)


def test_layer_norm_matches_torch():
    r = rng(1)
    x, g, b = r.normal(size=(5, 48)) * 3 + 1.5, r.normal(size=48), r.normal(size=48)
    ref = F.layer_norm(torch.tensor(x), (48,), torch.tensor(g), torch.tensor(b), eps=1e-5).numpy()
    np.testing.assert_allclose(O.layer_norm(x, g, b, 1e-5, f64), ref, rtol=0, atol=1e-12)
    # fp32 path stays within fp32 rounding of the fp64 result
    got32 = O.layer_norm(x.astype(np.float32), g.astype(np.float32), b.astype(np.float32), 1e-5)
    assert got32.dtype == np.float32
    np.testing.assert_allclose(got32, ref, atol=2e-6 * np.abs(ref).max())


def test_rms_norm_matches_torch():
    r = rng(2)
    x, g = r.normal(size=(4, 40)) * 2 + 0.3, r.normal(size=40)
    ref = F.rms_norm(torch.tensor(x), (40,), torch.tensor(g), eps=1e-5).numpy()
    np.testing.assert_allclose(O.rms_norm(x, g, 1e-5, f64), ref, atol=1e-12)


def test_gelu_is_erf_form_and_silu():
    t = np.linspace(-6, 6, 241)
    np.testing.assert_allclose(O.gelu(t, f64), F.gelu(torch.tensor(t), approximate="none").numpy(), atol=1e-14)
    # the tanh approximation differs visibly: make sure we did not pick it
    assert np.abs(O.gelu(t, f64) - F.gelu(torch.tensor(t), approximate="tanh").numpy()).max() > 1e-4
    np.testing.assert_allclose(O.silu(t, f64), F.silu(torch.tensor(t)).numpy(), atol=1e-14)
    assert O.gelu(np.array([1.0]), f64)[0] == pytest.approx(0.8413447460685429, abs=1e-15)  # Phi(1)


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (4, 2), (8, 2)])
def test_attention_matches_torch_sdpa(Hq, Hkv):
    r = rng(3)
    n, h = 9, 8
    q, k, v = r.normal(size=(n, Hq, h)), r.normal(size=(n, Hkv, h)), r.normal(size=(n, Hkv, h))
    got = O.attention(q, k, v, np.arange(n), f64)
    tq = torch.tensor(q).permute(1, 0, 2)[None]
    tk = torch.tensor(k).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    tv = torch.tensor(v).permute(1, 0, 2).repeat_interleave(Hq // Hkv, dim=0)[None]
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, ref, atol=1e-12)


def test_attention_decode_row_equals_prefill_row():
    r = rng(4)
    n, H, h = 7, 2, 4
    q, k, v = r.normal(size=(n, H, h)), r.normal(size=(n, H, h)), r.normal(size=(n, H, h))
    full = O.attention(q, k, v, np.arange(n), f64)
    for p in range(n):
        row = O.attention(q[p:p + 1], k[:p + 1], v[:p + 1], np.array([p]), f64)
        np.testing.assert_allclose(row[0], full[p], atol=1e-13)


@pytest.mark.parametrize("h,r", [(8, 4), (8, 8), (80, 20), (32, 8)])
def test_rotary_is_complex_multiplication(h, r):
    g = rng(5)
    n, H = 6, 3
    theta = 10000.0
    u = g.normal(size=(n, H, h))
    pos = np.array([0, 1, 2, 17, 511, 1535])
    got = O.rotary(u, pos, r, theta, f64)
    half = r // 2
    z = u[..., :half] + 1j * u[..., half:r]
    ang = pos[:, None] * theta ** (-2.0 * np.arange(half) / r)[None, :]
    zr = z * np.exp(1j * ang)[:, None, :]
    np.testing.assert_allclose(got[..., :half], zr.real, atol=1e-12)
    np.testing.assert_allclose(got[..., half:r], zr.imag, atol=1e-12)
    np.testing.assert_array_equal(got[..., r:], u[..., r:])       # pass-through dims untouched
    np.testing.assert_array_equal(got[0], u[0])                    # position 0 is the identity
    np.testing.assert_allclose(np.hypot(got[..., :half], got[..., half:r]),
                               np.hypot(u[..., :half], u[..., half:r]), atol=1e-12)


def test_rotary_scores_depend_on_relative_position_only():
    g = rng(6)
    h, r = 8, 8
    q, k = g.normal(size=(1, 1, h)), g.normal(size=(1, 1, h))
    def dot(p, s):
        return float((O.rotary(q, [p], r, 500000.0, f64) * O.rotary(k, [s], r, 500000.0, f64)).sum())
    assert dot(10, 3) == pytest.approx(dot(107, 100), abs=1e-12)
    assert dot(10, 3) != pytest.approx(dot(10, 4), abs=1e-6)


def test_tempered_log_softmax_rows_sum_to_one_and_match_scipy():
    g = rng(7)
    z = (g.normal(size=(6, 1000)) * 3).astype(np.float32)
    lp = O.tempered_log_softmax(z, 0.7)
    assert np.abs(np.exp(lp).sum(axis=1) - 1).max() < 1e-6
    ref = sps.log_softmax((z / np.float32(0.7)).astype(f64), axis=1)
    np.testing.assert_allclose(lp, ref, atol=1e-12)
    # large logits do not overflow
    big = np.array([1e4, 1e4 - 1, -1e4], dtype=np.float32)
    assert np.isfinite(O.tempered_log_softmax(big, 0.7)).all()


def explicit_cdf_scan(logp, u):
    """Independent reference for the sampler: plain Python floats, one token at a time."""
    acc, last_pos = 0.0, None
    for j, lp in enumerate(logp):
        p = math.exp(float(lp))
        if p > 0:
            last_pos = j
        acc += p
        if acc > float(u):
            return j
    return last_pos


def test_sampler_reproduces_explicit_cdf_scan():
    g = rng(8)
    for V in (5, 16, 257):
        lp = O.tempered_log_softmax((g.normal(size=V) * 2).astype(np.float32), 0.7)
        for u in np.concatenate([g.random(200, dtype=np.float32), np.float32([0.0, 0.99999994])]):
            tok, margin = O.sample_inverse_cdf(lp, u)
            assert tok == explicit_cdf_scan(lp, u)
            assert margin >= 0


def test_sampler_edges_and_margin():
    lp = np.log(np.array([0.0, 0.25, 0.0, 0.5, 0.25, 0.0]) + 0.0, where=[False, True, False, True, True, False],
                out=np.full(6, -np.inf))
    assert O.sample_inverse_cdf(lp, 0.0)[0] == 1              # u = 0 -> first token with p > 0
    assert O.sample_inverse_cdf(lp, 0.2499)[0] == 1
    assert O.sample_inverse_cdf(lp, 0.25)[0] == 3             # strict inequality: C_1 = 0.25 is not > u
    assert O.sample_inverse_cdf(lp, 0.75)[0] == 4
    assert O.sample_inverse_cdf(lp, 0.99999)[0] == 4          # zero-probability tail never drawn
    tok, margin = O.sample_inverse_cdf(lp, 0.40)
    assert tok == 3 and margin == pytest.approx(0.15)
    tok, margin = O.sample_inverse_cdf(lp, 0.10)
    assert tok == 1 and margin == pytest.approx(0.10)         # lower edge is 0 for the first bucket
    tok, margin = O.sample_inverse_cdf(lp, 0.80)
    assert tok == 4 and margin == pytest.approx(0.05)         # u - C_3; upper edge is 1
    # a CDF that falls short of u by rounding falls back to the last positive-probability token
    short = np.log(np.array([0.5, 0.4999999, 1e-300]))
    assert O.sample_inverse_cdf(short, 0.99999994)[0] == 2


def test_sampler_is_monotone_in_u_and_matches_distribution():
    g = rng(9)
    V = 16
    lp = O.tempered_log_softmax((g.normal(size=V) * 1.5).astype(np.float32), 0.7)
    us = np.sort(g.random(100_000))
    toks = np.array([O.sample_inverse_cdf(lp, u)[0] for u in us])
    assert (np.diff(toks) >= 0).all()
    counts = np.bincount(toks, minlength=V)
    expect = np.exp(lp) * len(us)
    chi2 = ((counts - expect) ** 2 / expect).sum()
    assert chi2 < 50.0       # 15 degrees of freedom: P(chi2 > 50) ~ 1e-5


def test_cdf_bucket_is_the_interval_of_uniforms_that_draw_the_token():
    """Pins for cdf_bucket: a worked distribution written out; the buckets of consecutive tokens tile [0, 1) (each
    starts where the previous one ends, the first at 0, the last ends at 1 up to rounding); bucket edges against
    exact sums (math.fsum over Python floats); and the bucket of the token sample_inverse_cdf draws contains the
    uniform it was drawn with, while every other token's bucket does not."""
    lp = np.log(np.array([0.25, 0.5, 0.125, 0.125]))
    assert O.cdf_bucket(lp, 0) == (0.0, 0.25)
    assert O.cdf_bucket(lp, 1) == (0.25, 0.75)
    assert O.cdf_bucket(lp, 2) == (0.75, 0.875)
    assert O.cdf_bucket(lp, 3) == (0.875, 1.0)
    g = rng(12)
    for V in (3, 16, 257):
        lp = O.tempered_log_softmax((g.normal(size=V) * 2).astype(np.float32), 0.7)
        p = [math.exp(float(x)) for x in lp]
        edges = [O.cdf_bucket(lp, j) for j in range(V)]
        assert edges[0][0] == 0.0 and abs(edges[-1][1] - 1.0) < 1e-12
        for j in range(V):
            lo, hi = edges[j]
            assert lo == pytest.approx(math.fsum(p[:j]), abs=1e-13) and hi == pytest.approx(math.fsum(p[:j + 1]), abs=1e-13)
            assert hi - lo == pytest.approx(p[j], abs=1e-13)
            if j:
                assert lo == edges[j - 1][1]
        for u in g.random(300, dtype=np.float32):
            tok, margin = O.sample_inverse_cdf(lp, u)
            lo, hi = edges[tok]
            assert lo <= float(u) < hi
            assert margin == pytest.approx(min(float(u) - lo, (1.0 if tok == V - 1 else hi) - float(u)), abs=1e-15)
            inside = [j for j in range(V) if edges[j][0] <= float(u) < edges[j][1]]
            assert inside == [tok]


def test_sequence_logprob_is_the_exact_sum_of_the_response_terms():
    """Pins for sequence_logprob: exact sums (math.fsum), the half-open range [score_from, length), and additivity
    over a split of the range."""
    g = rng(13)
    tlp = (-g.random(70) * 12).astype(np.float32)
    for lo, hi in [(0, 70), (5, 70), (17, 18), (33, 64), (69, 70)]:
        assert O.sequence_logprob(tlp, lo, hi) == pytest.approx(math.fsum(float(x) for x in tlp[lo:hi]), abs=1e-12)
    assert O.sequence_logprob(tlp, 40, 40) == 0.0 and O.sequence_logprob(tlp, 50, 40) == 0.0
    assert O.sequence_logprob(tlp, 3, 60) == pytest.approx(O.sequence_logprob(tlp, 3, 31) + O.sequence_logprob(tlp, 31, 60), abs=1e-12)
    # position `length` itself is outside, position `score_from` inside
    one_hot = np.zeros(10, np.float32); one_hot[4] = -2.5
    assert O.sequence_logprob(one_hot, 4, 5) == -2.5 and O.sequence_logprob(one_hot, 5, 10) == 0.0 and O.sequence_logprob(one_hot, 0, 4) == 0.0


def test_dpo_pair_loss_closed_forms():
    assert O.dpo_pair_loss(-3.0, -3.0, -5.0, -5.0, 0.1) == pytest.approx(math.log(2.0), abs=1e-15)
    # beta * delta = 0.1 * ((-10+20) - (-30+30)) = 1  ->  -log sigmoid(1)
    assert O.dpo_pair_loss(-10.0, -20.0, -30.0, -30.0, 0.1) == pytest.approx(0.31326168751822286, abs=1e-14)
    x = np.linspace(-40, 40, 33)
    ref = -F.logsigmoid(torch.tensor(0.05 * x)).numpy()
    np.testing.assert_allclose(O.dpo_pair_loss(x, 0.0, 0.0, 0.0, 0.05), ref, atol=1e-13)
    # swapping the pair flips the sign of the argument: loss(+) - loss(-) = -beta*delta
    a, b = O.dpo_pair_loss(-1.0, -2.0, -4.0, -3.0, 0.03), O.dpo_pair_loss(-4.0, -3.0, -1.0, -2.0, 0.03)
    assert a - b == pytest.approx(-0.03 * 2.0, abs=1e-14)


def test_select_pair_is_the_extremes_of_a_stable_ranking():
    """Pins: the K = 2 cases written out; against a ranking by stable sort on random rewards with many ties."""
    assert O.select_pair([1.0, 2.0]) == (1, 0)
    assert O.select_pair([2.0, 1.0]) == (0, 1)
    assert O.select_pair([1.0, 1.0]) == (0, 1)
    assert O.select_pair([0.5]) == (0, 0)
    assert O.select_pair([0.0, 3.0, -1.0, 3.0]) == (1, 2)
    rng = np.random.default_rng(5)
    for K in (2, 3, 4, 7):
        for _ in range(200):
            r = rng.integers(0, 3, size=K).astype(np.float64)        # few distinct values: ties are common
            pos, neg = O.select_pair(r)
            best_first = np.argsort(-r, kind="stable")                # descending, earlier index first among equals
            assert pos == best_first[0]
            assert neg == K - 1 - np.argsort(r[::-1], kind="stable")[0]   # last of the lowest
            assert r[pos] == r.max() and r[neg] == r.min() and pos != neg


def test_proximal_rloo_objective_is_the_clipped_surrogate():
    """Pins (Appendix B, Eq. 1): worked k = 2 values; on-policy (ratio 1) the objective is the advantage R1 - R2;
    the four regimes of the clipped minimum written case by case (positive advantage caps the ratio from above,
    negative advantage from below); advantages of a prompt's completions sum to zero at ratio 1; brute force of
    the leave-one-out baseline for k > 2."""
    # ratio = e^{0.5} > 1.2, A = +2 -> clipped at 1.2 * 2 ; second completion: ratio e^{-0.5} < 0.8, A = -2 -> 0.8 * -2
    got = O.proximal_rloo_objective([-9.5, -10.5], [-10.0, -10.0], [3.0, 1.0], 0.2)
    np.testing.assert_allclose(got, [2.4, -1.6], atol=1e-14)
    # ratio above the band with a negative advantage is NOT clipped (the minimum keeps the more negative value)
    got = O.proximal_rloo_objective([-9.5, -10.0], [-10.0, -10.0], [1.0, 3.0], 0.2)
    np.testing.assert_allclose(got, [-2.0 * np.exp(0.5), 2.0], atol=1e-14)
    # ratio below the band with a positive advantage is not clipped either
    got = O.proximal_rloo_objective([-11.0, -10.0], [-10.0, -10.0], [3.0, 1.0], 0.2)
    np.testing.assert_allclose(got, [2.0 * np.exp(-1.0), -2.0], atol=1e-14)
    rng = np.random.default_rng(11)
    for k in (2, 3, 4, 8):
        for _ in range(100):
            lp_old = -rng.random(k) * 50
            lp_pol = lp_old + rng.standard_normal(k) * 0.3
            rew = rng.standard_normal(k)
            eps = float(rng.choice([0.0, 0.1, 0.2]))
            got = O.proximal_rloo_objective(lp_pol, lp_old, rew, eps)
            on_policy = O.proximal_rloo_objective(lp_old, lp_old, rew, eps)
            adv = (rew - (rew.sum() - rew) / (k - 1))                 # leave-one-out mean, vectorised
            np.testing.assert_allclose(on_policy, adv, atol=1e-12)
            assert abs(on_policy.sum()) < 1e-12
            if k == 2:
                np.testing.assert_allclose(adv, [rew[0] - rew[1], rew[1] - rew[0]], atol=1e-12)
            ratio = np.exp(lp_pol - lp_old)
            by_case = np.where(adv >= 0, np.minimum(ratio, 1 + eps) * adv, np.maximum(ratio, 1 - eps) * adv)
            np.testing.assert_allclose(got, by_case, atol=1e-12)
            assert (got <= ratio * adv + 1e-12).all()                 # a lower bound of the unclipped surrogate
