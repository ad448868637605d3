"""GPU parity: every entry point of librlgen.so against the CPU oracle, element by element, on the
same seeded inputs.  Tolerances: raw logits 2e-2 max-abs, token log-probs 1e-2 max-abs, tokens
identical wherever the oracle's CDF margin exceeds 1e-3 (the oracle's token forced elsewhere)."""
import math

import numpy as np
import pytest
import torch

from oracle import decoder as O
from workloads import get_config, make_prompts, make_uniforms, make_weights, ModelShape, Weights
from gpu_util import (report, GPU_SHAPES, MARGIN, TOL_LOGITS, TOL_LOGPROB, R, dev_f32, dev_i32, make_policy,
                      oracle_generate_batch, padded, reference_decoder, scaled_bf16_weights)

pytestmark = pytest.mark.gpu


def rand_seqs(rng, vocab, lens):
    return [rng.integers(0, vocab, size=n) for n in lens]


class Case(tuple):
    """(model shape, weights, reference decoder, context) of a fixture, plus the mode the context was created in."""
    precise = 0


# Every shape in the default formats; the Llama shapes (and one GPT-NeoX shape) again in precise mode, where they are
# held against the plain oracle (see gpu_util.reference_decoder).
PRECISE_SHAPES = ["llama-gqa4-h16", "llama-gqa16-h16", "llama-gqa2-h128", "neox-h80"]
SMALL_CASES = list(GPU_SHAPES) + [n + "/precise" for n in PRECISE_SHAPES]


def _case(param, **policy_args):
    name, _, mode = param.partition("/")
    m = GPU_SHAPES[name]
    W = scaled_bf16_weights(m)
    c = Case((m, W, reference_decoder(W, m, precise=bool(mode)), make_policy(W, precise=1 if mode else 0, **policy_args)))
    c.precise = 1 if mode else 0
    return c


@pytest.fixture(scope="module", params=SMALL_CASES)
def small(request):
    # max_batch_tokens == max_seq_len forces several chunks in prefill and scoring
    c = _case(request.param, max_seqs=12, max_seq_len=80, max_batch_tokens=80)
    yield c
    c[3].close()


def test_logits_match_oracle(small):
    m, W, dec, pol = small
    rng = np.random.default_rng(31)
    seqs = rand_seqs(rng, m.vocab, [1, 2, 16, 17, 31, 32, 33, 64, 65, 80, 47, 5])
    arr, lens = padded(seqs, pad=10 ** 6)          # pad cells hold an out-of-range id: never read
    got = R().rlgen_debug_logits(pol, dev_i32(arr), lens).cpu().numpy()
    ref = np.stack([O.last_logits(dec, s) for s in seqs])
    report("logits", err=np.abs(got - ref).max(), ref_std=ref.std(), ref_max=np.abs(ref).max(), d=m.d_model, h=m.head_dim,
           precise=small.precise)
    assert np.abs(ref).max() > 0.3
    assert np.abs(got - ref).max() < (TOL_LOGITS / 20 if small.precise else TOL_LOGITS)     # precise mode: 16 bits instead of 8 to 11
    assert R().rlgen_status(pol) == 0


def test_score_matches_oracle(small):
    m, W, dec, pol = small
    rng = np.random.default_rng(32)
    seqs = rand_seqs(rng, m.vocab, [80, 3, 33, 64, 1, 2, 70])
    arr, lens = padded(seqs, pad=-5)
    score_from = np.array([40, 1, 0, 60, 1, 1, 69], np.int32)
    for sf in (None, score_from):
        got = R().rlgen_score(pol, dev_i32(arr), lens, 0.7, sf).cpu().numpy()
        for i, s in enumerate(seqs):
            ref = O.score(dec, s, 0.7, 1 if sf is None else sf[i])
            report("score", err=np.abs(got[i, :len(s)] - ref).max(), n=len(s), h=m.head_dim, precise=small.precise)
            assert np.abs(got[i, :len(s)] - ref).max() < (TOL_LOGPROB / 20 if small.precise else TOL_LOGPROB), (i, sf is None)
            assert (got[i, len(s):] == 0).all()
            lo = max(1, 1 if sf is None else sf[i])
            assert (got[i, :lo] == 0).all()
    assert R().rlgen_status(pol) == 0


def test_generate_matches_oracle(small):
    m, W, dec, pol = small
    rng = np.random.default_rng(33)
    B, k, T, temp = 5, 2, 9, 0.7
    prompts = rand_seqs(rng, m.vocab, [30, 1, 33, 64, 71])
    arr, lens = padded(prompts, pad=-1)
    u = rng.random((B, k, T), dtype=np.float32)
    u[0, 1] = u[0, 0]                                   # equal uniforms -> equal samples
    r = R()
    # (1) the literal rule: oracle first, force its token where the margin is small, compare the rest
    t_o, l_o, margins, z_o, _ = oracle_generate_batch(dec, arr, lens, k, T, temp, u)
    forced = np.where(margins > MARGIN, -1, t_o).astype(np.int32)
    t_g, l_g = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u), dev_i32(forced))
    t_g, l_g = t_g.cpu().numpy(), l_g.cpu().numpy()
    report("generate-forced", err=np.abs(l_g - l_o).max(), mismatches=(t_g != t_o).sum(), free=(forced < 0).mean(), h=m.head_dim)
    np.testing.assert_array_equal(t_g, t_o)
    assert np.abs(l_g - l_o).max() < TOL_LOGPROB
    assert (forced < 0).mean() > 0.2                    # the comparison of free tokens is not vacuous
    # (2) unforced run: the GPU's token must be a valid draw under the oracle's CDF along the GPU's own path
    t_f, l_f = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u))
    t_f, l_f = t_f.cpu().numpy(), l_f.cpu().numpy()
    _, l_t, _, z_t, buckets = oracle_generate_batch(dec, arr, lens, k, T, temp, u, forced=t_f, with_buckets=True)
    report("generate-free", err=np.abs(l_f - l_t).max(), cdf_slack=max((buckets[..., 0] - u).max(), (u - buckets[..., 1]).max()),
           same_as_oracle=(t_f == t_o).mean(), h=m.head_dim)
    assert (buckets[..., 0] - MARGIN <= u).all() and (u <= buckets[..., 1] + MARGIN).all()
    assert np.abs(l_f - l_t).max() < TOL_LOGPROB
    np.testing.assert_array_equal(t_f[0, 0], t_f[0, 1])
    # (3) logits after the last generated token, through the prompt-pass kernels
    full = [np.concatenate([prompts[b], t_f[b, j]]) for b in range(B) for j in range(k)]
    farr, flens = padded(full)
    z_g = r.rlgen_debug_logits(pol, dev_i32(farr), flens).cpu().numpy()
    report("generate-final-logits", err=np.abs(z_g - z_t.reshape(B * k, -1)).max(), h=m.head_dim)
    assert np.abs(z_g - z_t.reshape(B * k, -1)).max() < TOL_LOGITS
    # (4) scoring the generated sequences reproduces generate's log-probs (prefill kernels vs decode kernels)
    sc = r.rlgen_score(pol, dev_i32(farr), flens, temp, np.repeat(lens, k)).cpu().numpy()
    for i in range(B * k):
        P = flens[i] - T
        assert np.abs(sc[i, P:flens[i]] - l_f.reshape(B * k, T)[i]).max() < TOL_LOGPROB
    # (5) bit-for-bit determinism
    t_2, l_2 = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u))
    assert torch.equal(t_2.cpu(), torch.from_numpy(t_f)) and torch.equal(l_2.cpu(), torch.from_numpy(l_f))
    assert r.rlgen_status(pol) == 0


def test_batch_composition_does_not_change_a_sequence(small):
    m, W, dec, pol = small
    rng = np.random.default_rng(34)
    prompts = rand_seqs(rng, m.vocab, [20, 45, 7, 64])
    u = rng.random((4, 2, 6), dtype=np.float32)
    r = R()
    arr, lens = padded(prompts, pad=-1)
    ta, la = r.rlgen_generate(pol, dev_i32(arr), lens, 2, 6, 0.7, dev_f32(u))
    order = [2, 0, 3, 1]
    arr2, lens2 = padded([prompts[i] for i in order], pad=10 ** 7)
    tb, lb = r.rlgen_generate(pol, dev_i32(arr2), lens2, 2, 6, 0.7, dev_f32(u[order]))
    assert torch.equal(ta[order], tb) and torch.equal(la[order], lb)
    arr3, lens3 = padded([prompts[1]])
    tc, lc = r.rlgen_generate(pol, dev_i32(arr3), lens3, 2, 6, 0.7, dev_f32(u[1:2]))
    assert torch.equal(ta[1:2], tc) and torch.equal(la[1:2], lc)


def test_sampler_exact_on_all_zero_model():
    """Every logit is exactly 0 on both sides: token = floor(u V) and log-prob = -ln V test the group
    search, the in-group scan and the ragged last group without any rounding slack."""
    for name in ("neox-h16-raggedV", "llama-gqa4-h16"):
        m = GPU_SHAPES[name]
        W = make_weights(m, 1, bf16=False)
        W = Weights(m, {k: np.zeros_like(v) for k, v in W.tensors.items()}, False)
        pol = make_policy(W, max_seqs=64, max_seq_len=40)
        rng = np.random.default_rng(35)
        u = rng.random((32, 2, 4), dtype=np.float32)
        u[0, 0, :] = [0.0, 0.99999994, 0.5, 63.5 / m.vocab]
        keep = np.abs(u.astype(np.float64) * m.vocab - np.round(u.astype(np.float64) * m.vocab)) > 1e-3
        prompts = np.zeros((32, 3), np.int32)
        t, l = R().rlgen_generate(pol, dev_i32(prompts), np.full(32, 3), 2, 4, 0.7, dev_f32(u))
        t, l = t.cpu().numpy(), l.cpu().numpy()
        want = np.floor(u.astype(np.float64) * m.vocab).astype(np.int32)
        np.testing.assert_array_equal(t[keep], want[keep])
        assert np.abs(l + math.log(m.vocab)).max() < 1e-5
        pol.close()


@pytest.mark.parametrize("peak", [1.0, 8.0])
def test_sampler_in_isolation_on_exact_logits(peak):
    """With final-norm gain 0 and a one-hot final-norm bias the LM-head input is exactly e_j, so the
    logits are exactly column j of the bf16 LM head on both sides: any token mismatch outside a 1e-6
    margin is the sampler's fault.  peak > 1 scales the LM head so that few tokens carry the mass."""
    m = GPU_SHAPES["neox-h80"]
    W = scaled_bf16_weights(m, seed=36, scale=5.0 * 6, lm_head_scale=peak)
    t = dict(W.tensors)
    from workloads import f32_to_bf16_bits
    g = np.zeros(m.d_model, np.float32)
    b = np.zeros(m.d_model, np.float32)
    b[7] = 1.0
    t["final_norm_g"], t["final_norm_b"] = f32_to_bf16_bits(g), f32_to_bf16_bits(b)
    W = Weights(m, t, True)
    dec = O.Decoder(W, m)
    pol = make_policy(W, max_seqs=512, max_seq_len=40, max_batch_tokens=512)
    rng = np.random.default_rng(37)
    Rr = 400
    hidden = rng.normal(size=(Rr, m.d_model)).astype(np.float32)
    u = rng.random(Rr, dtype=np.float32)
    tok, lp = R().rlgen_debug_sample(pol, dev_f32(hidden), 0.7, dev_f32(u))
    tok, lp = tok.cpu().numpy(), lp.cpu().numpy()
    z = dec.logits(hidden)
    np.testing.assert_array_equal(z[0], W.f32("lm_head")[:, 7])
    logp = O.tempered_log_softmax(z, 0.7)
    checked = 0
    for i in range(Rr):
        want, margin = O.sample_inverse_cdf(logp[i], u[i])
        if margin > 1e-6:
            assert tok[i] == want, i
            checked += 1
        assert abs(lp[i] - logp[i][tok[i]]) < 1e-5
    assert checked > 0.95 * Rr
    # forced tokens: the reported log-prob is that token's
    forced = rng.integers(0, m.vocab, size=Rr).astype(np.int32)
    forced[::3] = -1
    tok2, lp2 = R().rlgen_debug_sample(pol, dev_f32(hidden), 0.7, dev_f32(u), dev_i32(forced))
    tok2, lp2 = tok2.cpu().numpy(), lp2.cpu().numpy()
    np.testing.assert_array_equal(tok2[forced >= 0], forced[forced >= 0])
    np.testing.assert_array_equal(tok2[forced < 0], tok[forced < 0])
    assert np.abs(lp2 - logp[np.arange(Rr), tok2]).max() < 1e-5
    pol.close()


BIG_VOCAB_SHAPES = {V: ModelShape(0, 1, 64, 4, 4, 16, 64, V, rotary_dim=4) for V in (50304, 128256)}


@pytest.mark.parametrize("V", [50304, 128256])
def test_sampler_group_search_at_full_vocabulary(V):
    """The vocabularies of workloads 2-5 have 786 and 2004 groups of 64 columns, so every lane of the sampler's wave
    owns a run of several groups (the small shapes have at most 16 groups: one per lane).  (1) All-zero model: every
    logit is exactly 0 on both sides, token = floor(u V) and log-prob = -ln V with no rounding slack.  (2) Exact-logit
    model (final-norm gain 0, one-hot bias: the LM-head input is e_j, the logits column j of the bf16 LM head on both
    sides), flat and peaked: tokens must agree with the oracle's draw wherever its margin exceeds 1e-6, which at this
    vocabulary is only possible if the group search, the exclusive prefix and the in-group scan are all right."""
    m = BIG_VOCAB_SHAPES[V]
    r = R()
    W0 = make_weights(m, 1, bf16=False)
    zero = Weights(m, {k: np.zeros_like(v) for k, v in W0.tensors.items()}, False)
    pol = make_policy(zero, max_seqs=64, max_seq_len=40)
    rng = np.random.default_rng(135)
    u = rng.random((32, 2, 3), dtype=np.float32)
    u[0, 0, :] = [0.0, 0.99999994, (V - 0.5) / V]
    t, l = r.rlgen_generate(pol, dev_i32(np.zeros((32, 3), np.int32)), np.full(32, 3), 2, 3, 0.7, dev_f32(u))
    t, l = t.cpu().numpy(), l.cpu().numpy()
    uv = u.astype(np.float64) * V
    keep = np.abs(uv - np.round(uv)) > 1e-2           # the 2e-5-wide buckets sit 1e-2 buckets away from u
    np.testing.assert_array_equal(t[keep], np.floor(uv).astype(np.int32)[keep])
    assert keep.mean() > 0.9 and np.abs(l + math.log(V)).max() < 1e-5
    pol.close()
    from workloads import f32_to_bf16_bits
    for peak in (1.0, 8.0):
        Wp = scaled_bf16_weights(m, seed=36, scale=30.0, lm_head_scale=peak)
        tens = dict(Wp.tensors)
        b = np.zeros(m.d_model, np.float32)
        b[7] = 1.0
        tens["final_norm_g"], tens["final_norm_b"] = f32_to_bf16_bits(np.zeros(m.d_model, np.float32)), f32_to_bf16_bits(b)
        Wp = Weights(m, tens, True)
        dec = O.Decoder(Wp, m)
        pol = make_policy(Wp, max_seqs=256, max_seq_len=40, max_batch_tokens=256)
        Rr = 200
        hidden = rng.normal(size=(Rr, m.d_model)).astype(np.float32)
        uu = rng.random(Rr, dtype=np.float32)
        tok, lp = r.rlgen_debug_sample(pol, dev_f32(hidden), 0.7, dev_f32(uu))
        tok, lp = tok.cpu().numpy(), lp.cpu().numpy()
        logp = O.tempered_log_softmax(dec.logits(hidden[:1])[0], 0.7)       # every row has the same logits
        np.testing.assert_array_equal(dec.logits(hidden[:1])[0], Wp.f32("lm_head")[:, 7])
        checked = 0
        for i in range(Rr):
            want, margin = O.sample_inverse_cdf(logp, uu[i])
            lo, hi = O.cdf_bucket(logp, int(tok[i]))
            assert lo - 1e-6 <= uu[i] <= hi + 1e-6, (i, tok[i], want)       # a valid draw in any case
            if margin > 1e-6:
                assert tok[i] == want, (i, peak)
                checked += 1
            assert abs(lp[i] - logp[tok[i]]) < 2e-5
        report("sampler-big-vocab", V=V, peak=peak, checked=checked / Rr, max_p=float(np.exp(logp.max())))
        assert checked > (0.5 if peak == 1.0 else 0.9) * Rr
        pol.close()


# an FFN wide enough (K = 1024 for the down projection) that the K split of the decode GEMMs is more than one part
WIDE_FFN = ModelShape(0, 2, 64, 4, 4, 16, 1024, 200, rotary_dim=4)

@pytest.mark.parametrize("name", ["neox-h80", "llama-gqa4-h16", "neox-wide-ffn", "llama-gqa4-h16/precise", "neox-wide-ffn/precise"])
def test_results_do_not_depend_on_the_tile_shapes_a_context_picked(name):
    """A context chooses its GEMM tile shapes by timing them, so two contexts may choose differently; how a sum over the
    inner dimension is cut and ordered is fixed by the configuration.  Two contexts with the same weights are forced onto
    different tile shapes for every linear layer and every mode: tokens and log-probs must agree bit for bit."""
    name, _, mode = name.partition("/")
    precise = 1 if mode else 0
    m = WIDE_FFN if name == "neox-wide-ffn" else GPU_SHAPES[name]
    W = scaled_bf16_weights(m)
    r = R()
    rng = np.random.default_rng(91)
    prompts = rand_seqs(rng, m.vocab, [30, 1, 33, 64, 71])
    arr, lens = padded(prompts)
    u = rng.random((5, 2, 7), dtype=np.float32)
    outs, picks = [], []
    # contexts 0-2: the measured choice, and that choice moved on by one and by two in the list of legal shapes; then
    # (default formats) every layer that may take it forced onto the eight-wave small tile, and onto the sixteen-wave large one
    for shift in (0, 1, 2) if precise else (0, 1, 2, -9, -10):
        pol = make_policy(W, max_seqs=12, max_seq_len=80, max_batch_tokens=80, precise=precise)
        try:
            r.rlgen_set_decode_split_min(pol, 2 if shift == 2 else 0)      # the third context also decodes as two halves
            chosen = []
            for mode in (0, 1, 2):
                for which in range(5):
                    v0, sp = r.rlgen_debug_get_gemm(pol, mode, which)
                    wide_only = which == 4 or (which == 2 and m.arch == 1)
                    legal = [0, 3, 5] + ([] if wide_only else [7]) if precise else (list(range(6)) + [10] if wide_only else list(range(11)))
                    if shift < 0:
                        v = -shift if -shift in legal else v0
                    else:
                        v = v0 if shift == 0 else legal[(legal.index(max(v0, 0)) + shift) % len(legal)]
                    if shift:
                        r.rlgen_debug_set_gemm(pol, mode, which, v)
                    chosen.append((v, sp))
            picks.append(chosen)
            t, l = r.rlgen_generate(pol, dev_i32(arr), lens, 2, 7, 0.7, dev_f32(u))
            full, flens = padded([np.concatenate([prompts[b], t[b, j].cpu().numpy()]) for b in range(5) for j in range(2)])
            sc = r.rlgen_score(pol, dev_i32(full), flens, 0.7)
            z = r.rlgen_debug_logits(pol, dev_i32(full), flens)
            assert r.rlgen_status(pol) == 0
            outs.append((t.cpu(), l.cpu(), sc.cpu(), z.cpu()))
        finally:
            pol.close()
    assert all([sp for _, sp in p] == [sp for _, sp in picks[0]] for p in picks[1:])                  # the K split is the rule's
    assert [v for v, _ in picks[0]] != [v for v, _ in picks[1]]
    if name == "neox-wide-ffn":
        assert any(sp > 1 for _, sp in picks[0])                               # the test covers a split product
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            assert torch.equal(a, b)


def test_values_beyond_fp16_are_clamped_and_flagged():
    """The inputs of the matrix products are fp16.  A value just inside its range (60 000) passes unflagged and the result
    matches the oracle; a value beyond it (70 000) is clamped, never becomes infinity, and raises the sticky range bit.
    The large values meet zero weights (an LM-head column, an FFN-down column), so the oracle's result is the same in
    all three cases and the outputs must stay within tolerance of it."""
    from workloads import f32_to_bf16_bits, bf16_bits_to_f32
    m = GPU_SHAPES["neox-h80"]
    W = scaled_bf16_weights(m)
    r = R()
    rng = np.random.default_rng(92)
    seqs = rand_seqs(rng, m.vocab, [5, 40, 64])
    arr, lens = padded(seqs)

    def variant(final_bias, up_bias):
        t = dict(W.tensors)
        fb = bf16_bits_to_f32(t["final_norm_b"]).copy(); fb[5] = final_bias
        lm = bf16_bits_to_f32(t["lm_head"]).copy(); lm[:, 5] = 0.0
        bu = bf16_bits_to_f32(t["layers.0.b_up"]).copy(); bu[9] = up_bias
        wd = bf16_bits_to_f32(t["layers.0.w_down"]).copy(); wd[:, 9] = 0.0
        t.update({"final_norm_b": f32_to_bf16_bits(fb), "lm_head": f32_to_bf16_bits(lm), "layers.0.b_up": f32_to_bf16_bits(bu),
                  "layers.0.w_down": f32_to_bf16_bits(wd)})
        return Weights(m, t, True)

    for final_bias, up_bias, want_bits in ((60000.0, 60000.0, 0), (70000.0, 0.5, r.FAULT_RANGE), (0.5, 70000.0, r.FAULT_RANGE)):
        Wv = variant(final_bias, up_bias)
        ref = np.stack([O.last_logits(O.Decoder(Wv, m), s) for s in seqs])
        pol = make_policy(Wv, max_seqs=4, max_seq_len=80)
        try:
            z = r.rlgen_debug_logits(pol, dev_i32(arr), lens).cpu().numpy()
            sc = r.rlgen_score(pol, dev_i32(arr), lens, 0.7).cpu().numpy()
            assert r.rlgen_status_bits(pol) == want_bits, (final_bias, up_bias)
            assert r.rlgen_status(pol) == (r.ERR_DEVICE if want_bits else 0)
            assert np.isfinite(z).all() and np.isfinite(sc).all()
            assert np.abs(z - ref).max() < TOL_LOGITS, (final_bias, up_bias)
        finally:
            pol.close()


def test_config1_end_to_end():
    """Config 1 as specified: fp32 weights (the library rounds them to bf16), 4 prompts x 32 tokens,
    K = 2, 16 new tokens, temperature 0.7."""
    w = get_config(1)
    W = make_weights(w.model, w.seed_weights, w.bf16_weights)
    arr, lens = make_prompts(w)
    u = make_uniforms(w)
    dec = O.Decoder(W, w.model)
    pol = make_policy(W, max_seqs=w.n_prompts * w.k, max_seq_len=w.prompt_len_hi + w.max_new)
    r = R()
    t_o, l_o, margins, z_o, _ = oracle_generate_batch(dec, arr, lens, w.k, w.max_new, w.temperature, u)
    forced = np.where(margins > MARGIN, -1, t_o).astype(np.int32)
    t_g, l_g = r.rlgen_generate(pol, dev_i32(arr), lens, w.k, w.max_new, w.temperature, dev_f32(u), dev_i32(forced))
    np.testing.assert_array_equal(t_g.cpu().numpy(), t_o)
    assert np.abs(l_g.cpu().numpy() - l_o).max() < TOL_LOGPROB
    t_f, l_f = r.rlgen_generate(pol, dev_i32(arr), lens, w.k, w.max_new, w.temperature, dev_f32(u))
    t_f = t_f.cpu().numpy()
    _, l_t, _, z_t, buckets = oracle_generate_batch(dec, arr, lens, w.k, w.max_new, w.temperature, u, forced=t_f,
                                                    with_buckets=True)
    assert (buckets[..., 0] - MARGIN <= u).all() and (u <= buckets[..., 1] + MARGIN).all()
    assert np.abs(l_f.cpu().numpy() - l_t).max() < TOL_LOGPROB
    full = [np.concatenate([arr[b, :lens[b]], t_f[b, j]]) for b in range(w.n_prompts) for j in range(w.k)]
    farr, flens = padded(full)
    z_g = r.rlgen_debug_logits(pol, dev_i32(farr), flens).cpu().numpy()
    report("config1", logit_err=np.abs(z_g - z_t.reshape(len(full), -1)).max(), lp_err=np.abs(l_f.cpu().numpy() - l_t).max(),
           forced_fraction=(forced >= 0).mean(), z_std=z_t.std())
    assert np.abs(z_g - z_t.reshape(len(full), -1)).max() < TOL_LOGITS
    # the same model with weights pre-rounded to bf16 on the host: separates weight rounding from the rest
    decb = O.Decoder(W.rounded_to_bf16(), w.model)
    zb = np.stack([O.last_logits(decb, s) for s in full])
    assert np.abs(z_g - zb).max() <= np.abs(z_g - z_t.reshape(len(full), -1)).max() + 1e-3
    pol.close()


def test_argument_and_capacity_errors(small):
    m, W, dec, pol = small
    r = R()
    arr, lens = padded([[1, 2, 3], [4, 5]])
    u = dev_f32(np.zeros((2, 2, 4), np.float32))
    d = dev_i32(arr)

    def code(fn):
        with pytest.raises(r.RlgenError) as e:
            fn()
        return e.value.code

    assert code(lambda: r.rlgen_generate(pol, d, [3, 0], 2, 4, 0.7, u)) == r.ERR_BAD_ARG
    assert code(lambda: r.rlgen_generate(pol, d, [3, 4], 2, 4, 0.7, u)) == r.ERR_BAD_ARG          # longer than stride
    assert code(lambda: r.rlgen_generate(pol, d, lens, 2, 4, -0.5, u)) == r.ERR_BAD_ARG
    assert code(lambda: r.rlgen_generate(pol, d, lens, 2, 4, float("nan"), u)) == r.ERR_BAD_ARG
    assert code(lambda: r.rlgen_generate(pol, d, lens, 2, 4, -1.0, u)) == r.ERR_BAD_ARG
    big_u = dev_f32(np.zeros((2, 2, 78), np.float32))
    assert code(lambda: r.rlgen_generate(pol, d, lens, 2, 78, 0.7, big_u)) == r.ERR_CAPACITY      # 3 + 78 > 80
    many_u = dev_f32(np.zeros((2, 7, 4), np.float32))
    assert code(lambda: r.rlgen_generate(pol, d, lens, 7, 4, 0.7, many_u)) == r.ERR_CAPACITY      # 14 sequences > 12
    assert code(lambda: r.rlgen_score(pol, d, [3, 0], 0.7)) == r.ERR_BAD_ARG
    assert code(lambda: r.rlgen_score(pol, d, lens, 0.0)) == r.ERR_BAD_ARG
    long = dev_i32(np.zeros((1, 81), np.int32))
    assert code(lambda: r.rlgen_score(pol, long, [81], 0.7)) == r.ERR_CAPACITY
    assert r.rlgen_status(pol) == 0


def test_device_detected_faults_are_sticky_and_in_bounds():
    m = GPU_SHAPES["neox-h16-raggedV"]
    W = scaled_bf16_weights(m)
    pol = make_policy(W, max_seqs=4, max_seq_len=40)
    r = R()
    arr, lens = padded([[1, 2, m.vocab + 5], [4, -3, 0]])
    u = np.full((2, 1, 3), 0.5, np.float32)
    t, l = r.rlgen_generate(pol, dev_i32(arr), lens, 1, 3, 0.7, dev_f32(u))
    assert r.rlgen_status(pol) == r.ERR_DEVICE
    t = t.cpu().numpy()
    assert ((0 <= t) & (t < m.vocab)).all() and np.isfinite(l.cpu().numpy()).all()
    pol.close()
    pol = make_policy(W, max_seqs=4, max_seq_len=40)
    assert r.rlgen_status(pol) == 0
    u[0, 0, 1] = 1.0
    t, l = r.rlgen_generate(pol, dev_i32(np.array([[1, 2]], np.int32)), [2], 1, 3, 0.7, dev_f32(u[:1]))
    assert r.rlgen_status(pol) == r.ERR_DEVICE
    assert ((0 <= t.cpu().numpy()) & (t.cpu().numpy() < m.vocab)).all()
    pol.close()


def test_dpo_loss_and_sequence_logprob_match_oracle():
    rng = np.random.default_rng(38)
    r = R()
    N, stride = 37, 50
    tlp = -rng.random((N, stride)).astype(np.float32) * 5
    lens = rng.integers(1, stride + 1, size=N).astype(np.int32)
    start = np.minimum(rng.integers(0, stride, size=N), lens).astype(np.int32)
    got = r.rlgen_sequence_logprob(dev_f32(tlp), dev_i32(start), dev_i32(lens)).cpu().numpy()
    ref = np.array([O.sequence_logprob(tlp[i], start[i], lens[i]) for i in range(N)])
    assert np.abs(got - ref).max() < 1e-4
    P = 101
    a, b, c, d = (-(rng.random(P) * 200).astype(np.float32) for _ in range(4))
    for beta in (0.1, 0.05, 0.03):
        got = r.rlgen_dpo_loss(dev_f32(a), dev_f32(b), dev_f32(c), dev_f32(d), beta).cpu().numpy()
        ref = O.dpo_pair_loss(a.astype(np.float64), b.astype(np.float64), c.astype(np.float64), d.astype(np.float64), beta)
        assert np.abs(got - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())


def test_proximal_rloo_matches_oracle():
    rng = np.random.default_rng(40)
    r = R()
    for B, k, eps in ((1, 2, 0.2), (513, 2, 0.2), (300, 4, 0.1), (65, 7, 0.0)):
        lp_old = (-rng.random((B, k)) * 100).astype(np.float32)
        lp_pol = (lp_old + rng.standard_normal((B, k)).astype(np.float32) * 0.4).astype(np.float32)
        rew = rng.standard_normal((B, k)).astype(np.float32)
        got = r.rlgen_proximal_rloo(dev_f32(lp_pol), dev_f32(lp_old), dev_f32(rew), eps).cpu().numpy()
        ref = np.stack([O.proximal_rloo_objective(lp_pol[b], lp_old[b], rew[b], np.float64(np.float32(eps))) for b in range(B)])
        assert got.shape == (B, k)
        assert np.abs(got - ref).max() < 1e-5 * max(1.0, np.abs(ref).max())
    z = dev_f32(np.zeros((2, 1), np.float32))
    with pytest.raises(r.RlgenError) as e:
        r.rlgen_proximal_rloo(z, z, z, 0.2)                           # k = 1 has no baseline
    assert e.value.code == r.ERR_BAD_ARG


def test_select_pairs_matches_oracle():
    rng = np.random.default_rng(39)
    r = R()
    for B, k in ((1, 1), (513, 2), (300, 4), (65, 7)):
        rew = rng.integers(-2, 3, size=(B, k)).astype(np.float32)         # few distinct values: many ties
        rew[::3] += rng.standard_normal((len(rew[::3]), k)).astype(np.float32)
        pos, neg = r.rlgen_select_pairs(dev_f32(rew))
        ref = np.array([O.select_pair(row) for row in rew], np.int32)
        np.testing.assert_array_equal(pos.cpu().numpy(), ref[:, 0])
        np.testing.assert_array_equal(neg.cpu().numpy(), ref[:, 1])


def test_update_weights_replaces_the_policy():
    """The parameter hand-off of the asynchronous loop (Appendix D, Algorithm 1): after the update the context
    generates exactly what a context created with the new weights generates."""
    m = GPU_SHAPES["neox-h80"]
    r = R()
    W1, W2 = scaled_bf16_weights(m, seed=21), scaled_bf16_weights(m, seed=22)
    rng = np.random.default_rng(41)
    prompts = rand_seqs(rng, m.vocab, [17, 40, 5])
    arr, lens = padded(prompts)
    u = rng.random((3, 2, 6), dtype=np.float32)
    pol = make_policy(W1, max_seqs=6, max_seq_len=64)
    ref2 = make_policy(W2, max_seqs=6, max_seq_len=64)
    try:
        a1 = r.rlgen_generate(pol, dev_i32(arr), lens, 2, 6, 0.7, dev_f32(u))
        b2 = r.rlgen_generate(ref2, dev_i32(arr), lens, 2, 6, 0.7, dev_f32(u))
        assert not torch.equal(a1[1], b2[1])
        r.rlgen_update_weights(pol, r.upload_weights(W2.tensors))
        a2 = r.rlgen_generate(pol, dev_i32(arr), lens, 2, 6, 0.7, dev_f32(u))
        assert torch.equal(a2[0], b2[0]) and torch.equal(a2[1], b2[1])
        # and what the oracle generates from the new weights (the old ones give something else)
        t_o, l_o, margins, _, _ = oracle_generate_batch(O.Decoder(W2, m), arr, lens, 2, 6, 0.7, u)
        forced = np.where(margins > MARGIN, -1, t_o).astype(np.int32)
        t_g, l_g = r.rlgen_generate(pol, dev_i32(arr), lens, 2, 6, 0.7, dev_f32(u), dev_i32(forced))
        np.testing.assert_array_equal(t_g.cpu().numpy(), t_o)
        assert np.abs(l_g.cpu().numpy() - l_o).max() < TOL_LOGPROB
        _, l_old, _, _, _ = oracle_generate_batch(O.Decoder(W1, m), arr, lens, 2, 6, 0.7, u, forced=t_o)
        assert np.abs(l_g.cpu().numpy() - l_old).max() > 10 * TOL_LOGPROB
        farr, flens = padded([np.concatenate([prompts[b], a2[0][b, j].cpu().numpy()]) for b in range(3) for j in range(2)])
        assert torch.equal(r.rlgen_score(pol, dev_i32(farr), flens, 0.7), r.rlgen_score(ref2, dev_i32(farr), flens, 0.7))
    finally:
        pol.close()
        ref2.close()


# ---------------------------------------------------------------- prompt cache shared by the k samples of a prompt
@pytest.fixture(scope="module", params=list(GPU_SHAPES) + ["llama-gqa4-h16/precise", "neox-h80/precise"])
def shared(request):
    c = _case(request.param, max_seqs=20, max_seq_len=112, max_kv_tokens=2048, max_batch_tokens=112, share_prompt_kv=1)
    yield c
    c[3].close()


@pytest.mark.parametrize("k", [1, 2, 3, 5])
def test_shared_prompt_cache_matches_oracle(shared, k):
    """The k samples of a prompt read one copy of the prompt's keys and values; 35 new tokens cross a
    32-key block of the per-sample streams."""
    m, W, dec, pol = shared
    G = m.n_q_heads // m.n_kv_heads
    rng = np.random.default_rng(40 + k)
    B, T, temp = 4, (35 if k == 3 else 6), 0.7
    prompts = rand_seqs(rng, m.vocab, [31, 1, 64, 70])
    arr, lens = padded(prompts, pad=-1)
    u = rng.random((B, k, T), dtype=np.float32)
    r = R()
    if k * G > 16:
        with pytest.raises(r.RlgenError) as e:
            r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u))
        assert e.value.code == r.ERR_BAD_ARG
        return
    t_o, l_o, margins, _, _ = oracle_generate_batch(dec, arr, lens, k, T, temp, u)
    forced = np.where(margins > MARGIN, -1, t_o).astype(np.int32)
    t_g, l_g = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u), dev_i32(forced))
    t_g, l_g = t_g.cpu().numpy(), l_g.cpu().numpy()
    report("generate-shared-forced", err=np.abs(l_g - l_o).max(), mismatches=(t_g != t_o).sum(), k=k, h=m.head_dim)
    np.testing.assert_array_equal(t_g, t_o)
    assert np.abs(l_g - l_o).max() < TOL_LOGPROB
    # unforced: a valid draw under the oracle's CDF along the GPU's own path
    t_f, l_f = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u))
    t_f, l_f = t_f.cpu().numpy(), l_f.cpu().numpy()
    _, l_t, _, _, buckets = oracle_generate_batch(dec, arr, lens, k, T, temp, u, forced=t_f, with_buckets=True)
    assert (buckets[..., 0] - MARGIN <= u).all() and (u <= buckets[..., 1] + MARGIN).all()
    assert np.abs(l_f - l_t).max() < TOL_LOGPROB
    # scoring (per-sequence cache, prompt-pass kernels) agrees with the shared-cache decode
    full = [np.concatenate([prompts[b], t_f[b, j]]) for b in range(B) for j in range(k)]
    farr, flens = padded(full)
    sc = r.rlgen_score(pol, dev_i32(farr), flens, temp, np.repeat(lens, k)).cpu().numpy()
    for i in range(B * k):
        P = flens[i] - T
        assert np.abs(sc[i, P:flens[i]] - l_f.reshape(B * k, T)[i]).max() < TOL_LOGPROB
    # deterministic, and independent of what else is in the batch
    order = [2, 0, 3, 1]
    arr2, lens2 = padded([prompts[i] for i in order], pad=10 ** 7)
    t_2, l_2 = r.rlgen_generate(pol, dev_i32(arr2), lens2, k, T, temp, dev_f32(u[order]))
    assert np.array_equal(t_2.cpu().numpy(), t_f[order]) and np.array_equal(l_2.cpu().numpy(), l_f[order])
    assert r.rlgen_status(pol) == 0


def test_shared_prompt_cache_capacity(shared):
    """Cache need = sum of prompts rounded to 32 + sequences * new tokens rounded to 32 (here against 2048)."""
    m, W, dec, pol = shared
    if 2 * (m.n_q_heads // m.n_kv_heads) > 16:
        pytest.skip("k samples x query heads per kv head exceed the 16 MFMA columns")
    r = R()
    arr = np.zeros((8, 100), np.int32)
    lens = np.full(8, 100, np.int32)

    def run(B, k, T):
        return r.rlgen_generate(pol, dev_i32(arr[:B]), lens[:B], k, T, 0.7, dev_f32(np.full((B, k, T), 0.5, np.float32)))

    t, l = run(8, 2, 12)                       # 8 * 128 + 16 * 32 = 1536
    assert np.isfinite(l.cpu().numpy()).all()
    run(8, 2, 12)
    with pytest.raises(r.RlgenError) as e:
        run(8, 2, 13)                          # 100 + 13 > max_seq_len
    assert e.value.code == r.ERR_CAPACITY
    arr = np.zeros((16, 60), np.int32)
    lens = np.full(16, 60, np.int32)
    run(16, 1, 40)                             # 16 * 64 + 16 * 64 = 2048
    arr = np.zeros((16, 70), np.int32)
    lens = np.full(16, 70, np.int32)
    with pytest.raises(r.RlgenError) as e:
        run(16, 1, 40)                         # 16 * 96 + 16 * 64 = 2560 (one stream per sequence would need 16 * 128)
    assert e.value.code == r.ERR_CAPACITY


# ---------------------------------------------------------------- large batches decode as two concurrent halves
@pytest.mark.parametrize("share", [0, 1])
@pytest.mark.parametrize("name", ["neox-h80", "llama-gqa4-h16", "llama-gqa4-h16/precise"])
def test_split_decode_matches_oracle_and_unsplit(name, share):
    """The two-stream decode normally starts at 256 sequences; the threshold is lowered so that a batch the
    oracle can follow takes it (odd prompt count: the halves differ in size)."""
    m, W, dec, pol = _case(name, max_seqs=12, max_seq_len=80, max_batch_tokens=80, share_prompt_kv=share)
    R().rlgen_set_decode_split_min(pol, 2)
    try:
        rng = np.random.default_rng(77)
        B, k, T, temp = 5, 2, 7, 0.7
        prompts = rand_seqs(rng, m.vocab, [30, 1, 33, 64, 71])
        arr, lens = padded(prompts, pad=-1)
        u = rng.random((B, k, T), dtype=np.float32)
        r = R()
        t_o, l_o, margins, _, _ = oracle_generate_batch(dec, arr, lens, k, T, temp, u)
        forced = np.where(margins > MARGIN, -1, t_o).astype(np.int32)
        t_g, l_g = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u), dev_i32(forced))
        np.testing.assert_array_equal(t_g.cpu().numpy(), t_o)
        assert np.abs(l_g.cpu().numpy() - l_o).max() < TOL_LOGPROB
        t_a, l_a = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u))
        r.rlgen_set_decode_split(pol, False)
        t_b, l_b = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u))
        r.rlgen_set_decode_split(pol, True)
        assert torch.equal(t_a, t_b) and torch.equal(l_a, l_b)          # bit for bit
        assert r.rlgen_status(pol) == 0
    finally:
        pol.close()


# ---------------------------------------------------------------- greedy decoding and completions that end at EOS
GREEDY_MARGIN = 2 * TOL_LOGITS        # the oracle's arg max is unambiguous when its lead exceeds both sides' logit error


@pytest.mark.parametrize("share", [0, 1])
def test_greedy_matches_oracle(small, share):
    m, W, dec, pol0 = small
    if share and 2 * (m.n_q_heads // m.n_kv_heads) > 16:
        pytest.skip("k samples x query heads per kv head exceed the 16 MFMA columns: rejected, see test_shared_prompt_cache_matches_oracle")
    pol = pol0 if not share else make_policy(W, max_seqs=12, max_seq_len=80, max_batch_tokens=80, share_prompt_kv=1, precise=small.precise)
    try:
        rng = np.random.default_rng(51)
        B, k, T = 4, 2, 8
        prompts = rand_seqs(rng, m.vocab, [9, 33, 1, 64])
        arr, lens = padded(prompts)
        u = np.full((B, k, T), 0.123, np.float32)
        r = R()
        t_o, l_o, margins, _, _ = oracle_generate_batch(dec, arr, lens, k, T, 0.0, u)
        forced = np.where(margins > GREEDY_MARGIN, -1, t_o).astype(np.int32)
        t_g, l_g = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, 0.0, dev_f32(u), dev_i32(forced))
        t_g, l_g = t_g.cpu().numpy(), l_g.cpu().numpy()
        report("greedy", err=np.abs(l_g - l_o).max(), free=(forced < 0).mean(), h=m.head_dim)
        np.testing.assert_array_equal(t_g, t_o)
        assert np.abs(l_g - l_o).max() < TOL_LOGPROB
        assert (forced < 0).mean() > 0.3
        np.testing.assert_array_equal(t_g[:, 0], t_g[:, 1])          # both samples of a prompt are the same completion
        # unforced: along the GPU's own path every token's logit is within the logit tolerance of the oracle's maximum
        t_f, _ = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, 0.0, dev_f32(u))
        t_f = t_f.cpu().numpy()
        for b in range(B):
            seq = list(prompts[b])
            for t in range(T):
                z = O.last_logits(dec, seq)
                assert z[t_f[b, 0, t]] >= z.max() - GREEDY_MARGIN
                seq.append(int(t_f[b, 0, t]))
        assert r.rlgen_status(pol) == 0
    finally:
        if share:
            pol.close()


@pytest.mark.parametrize("share", [0, 1])
@pytest.mark.parametrize("temp", [0.7, 0.0])
def test_eos_ends_completions(small, temp, share):
    """Ended completions report EOS at log-prob 0 from then on, and decode attention stops reading their cache
    (with a shared prompt cache: the prompt's stream is skipped once all its samples have ended)."""
    m, W, dec, pol0 = small
    if share and 2 * (m.n_q_heads // m.n_kv_heads) > 16:
        pytest.skip("k samples x query heads per kv head exceed the 16 MFMA columns")
    if share:
        pol = make_policy(W, max_seqs=12, max_seq_len=80, max_batch_tokens=80, share_prompt_kv=1, precise=small.precise)
        try:
            _check_eos(m, dec, pol, temp)
        finally:
            pol.close()
    else:
        _check_eos(m, dec, pol0, temp)


def _check_eos(m, dec, pol, temp):
    rng = np.random.default_rng(52)
    B, k, T = 5, 2, 9
    prompts = rand_seqs(rng, m.vocab, [12, 40, 3, 64, 21])
    arr, lens = padded(prompts)
    u = rng.random((B, k, T), dtype=np.float32)
    r = R()
    t0, _, _, _, _ = oracle_generate_batch(dec, arr, lens, k, T, temp, u)
    eos = int(np.bincount(t0[:, :, 2:6].ravel()).argmax())            # a token several completions emit mid-way
    t_o, l_o, margins, _, _ = oracle_generate_batch(dec, arr, lens, k, T, temp, u, eos=eos)
    ended = (t_o == eos).any(axis=2)
    assert ended.any() and (t_o[:, :, -1] == eos).any()
    forced = np.where(margins > (MARGIN if temp > 0 else GREEDY_MARGIN), -1, t_o).astype(np.int32)
    try:
        r.rlgen_set_eos(pol, eos)
        t_g, l_g = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u), dev_i32(forced))
        t_g, l_g = t_g.cpu().numpy(), l_g.cpu().numpy()
        np.testing.assert_array_equal(t_g, t_o)
        assert np.abs(l_g - l_o).max() < TOL_LOGPROB
        after = np.cumsum(np.cumsum(t_o == eos, axis=2), axis=2) > 1      # strictly after the first EOS
        assert (l_g[after] == 0).all() and (t_g[after] == eos).all()
        with pytest.raises(r.RlgenError):
            r.rlgen_set_eos(pol, m.vocab)
    finally:
        r.rlgen_set_eos(pol, -1)
    t_n, _ = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u), dev_i32(np.where(forced >= 0, t0, -1).astype(np.int32)))
    assert r.rlgen_status(pol) == 0


# ---------------------------------------------------------------- degenerate sizes
@pytest.mark.parametrize("share", [0, 1])
def test_degenerate_sizes(small, share):
    """One prompt of one token, one sample, one new token (no decode step at all); then the context filled to its
    exact capacity in sequences, sequence length and cache tokens; with the two-stream decode forced on."""
    m, W, dec, _ = small
    if share and 3 * (m.n_q_heads // m.n_kv_heads) > 16:
        pytest.skip("k samples x query heads per kv head exceed the 16 MFMA columns")
    r = R()
    S, L = 6, 40
    need = S * 64 if not share else 3 * 32 + S * 32            # 3 prompts x 2 samples: prompts of 8 + 32 new tokens
    pol = make_policy(W, max_seqs=S, max_seq_len=L, max_kv_tokens=need, max_batch_tokens=L, share_prompt_kv=share, precise=small.precise)
    r.rlgen_set_decode_split_min(pol, 2)
    try:
        rng = np.random.default_rng(61)
        for B, k, P, T in ((1, 1, 1, 1), (1, 1, L - 1, 1), (3, 2, 8, 32), (2, 3, 8, 1)):
            prompts = rand_seqs(rng, m.vocab, [P] * B)
            arr, lens = padded(prompts)
            u = rng.random((B, k, T), dtype=np.float32)
            t_o, l_o, margins, _, _ = oracle_generate_batch(dec, arr, lens, k, T, 0.7, u)
            forced = np.where(margins > MARGIN, -1, t_o).astype(np.int32)
            t_g, l_g = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, 0.7, dev_f32(u), dev_i32(forced))
            np.testing.assert_array_equal(t_g.cpu().numpy(), t_o)
            assert np.abs(l_g.cpu().numpy() - l_o).max() < TOL_LOGPROB, (B, k, P, T)
        with pytest.raises(r.RlgenError) as e:                   # one more new token than the cache holds
            r.rlgen_generate(pol, dev_i32(arr), lens, 3, 33 if share else 57, 0.7, dev_f32(np.zeros((2, 3, 33 if share else 57), np.float32)))
        assert e.value.code == r.ERR_CAPACITY
        assert r.rlgen_status(pol) == 0
    finally:
        pol.close()


@pytest.mark.parametrize("every", [1, 2, 5])
@pytest.mark.parametrize("name", ["neox-h80", "llama-gqa4-h16", "llama-gqa4-h16/precise"])
def test_ended_sequences_leave_the_batch(name, every):
    """EOS is forced at chosen steps of chosen sequences (a forced token counts as emitted on both sides), so the
    batch shrinks several times, down to nothing before the last step in one case; outputs must match the oracle
    and, bit for bit, a context that keeps ended sequences in the batch."""
    precise = 1 if name.endswith("/precise") else 0
    m = GPU_SHAPES[name.partition("/")[0]]
    W = scaled_bf16_weights(m)
    dec = reference_decoder(W, m, precise)
    rng = np.random.default_rng(71)
    B, k, T, temp = 4, 2, 14, 0.7
    prompts = rand_seqs(rng, m.vocab, [30, 5, 64, 17])
    arr, lens = padded(prompts)
    u = rng.random((B, k, T), dtype=np.float32)
    eos = 3
    r = R()
    for schedule in ({0: 0, 1: 1, 2: 2, 5: 3, 7: 9}, {q: q % 3 for q in range(8)}):      # sequence -> step of its EOS
        plan = np.full((B * k, T), -1, np.int32)
        for q, t in schedule.items():
            plan[q, t] = eos
        plan = plan.reshape(B, k, T)
        t_o, l_o, margins, _, _ = oracle_generate_batch(dec, arr, lens, k, T, temp, u, forced=plan, eos=eos)
        forced = np.where(plan >= 0, plan, np.where(margins > MARGIN, -1, t_o)).astype(np.int32)
        outs = []
        for ev in (every, 0):
            pol = make_policy(W, max_seqs=8, max_seq_len=80, max_batch_tokens=80, precise=precise)
            try:
                r.rlgen_set_eos_compaction(pol, ev)
                r.rlgen_set_eos(pol, eos)
                t_g, l_g = r.rlgen_generate(pol, dev_i32(arr), lens, k, T, temp, dev_f32(u), dev_i32(forced))
                assert r.rlgen_status(pol) == 0
                outs.append((t_g.cpu().numpy(), l_g.cpu().numpy()))
            finally:
                pol.close()
        np.testing.assert_array_equal(outs[0][0], t_o)
        assert np.abs(outs[0][1] - l_o).max() < TOL_LOGPROB
        np.testing.assert_array_equal(outs[0][0], outs[1][0])
        np.testing.assert_array_equal(outs[0][1], outs[1][1])
        ended_at = {q: t for q, t in schedule.items()}
        flat_t, flat_l = outs[0][0].reshape(B * k, T), outs[0][1].reshape(B * k, T)
        for q, t in ended_at.items():
            assert (flat_t[q, t:] == eos).all() and (flat_l[q, t + 1:] == 0).all()


# ---------------------------------------------------------------- scoring a prompt's k completions with the prompt shared
@pytest.mark.parametrize("k", [2, 3])
def test_grouped_score_matches_oracle_and_plain(small, k):
    m, W, dec, pol = small
    rng = np.random.default_rng(81 + k)
    r = R()
    #            prompt length, completion lengths (0: a member that is the bare prompt)
    groups = [(30, [9, 1, 0][:k] + [5] * (k - 3)), (1, [20] * k), (33, [17, 16, 15][:k]), (16, [1] * k), (40, [30, 10, 20][:k])]
    if k == 3:
        groups = groups[:3] + groups[4:]          # 12 sequences: the context's capacity
    seqs, from_ = [], []
    for P, tails in groups:
        prompt = rng.integers(0, m.vocab, size=P)
        for L in tails:
            seqs.append(np.concatenate([prompt, rng.integers(0, m.vocab, size=L)]))
            from_.append(P)
    arr, lens = padded(seqs, pad=-3)
    from_ = np.array(from_, np.int32)
    plain = r.rlgen_score(pol, dev_i32(arr), lens, 0.7, from_).cpu().numpy()
    try:
        r.rlgen_set_score_groups(pol, k)
        got = r.rlgen_score(pol, dev_i32(arr), lens, 0.7, from_).cpu().numpy()
        assert r.rlgen_status(pol) == 0
        # the last group (40 + tails) does not fit a chunk of 80 rows when k = 3: the call then scores plainly
        for i, sq in enumerate(seqs):
            ref = O.score(dec, sq, 0.7, from_[i])
            assert np.abs(got[i, :len(sq)] - ref).max() < TOL_LOGPROB, i
            assert (got[i, len(sq):] == 0).all() and (got[i, :from_[i]] == 0).all()
        report("score-grouped", vs_plain=np.abs(got - plain).max(), k=k, h=m.head_dim)
        assert np.abs(got - plain).max() < TOL_LOGPROB
        # argument checks: N not a multiple of k, unequal score_from in a group, score_from beyond a member
        with pytest.raises(r.RlgenError):
            r.rlgen_score(pol, dev_i32(arr[:k + 1]), lens[:k + 1], 0.7, from_[:k + 1])
        bad = from_.copy(); bad[1] += 1
        with pytest.raises(r.RlgenError):
            r.rlgen_score(pol, dev_i32(arr), lens, 0.7, bad)
        with pytest.raises(r.RlgenError):
            r.rlgen_score(pol, dev_i32(arr), lens, 0.7, None)
    finally:
        r.rlgen_set_score_groups(pol, 1)
    # a member whose "shared" part differs is detected on the device (the flag is sticky: a context of its own)
    pol2 = make_policy(W, max_seqs=len(seqs), max_seq_len=80, precise=small.precise)
    try:
        r.rlgen_set_score_groups(pol2, k)
        r.rlgen_score(pol2, dev_i32(arr), lens, 0.7, from_)
        assert r.rlgen_status(pol2) == 0
        arr2 = arr.copy(); arr2[2 * k + 1, 5] = (arr2[2 * k + 1, 5] + 1) % m.vocab
        r.rlgen_score(pol2, dev_i32(arr2), lens, 0.7, from_)
        # (a model whose rotary width is not a multiple of 4 takes the separate rotary kernel, where grouping is off)
        assert r.rlgen_status(pol2) == (r.ERR_DEVICE if m.rotary_dim % 4 == 0 else 0)
    finally:
        pol2.close()
