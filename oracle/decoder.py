"""CPU oracle for the generation hot path of asynchronous online-DPO RLHF.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the HIP
library is checked against.  Only tests, the smoke check and the bench's CPU-baseline
leg may import it; the product path never does, and it shares no code with the HIP
sources.

What it computes (paper: Section 2.1, the Online DPO objective; Appendix D, Algorithm 1,
procedure Generate): K completions per prompt drawn autoregressively from the policy
pi_theta at a temperature (0.7 in Appendix A.1-A.3), and log pi(y_t | x, y_<t) of each
drawn token -- the per-token terms of log pi_theta(y|x) in the DPO objective and of
pi_old in the importance ratio of Appendix B, Eq. 1.

The paper does not define the policy network; the two decoder families it trains
(Pythia = GPT-NeoX, Llama-3.1) are implemented here from their public definitions:

  GPT-NeoX block:  a = LN1(x), m = LN2(x)
                   x <- x + Wo.attn(a) + bo + Wdown.gelu(Wup.m + bup) + bdown   (parallel residual)
  Llama block:     x <- x + Wo.attn(RMS1(x));  x <- x + Wdown.(silu(Wgate.m) * (Wup.m)), m = RMS2(x)

Rotary position embedding uses the half-split pairing (i, i + r/2) on the first r
dimensions of every head; Llama-3.1's long-context frequency rescaling is not applied.

Precision: matrix products in `dt` (float32 by default, float64 on request);
normalisation statistics, softmax, log-sum-exp and the CDF scan in float64.

Parity pins (tests/test_oracle_*.py): KV-cached decode against cache-free recompute,
softmax rows summing to one, causality, explicit CDF scan, CDF buckets tiling [0, 1) and
holding the uniform of the drawn token, sequence log-probs against exact sums, zero-weight closed forms,
temperature/LM-head equivalence, GQA replication, rotary against complex
multiplication, pieces against scipy/torch CPU routines, whole model against the
installed `transformers` classes used as a black box.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence

import numpy as np
from scipy.special import erf

ARCH_NEOX = 0
ARCH_LLAMA = 1


# ----------------------------------------------------------------------------- pieces

def layer_norm(x, g, b, eps, dt=np.float32):
    """(x - mean) / sqrt(biased variance + eps) * g + b over the last axis; statistics in float64."""
    x64 = x.astype(np.float64)
    mu = x64.mean(axis=-1, keepdims=True)
    var = ((x64 - mu) ** 2).mean(axis=-1, keepdims=True)
    y = (x64 - mu) / np.sqrt(var + eps)
    return (y * g.astype(np.float64) + b.astype(np.float64)).astype(dt)


def rms_norm(x, g, eps, dt=np.float32):
    """x / sqrt(mean(x^2) + eps) * g over the last axis; statistics in float64."""
    x64 = x.astype(np.float64)
    ms = (x64 ** 2).mean(axis=-1, keepdims=True)
    return (x64 / np.sqrt(ms + eps) * g.astype(np.float64)).astype(dt)


def gelu(t, dt=np.float32):
    """Exact (erf) form: t/2 * (1 + erf(t / sqrt 2))."""
    t64 = t.astype(np.float64)
    return (0.5 * t64 * (1.0 + erf(t64 / math.sqrt(2.0)))).astype(dt)


def silu(t, dt=np.float32):
    t64 = t.astype(np.float64)
    return (t64 / (1.0 + np.exp(-t64))).astype(dt)


def rotary(u, pos, rotary_dim, theta, dt=np.float32):
    """Rotate the first `rotary_dim` dims of every head.  u: [n, H, h]; pos: [n] integer positions.

    Pair (i, i + r/2) is rotated by the angle pos * theta^(-2i/r); angles in float64, cos and
    sin cast to `dt`.  Dimensions r..h-1 pass through unchanged."""
    r = rotary_dim
    half = r // 2
    i = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / r)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]      # [n, r/2]
    c = np.cos(ang).astype(dt)[:, None, :]
    s = np.sin(ang).astype(dt)[:, None, :]
    out = u.astype(dt, copy=True)
    a = u[..., :half].astype(dt)
    b = u[..., half:r].astype(dt)
    out[..., :half] = a * c - b * s
    out[..., half:r] = b * c + a * s
    return out


def attention(q, k, v, qpos, dt=np.float32):
    """Causal softmax attention.  q: [n, Hq, h]; k, v: [m, Hkv, h] where key s sits at position s;
    query i sees keys s <= qpos[i].  Query head j reads KV head j // (Hq / Hkv).  Softmax in float64."""
    n, Hq, h = q.shape
    m, Hkv, _ = k.shape
    group = Hq // Hkv
    scale = 1.0 / math.sqrt(h)
    visible = np.arange(m)[None, :] <= np.asarray(qpos)[:, None]
    out = np.empty((n, Hq, h), dtype=dt)
    for j in range(Hq):
        kj, vj = k[:, j // group, :], v[:, j // group, :]
        s = (q[:, j, :] @ kj.T).astype(np.float64) * scale
        s = np.where(visible, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, j, :] = p.astype(dt) @ vj
    return out


def linear(x, W, b=None):
    y = x @ W.T
    return y if b is None else y + b


# ----------------------------------------------------------------------------- the decoder

class KVCache:
    """Per layer: rotated keys and values of every position processed so far, [n, Hkv, h]."""

    def __init__(self, n_layers: int):
        self.k: List[Optional[np.ndarray]] = [None] * n_layers
        self.v: List[Optional[np.ndarray]] = [None] * n_layers
        self.length = 0

    def append(self, layer, k, v):
        self.k[layer] = k if self.k[layer] is None else np.concatenate([self.k[layer], k], axis=0)
        self.v[layer] = v if self.v[layer] is None else np.concatenate([self.v[layer], v], axis=0)

    def copy(self) -> "KVCache":
        c = KVCache(len(self.k))
        c.k = [None if a is None else a.copy() for a in self.k]
        c.v = [None if a is None else a.copy() for a in self.v]
        c.length = self.length
        return c


class Decoder:
    """A decoder-only transformer over a `workloads.Weights`-like object W (W.f32(name), W.has(name))
    and a model shape m (fields as in workloads.ModelShape)."""

    def __init__(self, W, m, dt=np.float32):
        self.W, self.m, self.dt = W, m, dt

    def w(self, name):
        t = self.W.f32(name)
        return t if t.dtype == self.dt else t.astype(self.dt)

    def lw(self, layer, name):
        return self.w(f"layers.{layer}.{name}")

    def _self_attention(self, layer, a, pos, cache: KVCache, biased: bool):
        m, dt = self.m, self.dt
        n = a.shape[0]
        q = linear(a, self.lw(layer, "wq"), self.lw(layer, "bq") if biased else None)
        k = linear(a, self.lw(layer, "wk"), self.lw(layer, "bk") if biased else None)
        v = linear(a, self.lw(layer, "wv"), self.lw(layer, "bv") if biased else None)
        q = rotary(q.reshape(n, m.n_q_heads, m.head_dim), pos, m.rotary_dim, m.rope_theta, dt)
        k = rotary(k.reshape(n, m.n_kv_heads, m.head_dim), pos, m.rotary_dim, m.rope_theta, dt)
        v = v.reshape(n, m.n_kv_heads, m.head_dim).astype(dt)
        cache.append(layer, k, v)
        o = attention(q, cache.k[layer], cache.v[layer], pos, dt)
        return linear(o.reshape(n, m.n_q_heads * m.head_dim), self.lw(layer, "wo"),
                      self.lw(layer, "bo") if biased else None)

    def _block(self, layer, x, pos, cache):
        m, dt = self.m, self.dt
        if m.arch == ARCH_NEOX:
            a = layer_norm(x, self.lw(layer, "norm1_g"), self.lw(layer, "norm1_b"), m.norm_eps, dt)
            mm = layer_norm(x, self.lw(layer, "norm2_g"), self.lw(layer, "norm2_b"), m.norm_eps, dt)
            attn = self._self_attention(layer, a, pos, cache, biased=True)
            up = gelu(linear(mm, self.lw(layer, "w_up"), self.lw(layer, "b_up")), dt)
            mlp = linear(up, self.lw(layer, "w_down"), self.lw(layer, "b_down"))
            return (x + attn + mlp).astype(dt)
        elif m.arch == ARCH_LLAMA:
            a = rms_norm(x, self.lw(layer, "norm1_g"), m.norm_eps, dt)
            x = (x + self._self_attention(layer, a, pos, cache, biased=False)).astype(dt)
            mm = rms_norm(x, self.lw(layer, "norm2_g"), m.norm_eps, dt)
            act = silu(linear(mm, self.lw(layer, "w_gate")), dt) * linear(mm, self.lw(layer, "w_up"))
            return (x + linear(act.astype(dt), self.lw(layer, "w_down"))).astype(dt)
        raise ValueError("unknown arch")

    def forward(self, tokens: Sequence[int], cache: KVCache):
        """Run the stack on `tokens`, which continue the sequence held in `cache`.
        Returns the residual stream after the last block, [n, d]."""
        tokens = np.asarray(tokens, dtype=np.int64)
        if tokens.min() < 0 or tokens.max() >= self.m.vocab:
            raise ValueError("token id out of range")
        pos = cache.length + np.arange(len(tokens))
        x = self.w("embed_in")[tokens].astype(self.dt)
        for layer in range(self.m.n_layers):
            x = self._block(layer, x, pos, cache)
        cache.length += len(tokens)
        return x

    def logits(self, x):
        """Raw (temperature 1) logits of residual rows x [n, d] -> [n, V]."""
        m, dt = self.m, self.dt
        if m.arch == ARCH_NEOX:
            hfin = layer_norm(x, self.w("final_norm_g"), self.w("final_norm_b"), m.norm_eps, dt)
        else:
            hfin = rms_norm(x, self.w("final_norm_g"), m.norm_eps, dt)
        return hfin @ self.w("lm_head").T


# ----------------------------------------------------------------------------- scoring and sampling

def tempered_log_softmax(z, temperature):
    """log softmax(z / T) in float64 for one row or a stack of rows of raw logits."""
    l = (z / z.dtype.type(temperature)).astype(np.float64)
    mx = l.max(axis=-1, keepdims=True)
    logZ = mx + np.log(np.exp(l - mx).sum(axis=-1, keepdims=True))
    return l - logZ


def sample_inverse_cdf(logp, u):
    """Inverse-CDF draw from one row of float64 log-probabilities with a uniform u in [0, 1).

    C_j = p_0 + ... + p_j accumulated in ascending index order; token = the first j with C_j > u;
    if rounding leaves no such j, the last token with p_j > 0.  Also returns the margin: the
    distance from u to the nearer edge of the chosen token's CDF bucket (upper edge 1 for the last
    positive-probability token)."""
    p = np.exp(logp)
    C = np.cumsum(p)
    u = float(u)
    V = len(p)
    tok = int(np.searchsorted(C, u, side="right"))
    last_pos = int(np.nonzero(p > 0)[0][-1])
    if tok >= V:
        tok = last_pos
    lower = C[tok - 1] if tok > 0 else 0.0
    upper = 1.0 if tok == last_pos else C[tok]
    return tok, min(u - lower, upper - u)


def cdf_bucket(logp, tok):
    """[C_{tok-1}, C_tok]: the interval of uniforms that the ascending-order CDF maps to `tok`."""
    C = np.cumsum(np.exp(logp))
    return (float(C[tok - 1]) if tok > 0 else 0.0), float(C[tok])


def greedy_pick(z):
    """Greedy decoding (Section 5.2: evaluation draws one completion per question greedily): the first index of
    the largest logit; its log-prob is taken under softmax(z) (temperature 1); the margin is the gap to the
    runner-up logit."""
    z = np.asarray(z, np.float64)
    tok = int(np.argmax(z))
    rest = np.delete(z, tok)
    margin = float(z[tok] - rest.max()) if len(rest) else np.inf
    return tok, margin


def generate(dec: Decoder, prompt, k, max_new, temperature, uniforms, forced=None,
             return_final_logits=False, buckets=None, eos=-1):
    """K completions of `max_new` tokens for one prompt (Algorithm 1, procedure Generate).

    uniforms: [k, max_new]; forced: optional [k, max_new] ints, entries >= 0 replace the draw.
    Returns tokens [k, max_new] int32, logprobs [k, max_new] float32 (of the emitted token under
    softmax(z / T)), margins [k, max_new] float64 (of the oracle's own draw).  The prompt is
    processed once; each sample continues from a copy of its KV cache.  If `buckets` is a float64
    array [k, max_new, 2] it receives the CDF interval of every emitted token.
    temperature == 0 decodes greedily (greedy_pick; uniforms are ignored).
    eos >= 0: a completion ends with its first `eos` token (the completions the paper scores end in an EOS token
    or are penalised for lacking one, Appendix A.1 / A.2 hyper-parameter tables); the remaining entries are
    filled with `eos` at log-prob 0 and margin inf."""
    uniforms = np.asarray(uniforms)
    assert uniforms.shape == (k, max_new)
    base = KVCache(dec.m.n_layers)
    x_last = dec.forward(prompt, base)[-1:]
    toks = np.zeros((k, max_new), np.int32)
    lps = np.zeros((k, max_new), np.float32)
    margins = np.zeros((k, max_new), np.float64)
    final_logits = []
    for j in range(k):
        cache, x = base.copy(), x_last
        done = False
        for t in range(max_new):
            if done:
                toks[j, t], lps[j, t], margins[j, t] = eos, 0.0, np.inf
                if buckets is not None:
                    buckets[j, t] = (0.0, 1.0)
                continue
            z = dec.logits(x)[0]
            if temperature == 0:
                logp = tempered_log_softmax(z, 1.0)
                tok, margins[j, t] = greedy_pick(z)
            else:
                logp = tempered_log_softmax(z, temperature)
                tok, margins[j, t] = sample_inverse_cdf(logp, uniforms[j, t])
            if forced is not None and forced[j][t] >= 0:
                tok = int(forced[j][t])
            toks[j, t], lps[j, t] = tok, logp[tok]
            if buckets is not None:
                buckets[j, t] = cdf_bucket(logp, tok)
            done = eos >= 0 and tok == eos
            if (t + 1 < max_new and not done) or return_final_logits:
                x = dec.forward([tok], cache)
        if return_final_logits:
            final_logits.append(dec.logits(x)[0])
    if return_final_logits:
        return toks, lps, margins, np.stack(final_logits)
    return toks, lps, margins


def generate_full_recompute(dec: Decoder, prompt, max_new, temperature, uniforms):
    """One completion without a KV cache: the whole prefix is re-run from scratch for every token.
    Returns tokens, logprobs and the raw logits used at every step."""
    seq = list(int(t) for t in prompt)
    toks, lps, zs = [], [], []
    for t in range(max_new):
        z = dec.logits(dec.forward(seq, KVCache(dec.m.n_layers))[-1:])[0]
        logp = tempered_log_softmax(z, temperature)
        tok, _ = sample_inverse_cdf(logp, uniforms[t])
        toks.append(tok), lps.append(np.float32(logp[tok])), zs.append(z)
        seq.append(tok)
    return np.array(toks, np.int32), np.array(lps, np.float32), np.stack(zs)


def score(dec: Decoder, seq, temperature, score_from=1):
    """Teacher-forced log-probabilities: out[t] = log softmax(z_{t-1} / T)[seq[t]] for
    max(1, score_from) <= t < len(seq), zero elsewhere.  Summed over the response positions this is
    log pi(y | x) of the DPO objective (Section 2.1)."""
    seq = np.asarray(seq, dtype=np.int64)
    n = len(seq)
    out = np.zeros(n, np.float32)
    lo = max(1, int(score_from))
    if lo >= n:
        return out
    x = dec.forward(seq, KVCache(dec.m.n_layers))
    logp = tempered_log_softmax(dec.logits(x[lo - 1:n - 1]), temperature)
    out[lo:] = logp[np.arange(n - lo), seq[lo:]]
    return out


def last_logits(dec: Decoder, seq):
    """Raw logits at the last position of `seq`."""
    return dec.logits(dec.forward(seq, KVCache(dec.m.n_layers))[-1:])[0]


# ----------------------------------------------------------------------------- consumers of the log-probs

def dpo_pair_loss(lp_pol_pos, lp_ref_pos, lp_pol_neg, lp_ref_neg, beta):
    """-log sigmoid(beta [ (log pi(y+) - log pi_init(y+)) - (log pi(y-) - log pi_init(y-)) ]) per pair
    (Section 2.1, DPO objective; the paper maximises log sigmoid, the loss is its negative).
    Arguments are sequence log-probabilities (sums of response-token log-probs), float64."""
    d = beta * ((np.asarray(lp_pol_pos, np.float64) - lp_ref_pos) - (np.asarray(lp_pol_neg, np.float64) - lp_ref_neg))
    return np.logaddexp(0.0, -d)


def proximal_rloo_objective(lp_pol, lp_old, rewards, epsilon):
    """Clipped importance-weighted RLOO objective of every one of a prompt's k >= 2 completions (Appendix B, Eq. 1):
    min(r A, clip(r, 1 - eps, 1 + eps) A) with r = pi_theta(y|x) / pi_old(y|x) = exp(lp_pol - lp_old) and A the
    completion's reward minus the baseline.  The appendix writes the baseline for k = 2 (the other completion's
    reward); for k > 2 this takes RLOO's leave-one-out mean of the other k - 1 rewards, which is the same thing at
    k = 2.  Arguments are [k] sequence log-probabilities and rewards; float64 throughout."""
    lp_pol = np.asarray(lp_pol, np.float64)
    lp_old = np.asarray(lp_old, np.float64)
    rew = np.asarray(rewards, np.float64)
    k = len(rew)
    out = np.zeros(k, np.float64)
    for i in range(k):
        baseline = sum(rew[j] for j in range(k) if j != i) / (k - 1)
        adv = rew[i] - baseline
        ratio = np.exp(lp_pol[i] - lp_old[i])
        clipped = min(max(ratio, 1.0 - epsilon), 1.0 + epsilon)
        out[i] = min(ratio * adv, clipped * adv)
    return out


def select_pair(rewards):
    """Indices (y+, y-) of the highest and the lowest rewarded of a prompt's K completions (Section 2.1: two samples
    ranked by the reward model; Section 4.2: of K samples only the highest and the lowest are trained on).  The
    paper does not say what happens on ties: here y+ is the first of the highest and y- the last of the lowest, so
    the two differ whenever K >= 2."""
    r = [float(x) for x in rewards]
    pos, neg = 0, 0
    for j in range(len(r)):
        if r[j] > r[pos]:
            pos = j
        if r[j] <= r[neg]:
            neg = j
    return pos, neg


def sequence_logprob(token_logprobs, score_from, length):
    """Sum of token log-probs over positions score_from <= t < length, in float64."""
    return float(np.asarray(token_logprobs[score_from:length], np.float64).sum())
