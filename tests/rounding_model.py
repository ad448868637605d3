"""The oracle with the library's rounding points switched on, one by one or together (test infrastructure).

The HIP library evaluates the same decoder as `oracle.decoder` but rounds at fixed points: the inputs of every
matrix product (the normalised rows, the attention output, the activated FFN rows, the final-norm rows), the
rotated queries, the keys and values it stores in its cache, and the softmax probabilities that multiply the
values.  `RoundedDecoder` is `oracle.decoder.Decoder` with a rounding function applied at each of those points,
so that the error the library's formats must produce on a given model can be computed on the CPU, without the
library, and attributed to single points.  Nothing here is used by the product.

Formats: "f16" (IEEE half, 11 significant bits), "bf16" (8 bits), "bf16x2" (a value held as the sum of two
bf16 numbers, hi = bf16(x), lo = bf16(x - hi): 16 significant bits with bf16's exponent range), None (exact).
"""
import numpy as np

from oracle import decoder as O
from workloads.synth import bf16_bits_to_f32, f32_to_bf16_bits


def _f16(a):
    return np.asarray(a, np.float32).astype(np.float16).astype(np.float32)


def _bf16(a):
    return bf16_bits_to_f32(f32_to_bf16_bits(np.asarray(a, np.float32)))


def _bf16x2(a):
    a = np.asarray(a, np.float32)
    hi = _bf16(a)
    return hi + _bf16(a - hi)


ROUNDERS = {None: lambda a: a, "f16": _f16, "bf16": _bf16, "bf16x2": _bf16x2}

# rounding points, in the order a block meets them
POINTS = ("n1", "q", "k", "v", "p", "attn", "n2", "act", "hfin")
# the library's default formats, and those of its precise mode (cfg.precise = 1)
DEFAULT_FORMATS = {"n1": "f16", "q": "f16", "k": "bf16", "v": "bf16", "p": "f16", "attn": "f16", "n2": "f16",
                   "act": "f16", "hfin": "f16"}
PRECISE_FORMATS = {p: "bf16x2" for p in POINTS}


class RoundedDecoder(O.Decoder):
    """formats: dict point -> format name; points left out stay exact."""

    def __init__(self, W, m, formats, dt=np.float32):
        super().__init__(W, m, dt)
        self.fmt = {p: ROUNDERS[formats.get(p)] for p in POINTS}

    def _attend(self, q, k, v, qpos):
        # oracle.decoder.attention with the probabilities rounded before they multiply the values; the library
        # rounds exp(s - max) (it normalises afterwards, by the unrounded sum)
        m, dt = self.m, self.dt
        n, Hq, h = q.shape
        group = Hq // k.shape[1]
        visible = np.arange(k.shape[0])[None, :] <= np.asarray(qpos)[:, None]
        out = np.empty((n, Hq, h), dtype=dt)
        for j in range(Hq):
            kj, vj = k[:, j // group, :], v[:, j // group, :]
            s = (q[:, j, :] @ kj.T).astype(np.float64) / np.sqrt(h)
            s = np.where(visible, s, -np.inf)
            e = np.exp(s - s.max(axis=1, keepdims=True))
            out[:, j, :] = (self.fmt["p"](e.astype(dt)) @ vj) / e.sum(axis=1, keepdims=True).astype(dt)
        return out

    def _self_attention(self, layer, a, pos, cache, biased):
        m, dt, f = self.m, self.dt, self.fmt
        n = a.shape[0]
        q = O.linear(a, self.lw(layer, "wq"), self.lw(layer, "bq") if biased else None)
        k = O.linear(a, self.lw(layer, "wk"), self.lw(layer, "bk") if biased else None)
        v = O.linear(a, self.lw(layer, "wv"), self.lw(layer, "bv") if biased else None)
        q = f["q"](O.rotary(q.reshape(n, m.n_q_heads, m.head_dim), pos, m.rotary_dim, m.rope_theta, dt))
        k = f["k"](O.rotary(k.reshape(n, m.n_kv_heads, m.head_dim), pos, m.rotary_dim, m.rope_theta, dt))
        v = f["v"](v.reshape(n, m.n_kv_heads, m.head_dim).astype(dt))
        cache.append(layer, k, v)
        o = f["attn"](self._attend(q, cache.k[layer], cache.v[layer], pos))
        return O.linear(o.reshape(n, m.n_q_heads * m.head_dim), self.lw(layer, "wo"), self.lw(layer, "bo") if biased else None)

    def _block(self, layer, x, pos, cache):
        m, dt, f = self.m, self.dt, self.fmt
        if m.arch == O.ARCH_NEOX:
            a = f["n1"](O.layer_norm(x, self.lw(layer, "norm1_g"), self.lw(layer, "norm1_b"), m.norm_eps, dt))
            mm = f["n2"](O.layer_norm(x, self.lw(layer, "norm2_g"), self.lw(layer, "norm2_b"), m.norm_eps, dt))
            attn = self._self_attention(layer, a, pos, cache, True)
            up = f["act"](O.gelu(O.linear(mm, self.lw(layer, "w_up"), self.lw(layer, "b_up")), dt))
            return (x + attn + O.linear(up, self.lw(layer, "w_down"), self.lw(layer, "b_down"))).astype(dt)
        a = f["n1"](O.rms_norm(x, self.lw(layer, "norm1_g"), m.norm_eps, dt))
        x = (x + self._self_attention(layer, a, pos, cache, False)).astype(dt)
        mm = f["n2"](O.rms_norm(x, self.lw(layer, "norm2_g"), m.norm_eps, dt))
        act = f["act"](O.silu(O.linear(mm, self.lw(layer, "w_gate")), dt) * O.linear(mm, self.lw(layer, "w_up")))
        return (x + O.linear(act.astype(dt), self.lw(layer, "w_down"))).astype(dt)

    def logits(self, x):
        m, dt = self.m, self.dt
        if m.arch == O.ARCH_NEOX:
            h = O.layer_norm(x, self.w("final_norm_g"), self.w("final_norm_b"), m.norm_eps, dt)
        else:
            h = O.rms_norm(x, self.w("final_norm_g"), m.norm_eps, dt)
        return self.fmt["hfin"](h) @ self.w("lm_head").T


def logit_error(W, m, seq, formats):
    """max |logits(rounded) - logits(oracle)| at the last position of `seq`, and the oracle's logit std."""
    ref = O.last_logits(O.Decoder(W, m), seq)
    got = O.last_logits(RoundedDecoder(W, m, formats), seq)
    return float(np.abs(got - ref).max()), float(ref.std())
