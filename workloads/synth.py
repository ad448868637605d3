"""Seeded random inputs: weights, prompts, uniforms.

Every tensor has its own seed derived from (workload seed, layer, tensor index), so the
values do not depend on generation order and large models can be drawn on several
threads.  Matrices and linear biases are N(0, 0.02); norm gains are 1 + N(0, 0.02);
norm biases are N(0, 0.02).  For the bf16 workloads the fp32 draws are rounded to the
nearest bf16 (ties to even) and kept as uint16 bit patterns; `Weights.f32` expands them
exactly, so the CPU oracle and the GPU see the same numeric values.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from typing import Dict, List, Tuple

import numpy as np

from .configs import ARCH_LLAMA, ARCH_NEOX, ModelShape, Workload

GLOBAL_TENSORS = ("embed_in", "final_norm_g", "final_norm_b", "lm_head")
LAYER_TENSORS = ("norm1_g", "norm1_b", "norm2_g", "norm2_b", "wq", "wk", "wv", "bq", "bk", "bv",
                 "wo", "bo", "w_up", "b_up", "w_gate", "w_down", "b_down")


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16, ties to even; returns the 16-bit patterns (finite inputs only)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def tensor_shapes(m: ModelShape) -> Tuple[Dict[str, tuple], Dict[str, tuple]]:
    """Canonical tensor shapes; linear layers compute y = W x + b with W stored [out, in]."""
    d, F, V = m.d_model, m.d_ffn, m.vocab
    qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    neox = m.arch == ARCH_NEOX
    g = {"embed_in": (V, d), "final_norm_g": (d,), "lm_head": (V, d)}
    if neox:
        g["final_norm_b"] = (d,)
    l = {"norm1_g": (d,), "norm2_g": (d,), "wq": (qd, d), "wk": (kvd, d), "wv": (kvd, d),
         "wo": (d, qd), "w_up": (F, d), "w_down": (d, F)}
    if neox:
        l.update({"norm1_b": (d,), "norm2_b": (d,), "bq": (qd,), "bk": (kvd,), "bv": (kvd,),
                  "bo": (d,), "b_up": (F,), "b_down": (d,)})
    else:
        l["w_gate"] = (F, d)
    return g, l


class Weights:
    """Container of canonical tensors, held either as fp32 or as bf16 bit patterns (uint16)."""

    def __init__(self, model: ModelShape, tensors: Dict[str, np.ndarray], is_bf16: bool):
        self.model = model
        self.tensors = tensors
        self.is_bf16 = is_bf16
        self._f32_cache: Dict[str, np.ndarray] = {}
        self.cache_f32 = True

    def has(self, name: str) -> bool:
        return name in self.tensors

    def raw(self, name: str) -> np.ndarray:
        return self.tensors[name]

    def f32(self, name: str) -> np.ndarray:
        t = self.tensors[name]
        if t.dtype == np.float32:
            return t
        if name in self._f32_cache:
            return self._f32_cache[name]
        out = bf16_bits_to_f32(t)
        if self.cache_f32:
            self._f32_cache[name] = out
        return out

    def drop_f32_cache(self):
        self._f32_cache.clear()

    def replaced(self, **new_f32) -> "Weights":
        """A copy in which the named tensors are replaced by the given fp32 arrays (stored as
        fp32, or re-rounded to bf16 when this container holds bf16)."""
        t = dict(self.tensors)
        for k, v in new_f32.items():
            v = np.ascontiguousarray(v, dtype=np.float32)
            assert v.shape == self.tensors[k].shape, k
            t[k] = f32_to_bf16_bits(v) if self.is_bf16 else v
        return Weights(self.model, t, self.is_bf16)

    def rounded_to_bf16(self) -> "Weights":
        if self.is_bf16:
            return self
        return Weights(self.model, {k: f32_to_bf16_bits(v) for k, v in self.tensors.items()}, True)

    def names(self) -> List[str]:
        return list(self.tensors)


def _draw(seed: int, layer: int, idx: int, shape: tuple, mean: float, scale: float) -> np.ndarray:
    rng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, layer, idx])))
    x = rng.standard_normal(shape, dtype=np.float32)
    x *= np.float32(0.02 * scale)
    if mean:
        x += np.float32(mean)
    return x


def make_weights(model: ModelShape, seed: int, bf16: bool, lm_head_scale: float = 1.0,
                 threads: int = 8) -> Weights:
    gshapes, lshapes = tensor_shapes(model)
    jobs = []
    for name, shp in gshapes.items():
        jobs.append((name, 0, GLOBAL_TENSORS.index(name), shp))
    for li in range(model.n_layers):
        for name, shp in lshapes.items():
            jobs.append((f"layers.{li}.{name}", li + 1, LAYER_TENSORS.index(name), shp))

    def run(job):
        name, layer, idx, shp = job
        base = name.rsplit(".", 1)[-1]
        mean = 1.0 if base.endswith("_g") else 0.0
        scale = lm_head_scale if base == "lm_head" else 1.0
        x = _draw(seed, layer, idx, shp, mean, scale)
        return name, (f32_to_bf16_bits(x) if bf16 else x)

    if threads > 1 and model.n_params > 5_000_000:
        with ThreadPoolExecutor(threads) as ex:
            out = dict(ex.map(run, jobs))
    else:
        out = dict(map(run, jobs))
    return Weights(model, out, bf16)


def make_prompts(w: Workload, pad_id: int = -1) -> Tuple[np.ndarray, np.ndarray]:
    """Right-padded prompt array [B, stride] (int32) and lengths [B] (int32).  Pad cells hold
    `pad_id`, an out-of-range id: nothing may read them."""
    rng = np.random.Generator(np.random.PCG64(w.seed_prompts))
    lens = rng.integers(w.prompt_len_lo, w.prompt_len_hi, size=w.n_prompts, endpoint=True).astype(np.int32)
    stride = int(lens.max())
    toks = rng.integers(0, w.model.vocab, size=(w.n_prompts, stride)).astype(np.int32)
    toks[np.arange(stride)[None, :] >= lens[:, None]] = pad_id
    return toks, lens


def make_uniforms(w: Workload) -> np.ndarray:
    """Uniforms in [0, 1), fp32, shape [B, K, max_new]: the random numbers the sampler consumes."""
    rng = np.random.Generator(np.random.PCG64(w.seed_uniforms))
    return rng.random((w.n_prompts, w.k, w.max_new), dtype=np.float32)


def parity_subset(lens: np.ndarray, n_first: int = 2) -> List[int]:
    """Deterministic prompt subset used where the oracle cannot run a whole workload: the
    shortest prompt, the longest prompt and the first `n_first` by index (duplicates removed)."""
    idx = [int(np.argmin(lens)), int(np.argmax(lens))] + list(range(min(n_first, len(lens))))
    seen, out = set(), []
    for i in idx:
        if i not in seen:
            seen.add(i)
            out.append(i)
    return out
