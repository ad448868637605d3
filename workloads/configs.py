"""Model and workload shapes.

The paper trains Pythia 410M / 1B / 2.8B policies on TL;DR summarisation (batch 512,
prompts up to 512 tokens, response 128, temperature 0.7, two samples per prompt:
Section 3, Appendix A.1 hyper-parameter table) and a Llama-3.1-8B chatbot (prompt up to
512, response up to 1024, temperature 0.7: Appendix A.2).  The five workloads below
stand in for those by shape only: random weights, random token ids.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

ARCH_NEOX = 0   # LayerNorm with bias, parallel residual, GELU (erf form), biased linears
ARCH_LLAMA = 1  # RMSNorm, sequential residual, SwiGLU, no biases, grouped-query attention


@dataclass(frozen=True)
class ModelShape:
    arch: int
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rotary_dim: int
    rope_theta: float = 10000.0
    norm_eps: float = 1e-5

    def __post_init__(self):
        assert self.d_model == self.n_q_heads * self.head_dim
        assert self.n_q_heads % self.n_kv_heads == 0
        assert self.rotary_dim % 2 == 0 and self.rotary_dim <= self.head_dim

    @property
    def n_params(self) -> int:
        d, F, V = self.d_model, self.d_ffn, self.vocab
        kvd = self.n_kv_heads * self.head_dim
        per_layer = d * d + 2 * kvd * d + d * d + (3 if self.arch == ARCH_LLAMA else 2) * d * F
        return self.n_layers * per_layer + 2 * V * d

    @property
    def kv_bytes_per_token(self) -> int:
        return 2 * 2 * self.n_layers * self.n_kv_heads * self.head_dim


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelShape
    n_prompts: int
    prompt_len_lo: int
    prompt_len_hi: int
    k: int
    max_new: int
    temperature: float
    bf16_weights: bool
    seed_weights: int
    seed_prompts: int
    seed_uniforms: int
    lm_head_scale: float = 1.0   # > 1 gives a peaked next-token distribution

    def peaked(self, scale: float = 8.0) -> "Workload":
        return replace(self, name=self.name + "-peaked", lm_head_scale=scale)


def _neox(L, d, H, F, V) -> ModelShape:
    h = d // H
    return ModelShape(ARCH_NEOX, L, d, H, H, h, F, V, rotary_dim=h // 4)


CONFIGS = {
    1: Workload("c1-tiny-neox", _neox(2, 128, 4, 512, 1024), 4, 32, 32, 2, 16, 0.7,
                bf16_weights=False, seed_weights=1001, seed_prompts=2001, seed_uniforms=3001),
    2: Workload("c2-pythia410m-shaped", _neox(24, 1024, 16, 4096, 50304), 64, 128, 512, 2, 64, 0.7,
                bf16_weights=True, seed_weights=1002, seed_prompts=2002, seed_uniforms=3002),
    3: Workload("c3-pythia1b-shaped", _neox(16, 2048, 8, 8192, 50304), 256, 128, 512, 2, 64, 0.7,
                bf16_weights=True, seed_weights=1003, seed_prompts=2003, seed_uniforms=3003),
    4: Workload("c4-pythia2.8b-shaped", _neox(32, 2560, 32, 10240, 50304), 512, 256, 512, 2, 64, 0.7,
                bf16_weights=True, seed_weights=1004, seed_prompts=2004, seed_uniforms=3004),
    5: Workload("c5-llama3.1-8b-shaped",
                ModelShape(ARCH_LLAMA, 32, 4096, 32, 8, 128, 14336, 128256, rotary_dim=128,
                           rope_theta=500000.0),
                128, 256, 1024, 2, 512, 0.7,
                bf16_weights=True, seed_weights=1005, seed_prompts=2005, seed_uniforms=3005),
}


def get_config(i: int) -> Workload:
    return CONFIGS[int(i)]


def tiny_neox(**kw) -> ModelShape:
    """A few-thousand-parameter GPT-NeoX shape for brute-force tests (rotary on part of the head)."""
    base = dict(arch=ARCH_NEOX, n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=4, head_dim=8,
                d_ffn=64, vocab=48, rotary_dim=4)
    base.update(kw)
    return ModelShape(**base)


def tiny_llama(**kw) -> ModelShape:
    """A few-thousand-parameter Llama shape (grouped-query attention, rotary on the whole head)."""
    base = dict(arch=ARCH_LLAMA, n_layers=2, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8,
                d_ffn=48, vocab=40, rotary_dim=8, rope_theta=500000.0)
    base.update(kw)
    return ModelShape(**base)
