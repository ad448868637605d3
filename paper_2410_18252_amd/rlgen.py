"""ctypes binding of librlgen.so: argument marshalling only.

Function names mirror include/rlgen.h.  Device buffers are torch tensors (torch is used for device
memory and streams, nothing else); every step of generation and scoring runs in the library's
kernels.  There is no fallback: if the shared library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "librlgen.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2410_18252_amd.build`")
lib = C.CDLL(LIB_PATH)

OK = 0
ERR_NULL, ERR_BAD_CFG, ERR_BAD_ARG, ERR_CAPACITY, ERR_WORKSPACE, ERR_UNIMPLEMENTED, ERR_DEVICE = -1, -2, -3, -4, -5, -6, -7
ARCH_NEOX, ARCH_LLAMA = 0, 1
DTYPE_F32, DTYPE_BF16 = 0, 1

EXPORTS = ["rlgen_workspace_bytes", "rlgen_create", "rlgen_update_weights", "rlgen_generate", "rlgen_score",
           "rlgen_debug_logits", "rlgen_debug_sample", "rlgen_sample_static", "rlgen_sequence_logprob", "rlgen_dpo_loss", "rlgen_select_pairs", "rlgen_proximal_rloo",
           "rlgen_get_timings", "rlgen_set_profiling", "rlgen_set_decode_split", "rlgen_set_decode_split_min", "rlgen_set_eos",
           "rlgen_set_eos_compaction", "rlgen_set_score_groups", "rlgen_debug_get_gemm", "rlgen_debug_set_gemm", "rlgen_status",
           "rlgen_status_bits", "rlgen_strerror", "rlgen_destroy"]
FAULT_TOKEN, FAULT_UNIFORM, FAULT_GROUP, FAULT_RANGE = 1, 2, 4, 8


class ModelCfg(C.Structure):
    _fields_ = [("arch", C.c_int32), ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rotary_dim", C.c_int32), ("rope_theta", C.c_float), ("norm_eps", C.c_float),
                ("weight_dtype", C.c_int32), ("max_seqs", C.c_int32), ("max_seq_len", C.c_int32),
                ("max_kv_tokens", C.c_int64), ("max_batch_tokens", C.c_int32), ("share_prompt_kv", C.c_int32),
                ("precise", C.c_int32)]


LAYER_FIELDS = ["norm1_g", "norm1_b", "norm2_g", "norm2_b", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "bo",
                "w_up", "b_up", "w_gate", "w_down", "b_down"]


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_FIELDS]


class Weights(C.Structure):
    _fields_ = [("embed_in", C.c_void_p), ("final_norm_g", C.c_void_p), ("final_norm_b", C.c_void_p),
                ("lm_head", C.c_void_p), ("layers", C.POINTER(LayerWeights))]


_vp, _i32, _f32 = C.c_void_p, C.c_int32, C.c_float
lib.rlgen_workspace_bytes.restype = C.c_size_t
lib.rlgen_workspace_bytes.argtypes = [C.POINTER(ModelCfg)]
lib.rlgen_create.restype = C.c_int
lib.rlgen_create.argtypes = [C.POINTER(ModelCfg), C.POINTER(Weights), _vp, C.c_size_t, _vp, C.POINTER(_vp)]
lib.rlgen_update_weights.restype = C.c_int
lib.rlgen_update_weights.argtypes = [_vp, C.POINTER(Weights), _vp]
lib.rlgen_generate.restype = C.c_int
lib.rlgen_generate.argtypes = [_vp, _vp, C.POINTER(_i32), _i32, _i32, _i32, _i32, _f32, _vp, _vp, _vp, _vp, _vp]
lib.rlgen_score.restype = C.c_int
lib.rlgen_score.argtypes = [_vp, _vp, C.POINTER(_i32), C.POINTER(_i32), _i32, _i32, _f32, _vp, _vp]
lib.rlgen_debug_logits.restype = C.c_int
lib.rlgen_debug_logits.argtypes = [_vp, _vp, C.POINTER(_i32), _i32, _i32, _vp, _vp]
lib.rlgen_debug_sample.restype = C.c_int
lib.rlgen_debug_sample.argtypes = [_vp, _vp, _i32, _f32, _vp, _vp, _vp, _vp, _vp]
lib.rlgen_sample_static.restype = C.c_int
lib.rlgen_sample_static.argtypes = [_vp, _vp, _i32, _f32, _vp, _vp, _vp, _vp, _vp]
lib.rlgen_sequence_logprob.restype = C.c_int
lib.rlgen_sequence_logprob.argtypes = [_vp, _vp, _vp, _i32, _i32, _vp, _vp]
lib.rlgen_select_pairs.restype = C.c_int
lib.rlgen_select_pairs.argtypes = [_vp, _i32, _i32, _vp, _vp, _vp]
lib.rlgen_proximal_rloo.restype = C.c_int
lib.rlgen_proximal_rloo.argtypes = [_vp, _vp, _vp, _i32, _i32, _f32, _vp, _vp]
lib.rlgen_dpo_loss.restype = C.c_int
lib.rlgen_dpo_loss.argtypes = [_vp, _vp, _vp, _vp, _i32, _f32, _vp, _vp]
lib.rlgen_get_timings.restype = C.c_int
lib.rlgen_get_timings.argtypes = [_vp, C.POINTER(_f32), C.POINTER(_f32), C.POINTER(_f32), C.POINTER(_i32)]
lib.rlgen_set_score_groups.restype = C.c_int
lib.rlgen_set_score_groups.argtypes = [_vp, _i32]
lib.rlgen_set_eos.restype = C.c_int
lib.rlgen_set_eos.argtypes = [_vp, _i32]
lib.rlgen_set_decode_split.restype = C.c_int
lib.rlgen_set_decode_split.argtypes = [_vp, _i32]
lib.rlgen_set_profiling.restype = C.c_int
lib.rlgen_set_profiling.argtypes = [_vp, _i32]
lib.rlgen_status.restype = C.c_int
lib.rlgen_status.argtypes = [_vp, _vp]
lib.rlgen_status_bits.restype = C.c_int
lib.rlgen_status_bits.argtypes = [_vp, _vp, C.POINTER(C.c_uint32)]
lib.rlgen_set_eos_compaction.restype = C.c_int
lib.rlgen_set_eos_compaction.argtypes = [_vp, _i32]
lib.rlgen_set_decode_split_min.restype = C.c_int
lib.rlgen_set_decode_split_min.argtypes = [_vp, _i32]
lib.rlgen_debug_get_gemm.restype = C.c_int
lib.rlgen_debug_get_gemm.argtypes = [_vp, _i32, _i32, C.POINTER(_i32), C.POINTER(_i32)]
lib.rlgen_debug_set_gemm.restype = C.c_int
lib.rlgen_debug_set_gemm.argtypes = [_vp, _i32, _i32, _i32]
lib.rlgen_strerror.restype = C.c_char_p
lib.rlgen_strerror.argtypes = [C.c_int]
lib.rlgen_destroy.restype = None
lib.rlgen_destroy.argtypes = [_vp]


class RlgenError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {rlgen_strerror(code)} ({code})")


def rlgen_strerror(code: int) -> str:
    return lib.rlgen_strerror(int(code)).decode()


def _check(code: int, where: str):
    if code != OK:
        raise RlgenError(code, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _host_i32(a):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.int32))
    return a, a.ctypes.data_as(C.POINTER(_i32))


def make_cfg(model, *, weight_dtype: int, max_seqs: int, max_seq_len: int, max_kv_tokens: int,
             max_batch_tokens: int = 0, share_prompt_kv: int = 0, precise: int = 0) -> ModelCfg:
    """ModelCfg from any object with the model-shape fields (arch, n_layers, d_model, ...)."""
    return ModelCfg(model.arch, model.n_layers, model.d_model, model.n_q_heads, model.n_kv_heads, model.head_dim,
                    model.d_ffn, model.vocab, model.rotary_dim, model.rope_theta, model.norm_eps, weight_dtype,
                    max_seqs, max_seq_len, max_kv_tokens, max_batch_tokens, share_prompt_kv, precise)


def rlgen_workspace_bytes(cfg: ModelCfg) -> int:
    return int(lib.rlgen_workspace_bytes(C.byref(cfg)))


def upload_weights(tensors: Dict[str, np.ndarray], device="cuda") -> Dict[str, torch.Tensor]:
    """Copies canonical tensors to the device: float32 arrays as fp32, uint16 arrays as bf16 bit patterns."""
    out = {}
    for k, v in tensors.items():
        if v.dtype == np.uint16:
            out[k] = torch.from_numpy(v.view(np.int16)).to(device).view(torch.bfloat16)
        else:
            out[k] = torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(device)
    return out


def _weights_struct(cfg: ModelCfg, dev: Dict[str, torch.Tensor]):
    want = torch.bfloat16 if cfg.weight_dtype == DTYPE_BF16 else torch.float32
    for k, t in dev.items():
        if t.dtype != want or not t.is_contiguous() or not t.is_cuda:
            raise ValueError(f"tensor {k}: expected contiguous device {want}")
    layers = (LayerWeights * cfg.n_layers)()
    for l in range(cfg.n_layers):
        for f in LAYER_FIELDS:
            t = dev.get(f"layers.{l}.{f}")
            setattr(layers[l], f, None if t is None else t.data_ptr())
    w = Weights(dev["embed_in"].data_ptr(), dev["final_norm_g"].data_ptr(),
                dev["final_norm_b"].data_ptr() if "final_norm_b" in dev else None, dev["lm_head"].data_ptr(), layers)
    return w, layers


class Policy:
    """Owns a context and the workspace tensor behind it."""

    def __init__(self, cfg: ModelCfg, dev_weights: Dict[str, torch.Tensor]):
        need = rlgen_workspace_bytes(cfg)
        if need == 0:
            raise RlgenError(ERR_BAD_CFG, "rlgen_workspace_bytes")
        self.cfg = cfg
        self.workspace = torch.empty(need, dtype=torch.uint8, device="cuda")
        w, keep = _weights_struct(cfg, dev_weights)
        ctx = C.c_void_p()
        _check(lib.rlgen_create(C.byref(cfg), C.byref(w), _ptr(self.workspace), need, _stream(), C.byref(ctx)),
               "rlgen_create")
        self.ctx = ctx
        torch.cuda.current_stream().synchronize()   # the library no longer reads dev_weights after this

    def close(self):
        if getattr(self, "ctx", None):
            lib.rlgen_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def update_weights(self, dev_weights):
        w, keep = _weights_struct(self.cfg, dev_weights)
        _check(lib.rlgen_update_weights(self.ctx, C.byref(w), _stream()), "rlgen_update_weights")
        torch.cuda.current_stream().synchronize()


def rlgen_update_weights(p: Policy, dev_weights: Dict[str, torch.Tensor]):
    p.update_weights(dev_weights)


def rlgen_generate(p: Policy, prompts: torch.Tensor, prompt_lens, k: int, max_new: int, temperature: float,
                   uniforms: torch.Tensor, forced: Optional[torch.Tensor] = None, out=None):
    """prompts int32 [B, stride] (device), prompt_lens host ints [B], uniforms fp32 [B, k, max_new] (device).
    Returns (tokens int32 [B, k, max_new], token_logprobs fp32 [B, k, max_new]) on the device; asynchronous."""
    B, stride = prompts.shape
    assert prompts.dtype == torch.int32 and prompts.is_contiguous() and prompts.is_cuda
    assert uniforms.dtype == torch.float32 and uniforms.is_contiguous() and tuple(uniforms.shape) == (B, k, max_new)
    if forced is not None:
        assert forced.dtype == torch.int32 and forced.is_contiguous() and tuple(forced.shape) == (B, k, max_new)
    lens, lens_p = _host_i32(prompt_lens)
    assert lens.shape == (B,)
    if out is None:
        tokens = torch.empty((B, k, max_new), dtype=torch.int32, device=prompts.device)
        lps = torch.empty((B, k, max_new), dtype=torch.float32, device=prompts.device)
    else:
        tokens, lps = out
    _check(lib.rlgen_generate(p.ctx, _ptr(prompts), lens_p, B, stride, k, max_new, temperature, _ptr(uniforms),
                              _ptr(forced), _ptr(tokens), _ptr(lps), _stream()), "rlgen_generate")
    return tokens, lps


def rlgen_score(p: Policy, seqs: torch.Tensor, seq_lens, temperature: float, score_from=None, out=None):
    N, stride = seqs.shape
    assert seqs.dtype == torch.int32 and seqs.is_contiguous() and seqs.is_cuda
    lens, lens_p = _host_i32(seq_lens)
    assert lens.shape == (N,)
    sf, sf_p = (None, None) if score_from is None else _host_i32(score_from)
    lps = torch.empty((N, stride), dtype=torch.float32, device=seqs.device) if out is None else out
    _check(lib.rlgen_score(p.ctx, _ptr(seqs), lens_p, sf_p, N, stride, temperature, _ptr(lps), _stream()), "rlgen_score")
    return lps


def rlgen_debug_logits(p: Policy, seqs: torch.Tensor, seq_lens):
    N, stride = seqs.shape
    assert seqs.dtype == torch.int32 and seqs.is_contiguous() and seqs.is_cuda
    lens, lens_p = _host_i32(seq_lens)
    logits = torch.empty((N, p.cfg.vocab), dtype=torch.float32, device=seqs.device)
    _check(lib.rlgen_debug_logits(p.ctx, _ptr(seqs), lens_p, N, stride, _ptr(logits), _stream()), "rlgen_debug_logits")
    return logits


def rlgen_debug_sample(p: Policy, hidden: torch.Tensor, temperature: float, uniforms: torch.Tensor,
                       forced: Optional[torch.Tensor] = None):
    R, d = hidden.shape
    assert hidden.dtype == torch.float32 and hidden.is_contiguous() and d == p.cfg.d_model
    assert uniforms.dtype == torch.float32 and tuple(uniforms.shape) == (R,)
    tokens = torch.empty(R, dtype=torch.int32, device=hidden.device)
    lps = torch.empty(R, dtype=torch.float32, device=hidden.device)
    _check(lib.rlgen_debug_sample(p.ctx, _ptr(hidden), R, temperature, _ptr(uniforms), _ptr(forced), _ptr(tokens),
                                  _ptr(lps), _stream()), "rlgen_debug_sample")
    return tokens, lps


def rlgen_sample_static(p: Policy, hidden: torch.Tensor, temperature: float, uniforms: torch.Tensor,
                        forced: Optional[torch.Tensor] = None, out=None):
    """rlgen_debug_sample with the library's static scratch; `out` = (tokens, token_logprobs) to write into."""
    R, d = hidden.shape
    assert hidden.dtype == torch.float32 and hidden.is_contiguous() and d == p.cfg.d_model
    assert uniforms.dtype == torch.float32 and tuple(uniforms.shape) == (R,)
    tokens, lps = out if out is not None else (torch.empty(R, dtype=torch.int32, device=hidden.device),
                                               torch.empty(R, dtype=torch.float32, device=hidden.device))
    _check(lib.rlgen_sample_static(p.ctx, _ptr(hidden), R, temperature, _ptr(uniforms), _ptr(forced), _ptr(tokens),
                                   _ptr(lps), _stream()), "rlgen_sample_static")
    return tokens, lps


def rlgen_sequence_logprob(token_logprobs: torch.Tensor, start: torch.Tensor, lens: torch.Tensor):
    N, stride = token_logprobs.shape
    assert token_logprobs.dtype == torch.float32 and token_logprobs.is_contiguous()
    assert start.dtype == torch.int32 and lens.dtype == torch.int32
    out = torch.empty(N, dtype=torch.float32, device=token_logprobs.device)
    _check(lib.rlgen_sequence_logprob(_ptr(token_logprobs), _ptr(start), _ptr(lens), N, stride, _ptr(out), _stream()),
           "rlgen_sequence_logprob")
    return out


def rlgen_dpo_loss(pol_pos, ref_pos, pol_neg, ref_neg, beta: float):
    P = pol_pos.numel()
    for t in (pol_pos, ref_pos, pol_neg, ref_neg):
        assert t.dtype == torch.float32 and t.is_contiguous() and t.numel() == P
    out = torch.empty(P, dtype=torch.float32, device=pol_pos.device)
    _check(lib.rlgen_dpo_loss(_ptr(pol_pos), _ptr(ref_pos), _ptr(pol_neg), _ptr(ref_neg), P, beta, _ptr(out), _stream()),
           "rlgen_dpo_loss")
    return out


def rlgen_proximal_rloo(pol_logprob, old_logprob, rewards, epsilon: float):
    """[B, k] fp32 sequence log-probs under pi_theta and pi_old and rewards -> [B, k] clipped objective."""
    assert rewards.dim() == 2
    B, k = rewards.shape
    for t in (pol_logprob, old_logprob, rewards):
        assert t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == (B, k)
    out = torch.empty(B, k, dtype=torch.float32, device=rewards.device)
    _check(lib.rlgen_proximal_rloo(_ptr(pol_logprob), _ptr(old_logprob), _ptr(rewards), B, k, epsilon, _ptr(out), _stream()),
           "rlgen_proximal_rloo")
    return out


def rlgen_select_pairs(rewards):
    """rewards [B, k] fp32 on the device -> (idx_pos, idx_neg), each [B] int32."""
    assert rewards.dtype == torch.float32 and rewards.is_contiguous() and rewards.dim() == 2
    B, k = rewards.shape
    pos = torch.empty(B, dtype=torch.int32, device=rewards.device)
    neg = torch.empty(B, dtype=torch.int32, device=rewards.device)
    _check(lib.rlgen_select_pairs(_ptr(rewards), B, k, _ptr(pos), _ptr(neg), _stream()), "rlgen_select_pairs")
    return pos, neg


def rlgen_get_timings(p: Policy):
    a, b, c, n = _f32(), _f32(), _f32(), _i32()
    _check(lib.rlgen_get_timings(p.ctx, C.byref(a), C.byref(b), C.byref(c), C.byref(n)), "rlgen_get_timings")
    return {"prefill_ms": a.value, "decode_ms": b.value, "decode_attn_ms": c.value, "decode_attn_launches": n.value}


def rlgen_set_score_groups(p: Policy, k: int):
    _check(lib.rlgen_set_score_groups(p.ctx, int(k)), "rlgen_set_score_groups")


def rlgen_set_eos(p: Policy, eos_token: int):
    _check(lib.rlgen_set_eos(p.ctx, int(eos_token)), "rlgen_set_eos")


def rlgen_set_decode_split(p: Policy, on: bool):
    _check(lib.rlgen_set_decode_split(p.ctx, 1 if on else 0), "rlgen_set_decode_split")


def rlgen_set_profiling(p: Policy, every: int):
    """every >= 1: bracket every `every`-th decode-attention launch with events; 0 / False: off."""
    _check(lib.rlgen_set_profiling(p.ctx, int(every)), "rlgen_set_profiling")


def rlgen_status(p: Policy) -> int:
    return int(lib.rlgen_status(p.ctx, _stream()))


def rlgen_status_bits(p: Policy) -> int:
    """The sticky fault bits (FAULT_*); synchronises the current stream."""
    bits = C.c_uint32()
    lib.rlgen_status_bits(p.ctx, _stream(), C.byref(bits))
    return int(bits.value)


def rlgen_set_eos_compaction(p: Policy, every: int):
    _check(lib.rlgen_set_eos_compaction(p.ctx, int(every)), "rlgen_set_eos_compaction")


def rlgen_set_decode_split_min(p: Policy, min_seqs: int):
    _check(lib.rlgen_set_decode_split_min(p.ctx, int(min_seqs)), "rlgen_set_decode_split_min")


def rlgen_debug_get_gemm(p: Policy, mode: int, which: int):
    """(tile-shape variant, K split) of linear layer `which` in `mode`."""
    v, sp = _i32(), _i32()
    _check(lib.rlgen_debug_get_gemm(p.ctx, mode, which, C.byref(v), C.byref(sp)), "rlgen_debug_get_gemm")
    return v.value, sp.value


def rlgen_debug_set_gemm(p: Policy, mode: int, which: int, variant: int):
    _check(lib.rlgen_debug_set_gemm(p.ctx, mode, which, int(variant)), "rlgen_debug_set_gemm")
