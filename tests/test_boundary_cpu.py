"""Host-only checks of the C-ABI: the library loads, exports every symbol the header declares, and
rejects bad configurations before touching the device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
R = pytest.importorskip("paper_2410_18252_amd.rlgen", reason="librlgen.so not built")
from workloads import get_config, tiny_neox  # noqa: E402


def header_symbols():
    text = open(os.path.join(ROOT, "include", "rlgen.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rlgen_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    syms = header_symbols()
    assert "rlgen_generate" in syms and "rlgen_score" in syms and "rlgen_create" in syms
    for s in syms:
        assert hasattr(R.lib, s), s
    assert sorted(R.EXPORTS) == syms


def good_cfg(**kw):
    w = get_config(1)
    cfg = R.make_cfg(w.model, weight_dtype=R.DTYPE_F32, max_seqs=8, max_seq_len=48, max_kv_tokens=8 * 64)
    for k, v in kw.items():
        setattr(cfg, k, v)
    return cfg


def test_workspace_bytes_grows_with_capacity_and_rejects_bad_cfg():
    a = R.rlgen_workspace_bytes(good_cfg())
    b = R.rlgen_workspace_bytes(good_cfg(max_kv_tokens=16 * 64))
    assert 0 < a < b
    kv_bytes_per_token = get_config(1).model.kv_bytes_per_token
    assert b - a == 8 * 64 * kv_bytes_per_token
    assert R.lib.rlgen_workspace_bytes(None) == 0
    bad = [dict(arch=7), dict(d_model=130), dict(n_kv_heads=3), dict(rotary_dim=7), dict(rotary_dim=64),
           dict(head_dim=24), dict(norm_eps=0.0), dict(rope_theta=-1.0), dict(weight_dtype=5), dict(max_seqs=0),
           dict(max_kv_tokens=8), dict(max_batch_tokens=16), dict(vocab=1), dict(n_layers=0), dict(d_ffn=100)]
    for kw in bad:
        assert R.rlgen_workspace_bytes(good_cfg(**kw)) == 0, kw


def test_create_validates_before_touching_the_device():
    cfg = good_cfg()
    w = R.Weights()
    ctx = C.c_void_p()
    dummy = C.c_void_p(256)
    assert R.lib.rlgen_create(None, C.byref(w), dummy, 1 << 30, None, C.byref(ctx)) == R.ERR_NULL
    assert R.lib.rlgen_create(C.byref(cfg), None, dummy, 1 << 30, None, C.byref(ctx)) == R.ERR_NULL
    assert R.lib.rlgen_create(C.byref(cfg), C.byref(w), None, 1 << 30, None, C.byref(ctx)) == R.ERR_NULL
    assert R.lib.rlgen_create(C.byref(cfg), C.byref(w), dummy, 1 << 30, None, None) == R.ERR_NULL
    bad = good_cfg(rotary_dim=7)
    assert R.lib.rlgen_create(C.byref(bad), C.byref(w), dummy, 1 << 30, None, C.byref(ctx)) == R.ERR_BAD_CFG
    assert R.lib.rlgen_create(C.byref(cfg), C.byref(w), dummy, 1024, None, C.byref(ctx)) == R.ERR_WORKSPACE
    assert R.lib.rlgen_create(C.byref(cfg), C.byref(w), C.c_void_p(257), 1 << 30, None, C.byref(ctx)) == R.ERR_WORKSPACE
    assert not ctx.value


def test_null_context_and_strerror():
    assert R.lib.rlgen_generate(None, None, None, 1, 1, 1, 1, 0.7, None, None, None, None, None) == R.ERR_NULL
    assert R.lib.rlgen_score(None, None, None, None, 1, 1, 0.7, None, None) == R.ERR_NULL
    assert R.lib.rlgen_status(None, None) == R.ERR_NULL
    R.lib.rlgen_destroy(None)
    for code in range(-7, 1):
        assert R.rlgen_strerror(code) and "unknown" not in R.rlgen_strerror(code)
    assert "unknown" in R.rlgen_strerror(-99)


def test_all_five_configs_have_a_valid_cfg():
    for i in range(1, 6):
        w = get_config(i)
        cap = w.prompt_len_hi + w.max_new
        cfg = R.make_cfg(w.model, weight_dtype=R.DTYPE_BF16 if w.bf16_weights else R.DTYPE_F32,
                         max_seqs=w.n_prompts * w.k, max_seq_len=cap, max_kv_tokens=w.n_prompts * w.k * (cap + 31))
        assert R.rlgen_workspace_bytes(cfg) > w.model.n_params * 2, i
