"""rlgen_sample_static (the sampling stage with its scratch in a static device array, for callers that cannot allocate)
against rlgen_debug_sample, the entry point it is a variant of: same kernels, so tokens and log-probs must be identical
bit for bit.  Two calls in a row, the second with fewer rows, so that what the first call left in the array would show."""
import numpy as np
import pytest
import torch

from gpu_util import GPU_SHAPES, R, dev_f32, dev_i32, make_policy, scaled_bf16_weights
from workloads import ModelShape

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["neox-h80", "llama-gqa4-h16", "vocab-50304"])
def test_static_scratch_sampling_equals_workspace_sampling(name):
    m = ModelShape(0, 1, 64, 4, 4, 16, 64, 50304, rotary_dim=4) if name == "vocab-50304" else GPU_SHAPES[name]
    W = scaled_bf16_weights(m, lm_head_scale=4.0)
    r = R()
    pol = make_policy(W, max_seqs=64, max_seq_len=40, max_batch_tokens=64)
    try:
        rng = np.random.default_rng(101)
        for rows in (64, 23, 1):
            hidden = dev_f32(rng.normal(size=(rows, m.d_model)))
            u = dev_f32(rng.random(rows, dtype=np.float32))
            forced = rng.integers(0, m.vocab, size=rows).astype(np.int32)
            forced[::2] = -1
            for f in (None, dev_i32(forced)):
                want_t, want_l = r.rlgen_debug_sample(pol, hidden, 0.7, u, f)
                # outputs pre-filled, so that a call that wrote nothing would be seen
                got = (torch.full((rows,), -7, dtype=torch.int32, device="cuda"), torch.full((rows,), 7.0, device="cuda"))
                r.rlgen_sample_static(pol, hidden, 0.7, u, f, out=got)
                torch.cuda.synchronize()
                assert torch.equal(got[0], want_t) and torch.equal(got[1], want_l), (rows, f is None)
                assert ((want_t >= 0) & (want_t < m.vocab)).all() and torch.isfinite(want_l).all()
        # a generate call between two static calls: the static call neither disturbs nor depends on the workspace buffers
        hidden = dev_f32(rng.normal(size=(8, m.d_model)))
        u = dev_f32(rng.random(8, dtype=np.float32))
        a = r.rlgen_sample_static(pol, hidden, 0.7, u)
        prompts = dev_i32(rng.integers(0, m.vocab, size=(3, 9)))
        gu = dev_f32(rng.random((3, 2, 5), dtype=np.float32))
        g1 = r.rlgen_generate(pol, prompts, [9, 4, 7], 2, 5, 0.7, gu)
        b = r.rlgen_sample_static(pol, hidden, 0.7, u)
        g2 = r.rlgen_generate(pol, prompts, [9, 4, 7], 2, 5, 0.7, gu)
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])
        assert torch.equal(g1[0], g2[0]) and torch.equal(g1[1], g2[1])
        # beyond the array's capacity: rejected, nothing written
        big = dev_f32(rng.normal(size=(65, m.d_model)))
        with pytest.raises(r.RlgenError) as e:
            r.rlgen_sample_static(pol, big, 0.7, dev_f32(rng.random(65, dtype=np.float32)))
        assert e.value.code == r.ERR_CAPACITY
        assert r.rlgen_status(pol) == 0
    finally:
        pol.close()
