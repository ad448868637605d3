"""What the library's storage formats cost on the Llama-3.1-8B-shaped workload, computed from the oracle alone.

The benchmark spec's tolerances (raw logits 2e-2, token log-probs 1e-2) are met by the library's default formats (fp16
matrix-product inputs, bf16 KV cache) on the GPT-NeoX-shaped workloads, but not on the Llama-shaped one: with N(0, 0.02)
weights at d_model 4096 every block amplifies a perturbation of its input, so the 16-bit roundings grow with depth.
These tests apply the formats to the oracle's own functions (tests/rounding_model.py) on that model shape (full width,
reduced vocabulary, 1 / 4 / 8 of its 32 layers) and pin down

  * that the default formats already exceed the logit tolerance at 8 layers, and by how much each rounding point
    contributes (the bf16 keys and values dominate, but fp16 everywhere is still over at 8 layers);
  * that bf16 hi/lo pairs at every point -- the library's precise mode -- stay two orders of magnitude below it.

No GPU and no library code is involved: this is the evidence for offering the precise mode, reproducible on any host."""
import dataclasses

import numpy as np
import pytest

from oracle import decoder as O
from rounding_model import DEFAULT_FORMATS, POINTS, PRECISE_FORMATS, RoundedDecoder
from workloads import get_config, make_weights, Weights

TOL_LOGITS = 2e-2
DEPTHS = (1, 4, 8)


@pytest.fixture(scope="module")
def llama8b_slices():
    """The first 8 layers of workload 5's model shape with a 1024-token vocabulary, its shallower prefixes, a 40-token
    sequence, and the oracle's logits for each depth."""
    full = get_config(5).model
    m8 = dataclasses.replace(full, n_layers=max(DEPTHS), vocab=1024)
    W8 = make_weights(m8, 7, bf16=True, threads=8)
    seq = np.random.default_rng(1).integers(0, m8.vocab, size=40)
    out = {}
    for L in DEPTHS:
        m = dataclasses.replace(m8, n_layers=L)
        W = Weights(m, W8.tensors, True)            # layer l of every depth is the same seeded draw
        W.cache_f32 = False
        out[L] = (m, W, O.last_logits(O.Decoder(W, m), seq))
    return out, seq


def _err(case, seq, formats):
    m, W, ref = case
    return float(np.abs(O.last_logits(RoundedDecoder(W, m, formats), seq) - ref).max())


def test_default_formats_exceed_the_logit_tolerance_on_the_llama_8b_shape(llama8b_slices, capsys):
    cases, seq = llama8b_slices
    default = {L: _err(cases[L], seq, DEFAULT_FORMATS) for L in DEPTHS}
    all_f16 = {L: _err(cases[L], seq, {p: "f16" for p in POINTS}) for L in DEPTHS}
    with capsys.disabled():
        print("\nLlama-3.1-8B-shaped, vocabulary 1024, 40 tokens: max |logit error| of the rounded oracle (logit std "
              f"{cases[8][2].std():.2f})")
        for L in DEPTHS:
            print(f"  {L} layers: default formats {default[L]:.4f}   fp16 at every point {all_f16[L]:.4f}")
    assert 1.0 < cases[8][2].std() < 1.6                     # the logits are O(1): the tolerance means what it says
    assert default[1] < default[4] < default[8]              # the error grows with depth ...
    assert default[8] > TOL_LOGITS                           # ... and is over the bound at a quarter of the depth
    assert default[8] < 4 * default[1] * np.sqrt(8)          # (roughly like sqrt(layers), not faster)
    # even fp16 for keys, values and everything else has used up half the bound at 8 of the 32 layers
    assert all_f16[8] > TOL_LOGITS / 2
    assert all_f16[8] < default[8]


def test_attribution_of_the_error_to_the_rounding_points(llama8b_slices, capsys):
    """Each point alone, in the library's default format, at 4 layers: keys and values (bf16, 8 significant bits)
    outweigh every fp16 point; no single point is negligible next to the bound once there are 32 layers."""
    cases, seq = llama8b_slices
    alone = {p: _err(cases[4], seq, {p: DEFAULT_FORMATS[p]}) for p in POINTS}
    with capsys.disabled():
        print("\n  4 layers, one rounding point at a time: " + "  ".join(f"{p} {alone[p]:.4f}" for p in POINTS))
    fp16_points = [p for p in POINTS if DEFAULT_FORMATS[p] == "f16" and p != "p"]
    assert min(alone["k"], alone["v"]) > max(alone[p] for p in fp16_points)
    # every fp16 input of a matrix product alone costs more than a hundredth of the bound at 4 layers
    assert min(alone[p] for p in fp16_points) > TOL_LOGITS / 100
    # widening only the cache leaves the fp16 points' share
    kv_wide = dict(DEFAULT_FORMATS, k="bf16x2", v="bf16x2")
    assert _err(cases[4], seq, kv_wide) > 0.2 * _err(cases[4], seq, DEFAULT_FORMATS)


def test_bf16_pairs_at_every_point_stay_far_below_the_tolerance(llama8b_slices, capsys):
    cases, seq = llama8b_slices
    precise = {L: _err(cases[L], seq, PRECISE_FORMATS) for L in DEPTHS}
    with capsys.disabled():
        print("\n  bf16 hi/lo pairs at every point: " + "  ".join(f"{L} layers {precise[L]:.2e}" for L in DEPTHS))
    assert precise[8] < TOL_LOGITS / 50
    # extrapolated to the 32 layers like sqrt(depth), with a factor 4 to spare for the longer prompts and the full vocabulary
    assert 4 * precise[8] * np.sqrt(32 / 8) < TOL_LOGITS / 10
