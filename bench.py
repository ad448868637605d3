#!/usr/bin/env python3
"""Throughput of the generation hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-cpu-baseline]

One step = one rlgen_generate call over the whole synthetic batch of the chosen workload (default:
workload 4, the Pythia-2.8B-shaped one the headline target is quoted on): prompt pass, K-way fan-out
and all decode steps, inputs already resident in HBM.  Prints ONE JSON line with generated tokens/s,
the roofline of the dominant kernel (decode attention, HBM-bound; its launch time is measured with HIP
events on the launch stream inside the timed region) and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2500.0        # dense fp16 / bf16 matrix peak of MI355X
# HBM bytes per decode-attention launch over its algorithmic bytes on workload 4, measured with rocprofv3
# FETCH_SIZE + WRITE_SIZE, each scaled by its reading for a plain 1 GiB copy (profiles/attention_decode_c4_hbm_traffic.txt).
TRAFFIC_OVER_ALGORITHMIC = 1.039
# The same for every kernel of the decode phase together, two-stream decode (profiles/decode_phase_c4_hbm_traffic.txt):
# weights are read once per half batch, whole super-blocks are loaded, activations and partial sums pass through HBM.
DECODE_TRAFFIC_OVER_ALGORITHMIC = 1.192


# every EVENT_EVERY-th decode-attention launch of the timed region is bracketed with HIP events (each bracket costs
# about 10 us of idle GPU, so bracketing all 2016 launches of a pass would itself slow the pass by 0.6 %)
EVENT_EVERY = 4


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--max-new", type=int, default=0, help="override the workload's number of new tokens (profiling runs)")
    ap.add_argument("--no-kernel-events", action="store_true",
                    help="do not bracket the decode-attention launches with HIP events (for rocprofv3 --pmc runs)")
    ap.add_argument("--share-prompt-kv", action="store_true",
                    help="the k samples of a prompt read one copy of the prompt's keys/values (not the headline layout)")
    ap.add_argument("--max-batch-tokens", type=int, default=0, help="rows per prompt-pass chunk (0 = the library's default)")
    ap.add_argument("--no-alone-pass", action="store_true",
                    help="skip the extra pass that times the attention kernel with nothing beside it")
    ap.add_argument("--no-decode-split", action="store_true",
                    help="decode the whole batch on one stream (every kernel runs alone; slower)")
    ap.add_argument("--eos-mix", action="store_true",
                    help="completions end at an EOS token forced at a step drawn uniformly from [1, max_new] (seeded): ended "
                         "sequences leave the batch; tokens/s then counts the tokens up to and including each EOS")
    ap.add_argument("--no-score", action="store_true",
                    help="workload 4 ends with rlgen_score over the generated sequences; this leaves it out of the step")
    ap.add_argument("--score-plain", action="store_true",
                    help="score every generated sequence on its own instead of a prompt once with its k completions")
    ap.add_argument("--k", type=int, default=0, help="override the workload's samples per prompt")
    ap.add_argument("--precise", action="store_true",
                    help="the library's precise mode (bf16 hi/lo pairs instead of fp16 / bf16 values): what its accuracy costs")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1")

    import torch
    import paper_2410_18252_amd.rlgen as R
    from workloads import get_config, make_prompts, make_uniforms, make_weights, parity_subset

    w = get_config(args.config)
    if args.max_new:
        import dataclasses
        w = dataclasses.replace(w, max_new=args.max_new, name=f"{w.name}-maxnew{args.max_new}")
    if args.k:
        import dataclasses
        w = dataclasses.replace(w, k=args.k, name=f"{w.name}-k{args.k}")
    m = w.model
    share = 1 if args.share_prompt_kv else 0
    t0 = time.time()
    W = make_weights(m, w.seed_weights, w.bf16_weights, threads=16)
    arr, lens = make_prompts(w)
    u = make_uniforms(w)
    B, k, T = w.n_prompts, w.k, w.max_new
    S = B * k
    r32 = lambda n: (int(n) + 31) // 32 * 32
    kv_tokens = int(sum(r32(n) + k * r32(T) for n in lens)) if share else int(sum(k * r32(int(n) + T) for n in lens))
    cfg = R.make_cfg(m, weight_dtype=R.DTYPE_BF16 if W.is_bf16 else R.DTYPE_F32, max_seqs=S,
                     max_seq_len=int(lens.max()) + T, max_kv_tokens=kv_tokens, share_prompt_kv=share,
                     max_batch_tokens=args.max_batch_tokens, precise=1 if args.precise else 0)
    dev = R.upload_weights(W.tensors)
    pol = R.Policy(cfg, dev)
    del dev
    torch.cuda.empty_cache()
    setup_s = time.time() - t0

    d_arr = torch.from_numpy(arr).cuda()
    d_u = torch.from_numpy(u).cuda()
    out = (torch.empty((B, k, T), dtype=torch.int32, device="cuda"),
           torch.empty((B, k, T), dtype=torch.float32, device="cuda"))

    d_forced, real_tokens = None, S * T
    if args.eos_mix:
        eos = 0
        ends = np.random.default_rng(4000 + args.config).integers(1, T + 1, size=(B, k))     # completion lengths
        forced = np.full((B, k, T), -1, np.int32)
        np.put_along_axis(forced, (ends - 1)[..., None], eos, axis=2)
        d_forced = torch.from_numpy(forced).cuda()
        real_tokens = int(ends.sum())
        R.rlgen_set_eos(pol, eos)

    # Workload 4 is "generate, then rlgen_score on the resulting sequences": the sequences (prompt + completion) are
    # assembled on the device by one scatter of the generated tokens into a buffer that already holds the prompts.
    with_score = args.config == 4 and not args.no_score and not args.eos_mix
    if with_score:
        seq_lens = np.repeat(lens, k).astype(np.int32) + T
        stride = int(lens.max()) + T
        h_full = np.full((S, stride), -1, np.int32)
        for b in range(B):
            h_full[b * k:(b + 1) * k, :lens[b]] = arr[b, :lens[b]]
        d_full = torch.from_numpy(h_full).cuda()
        d_pos = (torch.from_numpy(np.repeat(lens, k).astype(np.int64)).cuda()[:, None] + torch.arange(T, device="cuda")[None, :])
        score_from = np.repeat(lens, k).astype(np.int32)
        d_score = torch.empty((S, stride), dtype=torch.float32, device="cuda")
        if not args.score_plain:
            # the sequences are a prompt with its k completions each: the library runs the prompt once per group
            R.rlgen_set_score_groups(pol, k)
    score_ms = []

    def step(timed=False):
        R.rlgen_generate(pol, d_arr, lens, k, T, w.temperature, d_u, d_forced, out)
        tm = R.rlgen_get_timings(pol) if timed else None          # waits for the generation's events only
        if with_score:
            d_full.scatter_(1, d_pos, out[0].view(S, T))
            R.rlgen_score(pol, d_full, seq_lens, w.temperature, score_from, d_score)
            if timed:
                score_ms.append(R.rlgen_get_timings(pol)["prefill_ms"])
        return tm

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.no_decode_split:
        R.rlgen_set_decode_split(pol, False)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    R.rlgen_set_profiling(pol, 0 if args.no_kernel_events else EVENT_EVERY)
    prefill_ms, decode_ms, attn_ms, attn_launches = [], [], 0.0, 0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        tm = step(timed=True)
        prefill_ms.append(tm["prefill_ms"]); decode_ms.append(tm["decode_ms"])
        attn_ms += tm["decode_attn_ms"]; attn_launches += tm["decode_attn_launches"]
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    R.rlgen_set_profiling(pol, 0)
    assert R.rlgen_status(pol) == 0
    toks = out[0].cpu().numpy()
    assert ((toks >= 0) & (toks < m.vocab)).all()

    ms_per_step = 1e3 * elapsed / args.steps
    tokens_per_s = real_tokens / (elapsed / args.steps)

    # ---- roofline of the dominant kernel: decode attention.  Algorithmic bytes of one launch (one layer, one
    # decode step t): every sequence reads its K and V streams of ctx = prompt_len + t keys (bf16), plus q in
    # and the attention output out (fp16).
    seq_len = np.repeat(lens.astype(np.int64), k)
    per_key = 2 * 2 * m.n_kv_heads * m.head_dim * (2 if args.precise else 1)      # K and V, 2 bytes each (precise: two planes)
    qo = 2 * 2 * S * m.n_q_heads * m.head_dim
    # with a shared prompt cache a launch reads each prompt's keys once, and t new keys per sequence
    keys = (lambda t: int(lens.astype(np.int64).sum()) + S * t) if share else (lambda t: int((seq_len + t).sum()))
    if args.eos_mix:        # a sequence whose completion ended before step t is skipped by the attention launch of step t
        live = lambda t: (ends.reshape(-1) > t)
        if share:
            keys = lambda t: int((lens.astype(np.int64) * (ends > t).any(axis=1)).sum()) + int(live(t).sum()) * t
        else:
            keys = lambda t: int(((seq_len + t) * live(t)).sum())
    bytes_per_launch = np.mean([per_key * keys(t) + qo for t in range(1, T)]) if T > 1 else 0.0
    # A batch of >= 256 sequences decodes as two halves on two streams: every layer and step then has two attention
    # launches, each over half of the bytes, running beside the other half's linear layers.
    halves = max(1, round(attn_launches * EVENT_EVERY / max(1, args.steps * m.n_layers * (T - 1)))) if not args.eos_mix else 1
    bytes_per_launch /= halves

    def roofline_of(ms, launches, extra):
        us = 1e3 * ms / max(launches, 1)
        achieved = bytes_per_launch / (us * 1e-6) / 1e9 if launches else 0.0
        return {"bound": "hbm", "kernel": "attention_kernel<HD,decode>", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": int(round(TRAFFIC_OVER_ALGORITHMIC * bytes_per_launch)) if args.config == 4 and not share and not args.k else None,
                "algorithmic_bytes_per_launch": int(bytes_per_launch), "avg_launch_us": round(us, 2), "launches": launches, **extra}

    roofline = roofline_of(attn_ms, attn_launches, {
        "launches_per_layer_and_step": halves,
        "concurrency": "timed region: each launch shares the GPU with the other half's GEMMs" if halves > 1 else "none"})

    # whole decode phase: weights once per step + KV, over the measured decode time
    wbytes = 2 * (m.n_params - m.vocab * m.d_model)                # all matrices but the embedding table
    decode_bytes = sum(wbytes + m.n_layers * (per_key * keys(t) + per_key * S) for t in range(1, T))
    decode_gbs = decode_bytes / (np.mean(decode_ms) * 1e-3) / 1e9 if T > 1 else 0.0

    # ---- matrix-core roofline of the prompt pass and of the score pass: algorithmic flops over the measured time.
    # Linear layers: 2 flops per weight and row (every matrix of every block; the LM head only for the rows it serves);
    # attention: QK^T and PV over the causal triangle, 4 h flops per (query, visible key) and query head.
    body = m.n_params - 2 * m.vocab * m.d_model                     # weights of all blocks
    lm = m.vocab * m.d_model
    tri = lambda n: n * (n + 1) // 2
    L64 = lens.astype(np.int64)
    prefill_flops = 2.0 * float(L64.sum()) * body + 2.0 * S * lm \
        + 4.0 * m.head_dim * m.n_q_heads * m.n_layers * float(sum(tri(int(n)) for n in L64))

    def mfma_roofline(flops, ms, what):
        tf = flops / (ms * 1e-3) / 1e12 if ms else 0.0
        return {"bound": "mfma", "pass": what, "achieved": round(tf, 1), "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": round(tf / MFMA_F16_PEAK_TFLOPS, 4), "flops": float(flops), "ms": round(ms, 2)}

    result = {
        "metric": "generated tokens/s (K=2/prompt) at 1 GPU; decode HBM GB/s as % of peak",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 2), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16x2" if args.precise else "f16", "data": "synthetic",
        "config": {"workload": w.name, "prompts": B, "k": k, "max_new": T, "prompt_len": [w.prompt_len_lo, w.prompt_len_hi],
                   "temperature": w.temperature, "generated_tokens_per_step": real_tokens,
                   "step": ("rlgen_generate, then rlgen_score over the generated sequences"
                            + ("" if args.score_plain else f" (groups of {k} sharing their prompt)")) if with_score else "rlgen_generate",
                   "kv_layout": "prompt cache shared by the k samples" if share else "one contiguous cache per sequence",
                   "storage": ("bf16 weights; activations and KV cache as bf16 hi/lo pairs (precise mode), bf16 MFMA, fp32 accumulation"
                               if args.precise else
                               "bf16 weights (held as fp16, exact) and bf16 KV cache; fp16 MFMA inputs, fp32 accumulation"),
                   # tile-shape variant and K split per linear layer (QKV, O, FFN up, FFN down, LM head) as the context chose them
                   "gemm_choices": {name: [list(R.rlgen_debug_get_gemm(pol, mode, which)) for which in range(5)]
                                    for mode, name in ((0, "decode"), (1, "prompt_pass"), (2, "decode_half"))}},
        "prefill_ms": round(float(np.mean(prefill_ms)), 2), "decode_ms": round(float(np.mean(decode_ms)), 2),
        "score_ms": round(float(np.mean(score_ms)), 2) if score_ms else None,
        "generate_only_tokens_per_s": round(real_tokens / (1e-3 * float(np.mean(prefill_ms) + np.mean(decode_ms))), 1),
        "decode_algorithmic_GBps": round(decode_gbs, 1), "decode_frac_of_hbm_peak": round(decode_gbs / HBM_PEAK_GBS, 4),
        # HBM bytes actually moved over the decode time, from the counter-measured ratio above (headline layout only)
        "decode_hbm_GBps": round(decode_gbs * DECODE_TRAFFIC_OVER_ALGORITHMIC, 1)
        if args.config == 4 and halves > 1 and not share and not args.k and not args.eos_mix else None,
        "setup_s": round(setup_s, 1),
        "roofline": roofline,
        "roofline_prefill": mfma_roofline(prefill_flops, float(np.mean(prefill_ms)),
                                          "prompt pass of rlgen_generate (all layers, K-way cache fan-out, first LM head)"),
    }
    if roofline["traffic"] is not None:
        roofline["traffic_source"] = ("algorithmic bytes x 1.039, the ratio rocprofv3 FETCH_SIZE + WRITE_SIZE gave for this kernel "
                                      "on this workload (profiles/attention_decode_c4_hbm_traffic.txt); not re-measured in this run")
    if score_ms:
        # rows the score pass sends through the blocks: with grouping a prompt once and each completion's tail; else every sequence
        if args.score_plain:
            rows, att = float((L64 + T).sum() * k), float(sum(tri(int(n) + T) for n in L64) * k)
        else:
            rows = float(L64.sum() + S * T)
            att = float(sum(tri(int(n)) + k * (T * int(n) + tri(T)) for n in L64))
        score_flops = 2.0 * rows * body + 2.0 * S * T * lm + 4.0 * m.head_dim * m.n_q_heads * m.n_layers * att
        result["roofline_score"] = mfma_roofline(score_flops, float(np.mean(score_ms)),
                                                 "rlgen_score over the generated sequences (LM head on the response positions)")
    if halves > 1 and not args.no_kernel_events and not args.no_alone_pass:
        # the same kernel with nothing beside it: one more pass (not part of `value`) with the two-stream decode
        # switched off, so that a launch covers the whole batch and runs alone
        R.rlgen_set_decode_split(pol, False)
        R.rlgen_set_profiling(pol, EVENT_EVERY)
        R.rlgen_generate(pol, d_arr, lens, k, T, w.temperature, d_u, d_forced, out)
        tm = R.rlgen_get_timings(pol)
        R.rlgen_set_profiling(pol, 0)
        R.rlgen_set_decode_split(pol, True)
        bytes_per_launch *= halves
        result["roofline_kernel_alone"] = roofline_of(tm["decode_attn_ms"], tm["decode_attn_launches"], {
            "decode_ms": round(tm["decode_ms"], 2), "concurrency": "extra pass, whole batch per launch, single stream"})

    if not args.no_cpu_baseline:
        from oracle import decoder as O
        subset = parity_subset(lens, n_first=2) if args.config != 5 else parity_subset(lens, n_first=0)[:1]
        n_new = min(8, T)
        dec = O.Decoder(W, m)
        t0 = time.perf_counter()
        for b in subset:
            O.generate(dec, arr[b, :lens[b]], k, n_new, w.temperature, u[b][:, :n_new])
        cpu_s = time.perf_counter() - t0
        result["cpu_baseline"] = {
            "value": round(len(subset) * k * n_new / cpu_s, 3), "unit": "tokens/s", "cores": len(os.sched_getaffinity(0)),
            "kind": "oracle", "seconds": round(cpu_s, 1),
            "sample": f"prompts {subset} of the same workload (lengths {[int(lens[b]) for b in subset]}), "
                      f"K={k}, first {n_new} new tokens each, full-size weights; numpy fp32 (BLAS threads = cores)"}
    pol.close()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
