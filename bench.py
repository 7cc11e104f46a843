#!/usr/bin/env python3
"""Headline benchmark: generated tokens/s of speculative decoding at batch 1 on
the T5-XXL-shaped pair (gamma = 3 / 5 / 7), the verify forward's HBM rate, and
the speedup over the same build's plain target-model decoding.

One "step" is one run of Algorithm 1: gamma draft steps of Mq, one (gamma+1)-row
Mp forward, the accept / resample kernel and the roll-back.  Weights, encoder
outputs and KV caches are resident in HBM before the timed region; a sequence
generates 128 tokens and is then restarted (the restart, i.e. reset + prefill,
is outside the timed region).  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
GEN_LEN = 128                   # tokens generated per sequence (T5-XXL-shaped workload)
TEMPERATURE = 1.0
# HBM bytes of one FFN-in launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE counters, scaled by what
# the same counters read for a 256 MiB copy (profiles/ffn_in_hbm_traffic.txt has the run); None = not measured
TRAFFIC_FFN_IN = 168567808   # bytes: (82248.5 KiB fetched x 2.0 + 120 KiB written)


def expected_tokens(alpha, gamma):
    return float(gamma + 1) if alpha >= 1.0 else (1.0 - alpha ** (gamma + 1)) / (1.0 - alpha)


def timed_steps(dec, gamma, n_steps, temperature, urows, enc_p, enc_q, torch):
    """Run exactly n_steps runs of Algorithm 1; time only the sd_step calls."""
    total_s, tokens, accepted, tested, it = 0.0, 0, 0, 0, 0
    while it < n_steps:
        dec.reset()
        dec.prefill([0], enc_p, enc_q)
        torch.cuda.synchronize()
        gen = 0
        t0 = time.perf_counter()
        while it < n_steps and gen < GEN_LEN:
            n, toks = dec.step(gamma, temperature, urows[it % len(urows)])
            gen += n + 1
            accepted += n
            tested += min(n + 1, gamma)
            it += 1
        torch.cuda.synchronize()
        total_s += time.perf_counter() - t0
        tokens += gen
    return total_s, tokens, accepted, tested


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=120)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--gammas", type=str, default="3,5,7")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a 256 MiB device-to-device copy (reference for the profiler's byte counters)")
    ap.add_argument("--ctx", type=int, default=2048, help="gqa8b-batch16: tokens of context per sequence")
    ap.add_argument("--workload", type=str, default="t5xxl", choices=["t5xxl", "gqa8b-batch16"],
                    help="t5xxl: the headline configuration (default); gqa8b-batch16: the batched 8B-class "
                         "configuration (16 sequences, 2048-token contexts, gamma 4), a side measurement")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; --gpus must be 1 (nothing here uses a second GPU)")
    if args.workload == "gqa8b-batch16":
        return batched_gqa8b(args, ctx=args.ctx)

    import numpy as np
    import torch
    from paper_2211_17192_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    gammas = [int(g) for g in args.gammas.split(",")]
    cfg_p, w_p, cfg_q, w_q, enc_p, enc_q = synth.t5xxl_pair("cuda", gen_len=GEN_LEN)
    bytes_p, bytes_q = synth.model_bytes(cfg_p), synth.model_bytes(cfg_q)
    want_cpu = not args.no_cpu_baseline
    dec = binding.SpecDecoder(cfg_p, w_p, cfg_q, w_q, max_gamma=max(gammas), flags=binding.SD_FLAG_GRAPH)
    if not want_cpu:                                # the library holds its own re-tiled copy
        del w_p, w_q
        torch.cuda.empty_cache()

    per_gamma = {}

    def sweep(gamma):
        urows = synth.uniform_stream(100 + gamma, 512 * (2 * gamma + 1)).reshape(512, -1)
        timed_steps(dec, gamma, args.warmup, TEMPERATURE, urows, enc_p, enc_q, torch)
        secs, tokens, accepted, tested = timed_steps(dec, gamma, args.steps, TEMPERATURE, urows, enc_p, enc_q, torch)
        alpha = accepted / max(tested, 1)
        per_gamma[gamma] = {"tokens_per_s": tokens / secs, "ms_per_step": 1e3 * secs / args.steps,
                            "tokens_per_step": tokens / args.steps, "alpha": alpha,
                            "eq1_tokens_per_step": expected_tokens(alpha, gamma)}

    for gamma in gammas:
        sweep(gamma)
    # section 3.5: let the library choose gamma from what it has measured (alpha from the acceptance
    # tests of the last sequence, c from graph replays of one Mq step and one Mp step); if that
    # gamma is not among the requested ones it is timed like them
    tuned = dec.autotune_gamma(reps=10)
    if tuned["gamma"] not in gammas:
        gammas = gammas + [tuned["gamma"]]
        sweep(tuned["gamma"])

    # argmax sampling (temperature 0): the same launches, another acceptance rate (section 2.2:
    # acceptance then means "Mq's argmax is Mp's argmax")
    per_gamma_t0 = {}
    for gamma in gammas:
        urows = synth.uniform_stream(300 + gamma, 512 * (2 * gamma + 1)).reshape(512, -1)
        n_t0 = max(8, args.steps // 2)
        timed_steps(dec, gamma, min(args.warmup, 4), 0.0, urows, enc_p, enc_q, torch)
        secs, tokens, accepted, tested = timed_steps(dec, gamma, n_t0, 0.0, urows, enc_p, enc_q, torch)
        per_gamma_t0[gamma] = {"tokens_per_s": tokens / secs, "ms_per_step": 1e3 * secs / n_t0,
                               "tokens_per_step": tokens / n_t0, "alpha": accepted / max(tested, 1)}

    # plain Mp decoding: the denominator of the speedup.  One whole untimed sequence first: right
    # after the speculative runs the first ~100 plain steps are ~10 % slower than the steady state
    # (the chip's power management follows the change of load), which would flatter the speedup.
    ub = synth.uniform_stream(7, GEN_LEN)
    dec.reset(); dec.prefill([0], enc_p, enc_q)
    for i in range(GEN_LEN - 1):
        dec.step_baseline(TEMPERATURE, ub[i])
    dec.reset(); dec.prefill([0], enc_p, enc_q)
    for i in range(args.warmup):
        dec.step_baseline(TEMPERATURE, ub[i])
    torch.cuda.synchronize()
    n_base = min(args.steps, GEN_LEN - args.warmup)
    t0 = time.perf_counter()
    for i in range(n_base):
        dec.step_baseline(TEMPERATURE, ub[args.warmup + i])
    torch.cuda.synchronize()
    base_ms = 1e3 * (time.perf_counter() - t0) / n_base

    # phase and kernel timing with HIP events on the library's stream (eager launches)
    dec.set_flags(binding.SD_FLAG_PROFILE)
    prof = {}
    for gamma in gammas:
        dec.reset(); dec.prefill([0], enc_p, enc_q)
        urows = synth.uniform_stream(200 + gamma, 64 * (2 * gamma + 1)).reshape(64, -1)
        d = v = a = 0.0
        k_ms, k_n, n_it = 0.0, 0, 0
        for i in range(20):
            dec.step(gamma, TEMPERATURE, urows[i])
            st = dec.stats()
            if i >= 4:
                d += st["draft_ms"]; v += st["verify_ms"]; a += st["accept_ms"]; n_it += 1
        st = dec.stats()
        k_ms, k_n = st["ffn_in_ms_sum"], st["ffn_in_launches"]
        kv_bytes = bytes_p["kv_per_pos"] * (GEN_LEN // 2)           # mid-sequence self-attention cache
        b_verify = bytes_p["weights"] + bytes_p["cross_kv"] + kv_bytes + (gamma + 1) * cfg_p["vocab"] * 4
        prof[gamma] = {"draft_ms": d / n_it, "verify_ms": v / n_it, "accept_ms": a / n_it,
                       "verify_bytes": b_verify, "verify_GBps": b_verify / (v / n_it) / 1e6,
                       "c": (d / n_it / gamma) / base_ms, "ffn_in_us": 1e3 * k_ms / max(k_n, 1)}
    dec.set_flags(binding.SD_FLAG_GRAPH)

    best = max(gammas, key=lambda g: per_gamma[g]["tokens_per_s"])
    res = per_gamma[best]
    for g in gammas:
        pg, pr = per_gamma[g], prof[g]
        pg.update({"speedup_vs_plain": pg["tokens_per_s"] / (1e3 / base_ms),
                   "thm38_predicted_speedup": expected_tokens(pg["alpha"], g) / (g * pr["c"] + 1.0),
                   "draft_ms": pr["draft_ms"], "verify_ms": pr["verify_ms"], "accept_ms": pr["accept_ms"],
                   "c": pr["c"], "verify_GBps": pr["verify_GBps"],
                   "verify_frac_of_hbm_peak": pr["verify_GBps"] / HBM_PEAK_GBPS})

    # Roofline of the dominant kernel: the gated FFN-in GEMM streams both d_ff x d_model matrices
    # of a layer exactly once (algorithmic bytes per launch = 2 * d_ff * d_model * 2).  Its mean
    # launch duration: all 24 layers' launches, back to back from one graph, between two HIP events
    # on the library's stream (every launch reads another layer's weights, so nothing is cached).
    ffn_bytes = 2 * cfg_p["d_ff"] * cfg_p["d_model"] * 2
    ffn_us = dec.time_ffn_in(best + 1, reps=20)
    roofline = {"bound": "hbm", "kernel": "gemm_kernel<bf16, PRO_POST, EPI_GATED> (Mp FFN-in, gated GELU)",
                "achieved": ffn_bytes / ffn_us / 1e3, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": ffn_bytes / ffn_us / 1e3 / HBM_PEAK_GBPS, "bytes_per_launch": ffn_bytes,
                "us_per_launch": ffn_us, "us_per_launch_between_events_in_step": prof[best]["ffn_in_us"],
                "rows": best + 1, "traffic": TRAFFIC_FFN_IN}
    if args.calibrate:          # a plain copy of known size, for scaling the rocprofv3 byte counters
        src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    cpu = None
    if want_cpu:
        # the oracle's copy of the very same tensors, made only now: the conversion of 11 GB of
        # weights leaves the host busy enough to slow the timed loops above by about 10 %
        host_w = (synth.to_numpy_weights(w_p), synth.to_numpy_weights(w_q),
                  synth.to_numpy_weights({"p": enc_p, "q": enc_q}))
        del w_p, w_q
        cpu = cpu_baseline(cfg_p, cfg_q, host_w, synth)

    out = {
        "metric": "generated tokens/s at batch 1 (T5-XXL-shaped, gamma=3/5/7); verify-step HBM GB/s",
        "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "T5-XXL-shaped encoder-decoder pair (configs[3]): Mp 24L d4096 64x64 ff10240 "
                               "gated-GELU V32128 + 512-token cross-attention, Mq 6L d512 8x64 ff2048; batch 1, "
                               "temperature 1, 128 generated tokens per sequence",
                   "gamma": best, "temperature": TEMPERATURE, "gammas": gammas},
        "per_gamma": {str(g): per_gamma[g] for g in gammas},
        "per_gamma_temperature0": {str(g): per_gamma_t0[g] for g in gammas},
        "autotune": {"gamma": tuned["gamma"], "alpha": tuned["alpha"], "c": tuned["c"],
                     "thm38_predicted_speedup": tuned["improvement"],
                     "measured_speedup": per_gamma[tuned["gamma"]]["tokens_per_s"] / (1e3 / base_ms)},
        "plain_decode_tokens_per_s": 1e3 / base_ms, "plain_decode_ms_per_token": base_ms,
        "plain_decode_GBps": (bytes_p["weights"] + bytes_p["cross_kv"]) / base_ms / 1e6,
        "verify_GBps": res["verify_GBps"], "verify_frac_of_hbm_peak": res["verify_frac_of_hbm_peak"],
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    dec.close()


def batched_gqa8b(args, batch=16, ctx=2048):
    """Side measurement: the batched 8B-class pair (32-layer GQA target, 2-layer draft, bf16), every
    sequence with a ctx-token context written by a real prefill; Algorithm-1 iterations (gamma = 3 and
    4 unless --gammas says otherwise) against
    plain decoding steps of the same batch.  One JSON line; `value` is the best gamma's rate.  No CPU
    leg (the oracle needs minutes per row here)."""
    import torch
    from paper_2211_17192_amd import binding, synth
    gammas = [3, 4] if args.gammas == "3,5,7" else [int(g) for g in args.gammas.split(",")]
    cfg_p, w_p, cfg_q, w_q = synth.gqa8b_pair("cuda")
    dec = binding.SpecDecoder(cfg_p, w_p, cfg_q, w_q, max_gamma=max(gammas), flags=binding.SD_FLAG_GRAPH, batch=batch)
    del w_p, w_q
    torch.cuda.empty_cache()
    steps, warm = min(args.steps, 40), min(args.warmup, 4)
    prompts = [synth.random_tokens(300 + b, ctx, cfg_p["vocab"]) for b in range(batch)]
    per_gamma = {}
    for gamma in gammas:
        dec.reset()
        for b in range(batch):
            dec.prefill(prompts[b], row=b)
            print(f"gamma {gamma}: prefilled {b + 1} of {batch} sequences", file=sys.stderr, flush=True)
        U = synth.uniform_stream(9, (steps + warm) * batch * (2 * gamma + 1)).reshape(steps + warm, batch, -1)
        for i in range(warm):
            dec.step(gamma, TEMPERATURE, U[i])
        st0 = dec.stats()
        torch.cuda.synchronize()
        t0, tokens = time.perf_counter(), 0
        for i in range(steps):
            tokens += sum(n + 1 for n, _ in dec.step(gamma, TEMPERATURE, U[warm + i]))
        torch.cuda.synchronize()
        secs = time.perf_counter() - t0
        st = dec.stats()
        per_gamma[gamma] = {"tokens_per_s": tokens / secs, "ms_per_step": 1e3 * secs / steps, "tokens_per_step": tokens / steps,
                            "alpha": (st["accepted"] - st0["accepted"]) / max(st["tested"] - st0["tested"], 1)}
    ub = synth.uniform_stream(7, (steps + 2) * batch).reshape(steps + 2, batch)
    for i in range(2):
        dec.step_baseline(TEMPERATURE, ub[i])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        dec.step_baseline(TEMPERATURE, ub[2 + i])
    torch.cuda.synchronize()
    plain = time.perf_counter() - t0
    dec.close()
    best = max(per_gamma, key=lambda g: per_gamma[g]["tokens_per_s"])
    r = per_gamma[best]
    print(json.dumps({
        "metric": "tokens_per_s", "value": r["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warm,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "gqa8b-batch16: 8B-class GQA target + 2-layer draft, 16 sequences, "
                               f"{ctx}-token contexts, gamma {best}, temperature {TEMPERATURE}"},
        "tokens_per_step": r["tokens_per_step"], "alpha": r["alpha"], "per_gamma": per_gamma,
        "plain_decode_tokens_per_s": batch * steps / plain, "plain_decode_ms_per_step": 1e3 * plain / steps,
        "speedup_over_plain": r["tokens_per_s"] / (batch * steps / plain)}))


def cpu_baseline(cfg_p, cfg_q, host_w, synth):
    """The NumPy oracle, as it stands, on the host cores: one run of Algorithm 1
    (gamma = 3) on the same T5-XXL-shaped pair; tokens produced / wall time."""
    import numpy as np
    from oracle import decode, transformer as T
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    wp, wq, enc = host_w
    mp = T.Transformer(T.ModelConfig(**cfg_p), wp)
    mq = T.Transformer(T.ModelConfig(**cfg_q), wq)
    t0 = time.perf_counter()
    mp.set_encoder_output(enc["p"]); mq.set_encoder_output(enc["q"])
    t_enc = time.perf_counter() - t0
    gamma = 3
    u = synth.uniform_stream(5, 2 * gamma + 1)
    t0 = time.perf_counter()
    out, n, _ = decode.speculative_decoding_step(T.CachedScorer(mp), T.CachedScorer(mq), [0], gamma, TEMPERATURE, u)
    secs = time.perf_counter() - t0
    return {"value": (n + 1) / secs, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"one run of Algorithm 1 at gamma=3 on the full T5-XXL-shaped pair (float64 NumPy, "
                      f"{n + 1} tokens in {secs:.1f} s; cross-attention K/V set-up {t_enc:.1f} s not counted)",
            "host_cpus": os.cpu_count()}


if __name__ == "__main__":
    main()
