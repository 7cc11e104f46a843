#!/usr/bin/env python3
"""Headline benchmark: generated tokens/s of speculative decoding at batch 1 on
the T5-XXL-shaped pair (gamma = 3 / 5 / 7), the verify forward's HBM rate, and
the speedup over the same build's plain target-model decoding.

One "step" is one run of Algorithm 1: gamma draft steps of Mq, one (gamma+1)-row
Mp forward, the accept / resample kernel and the roll-back.  Weights, encoder
outputs and KV caches are resident in HBM before the timed region; a sequence
generates 128 tokens and is then restarted (the restart, i.e. reset + prefill,
is outside the timed region).  Prints ONE JSON line.

How the line is put together (so that it does not depend on the luck of a short run):
  * ms_per_step        exactly --steps timed runs of Algorithm 1 (it does not depend on what is accepted);
  * alpha, tokens/step pooled over those runs AND over five more whole 128-token sequences per gamma
                       (several hundred counted acceptance tests), each of which is timed by itself too
                       (median and minimum tokens/s over sequences are reported);
  * value              tokens/step (pooled) / ms_per_step of the gamma that Eq. 1 at the pooled alpha,
                       divided by ms_per_step, ranks first; the tokens/s of the --steps runs alone is
                       reported beside it as tokens_per_s_measured.

Side workloads (--workload): `sampler` (the isolated accept / resample kernel, 64 rows x gamma 7 x
vocabulary 32128), `gpt97m` (the GPT-like 97M / 6M pair, launch-latency regime), `gqa8b-batch16`.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
GEN_LEN = 128                   # tokens generated per sequence (T5-XXL-shaped workload)
TEMPERATURE = 1.0
EXTRA_SEQUENCES = 5             # whole sequences per gamma beyond the --steps runs
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "ffn_in_gemm_t5xxl_hbm_traffic.txt")


def traffic_from_profile():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary
    (FETCH_SIZE / WRITE_SIZE scaled by a copy of known size); None if the file does not say."""
    try:
        m = re.search(r"traffic per launch = \d+ KiB = (\d+) B", open(TRAFFIC_PROFILE).read())
        return int(m.group(1)) if m else None
    except OSError:
        return None


def expected_tokens(alpha, gamma):
    return float(gamma + 1) if alpha >= 1.0 else (1.0 - alpha ** (gamma + 1)) / (1.0 - alpha)


class Tally:
    def __init__(self):
        self.secs, self.tokens, self.accepted, self.tested, self.steps = 0.0, 0, 0, 0, 0

    def add(self, other):
        for k in ("secs", "tokens", "accepted", "tested", "steps"):
            setattr(self, k, getattr(self, k) + getattr(other, k))


def run_sequences(dec, gamma, temperature, urows, restart, torch, n_steps=None, n_sequences=None, gen_len=GEN_LEN):
    """Runs of Algorithm 1 in sequences of gen_len tokens; only the sd_step calls are timed.
    Either exactly n_steps runs (sequences restarted as needed) or n_sequences whole sequences.
    Returns (Tally, per-sequence tokens/s of the whole sequences)."""
    total, per_seq, it = Tally(), [], 0
    while (n_steps is not None and total.steps < n_steps) or (n_sequences is not None and len(per_seq) < n_sequences):
        restart()
        torch.cuda.synchronize()
        t = Tally()
        t0 = time.perf_counter()
        while t.tokens < gen_len and (n_steps is None or total.steps + t.steps < n_steps):
            n, _ = dec.step(gamma, temperature, urows[it % len(urows)])
            t.tokens += n + 1
            t.accepted += n
            t.tested += min(n + 1, gamma)
            t.steps += 1
            it += 1
        torch.cuda.synchronize()
        t.secs = time.perf_counter() - t0
        total.add(t)
        if t.tokens >= gen_len:
            per_seq.append(t.tokens / t.secs)
    return total, per_seq


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=120)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--gammas", type=str, default="3,5,7")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate", action="store_true",
                    help="also run a 256 MiB device-to-device copy (reference for the profiler's byte counters)")
    ap.add_argument("--counters-pass", action="store_true",
                    help="t5xxl: load the pair, run --warmup + --steps iterations at the first of --gammas (and the "
                         "copy of --calibrate), print a short line and stop: the pass `rocprofv3 --pmc` wraps, which "
                         "serialises every dispatch and would take many minutes over the whole benchmark")
    ap.add_argument("--ctx", type=int, default=2048, help="gqa8b-batch16: tokens of context per sequence")
    ap.add_argument("--workload", type=str, default="t5xxl", choices=["t5xxl", "gqa8b-batch16", "sampler", "gpt97m"],
                    help="t5xxl: the headline configuration (default); sampler: the isolated accept / resample "
                         "kernel (64 rows, gamma 7, vocabulary 32128); gpt97m: the GPT-like 97M / 6M pair; "
                         "gqa8b-batch16: the batched 8B-class configuration (16 sequences, 2048-token contexts)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU; --gpus must be 1 (nothing here uses a second GPU)")
    if args.workload == "gqa8b-batch16":
        return batched_gqa8b(args, ctx=args.ctx)
    if args.workload == "sampler":
        return sampler_workload(args)
    if args.workload == "gpt97m":
        return gpt97m_workload(args)

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

    def restart():
        dec.reset()
        dec.prefill([0], enc_p, enc_q)

    if args.counters_pass:
        gamma = gammas[0]
        urows = synth.uniform_stream(100 + gamma, 1024 * (2 * gamma + 1)).reshape(1024, -1)
        restart()
        tokens = 0
        for i in range(args.warmup + args.steps):
            n, _ = dec.step(gamma, TEMPERATURE, urows[i])
            tokens += n + 1
            if i % 4 == 0:
                print(f"counters pass: iteration {i}", file=sys.stderr, flush=True)
        if args.calibrate:
            src = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
            dst = torch.empty_like(src)
            for _ in range(4):
                dst.copy_(src)
            torch.cuda.synchronize()
        print(json.dumps({"counters_pass": True, "gamma": gamma, "iterations": args.warmup + args.steps, "tokens": tokens}))
        return

    per_gamma = {}

    def sweep(gamma):
        urows = synth.uniform_stream(100 + gamma, 1024 * (2 * gamma + 1)).reshape(1024, -1)
        run_sequences(dec, gamma, TEMPERATURE, urows, restart, torch, n_steps=args.warmup)
        timed, _ = run_sequences(dec, gamma, TEMPERATURE, urows, restart, torch, n_steps=args.steps)
        extra, per_seq = run_sequences(dec, gamma, TEMPERATURE, urows[256:], restart, torch, n_sequences=EXTRA_SEQUENCES)
        pool = Tally(); pool.add(timed); pool.add(extra)
        alpha = pool.accepted / max(pool.tested, 1)
        ms = 1e3 * timed.secs / args.steps
        per_gamma[gamma] = {
            "tokens_per_s": (pool.tokens / pool.steps) / ms * 1e3, "ms_per_step": ms,
            "tokens_per_s_measured": timed.tokens / timed.secs, "tokens_per_step_measured": timed.tokens / args.steps,
            "tokens_per_step": pool.tokens / pool.steps, "alpha": alpha, "alpha_tests": pool.tested,
            "eq1_tokens_per_step": expected_tokens(alpha, gamma),
            "eq1_tokens_per_s": expected_tokens(alpha, gamma) / ms * 1e3,
            "sequences": {"n": len(per_seq), "tokens": GEN_LEN, "tokens_per_s_median": statistics.median(per_seq),
                          "tokens_per_s_min": min(per_seq), "tokens_per_s_max": max(per_seq),
                          "ms_per_step": 1e3 * extra.secs / extra.steps}}

    for gamma in gammas:
        sweep(gamma)
    # section 3.5: let the library choose gamma from what it has measured (alpha from all acceptance
    # tests so far, c from graph replays of one Mq step and one Mp step); if that gamma is not among
    # the requested ones it is timed like them
    tuned = dec.autotune_gamma(reps=10)
    if tuned["gamma"] not in gammas:
        gammas = gammas + [tuned["gamma"]]
        sweep(tuned["gamma"])

    # argmax sampling (temperature 0): the same launches, another acceptance rate (section 2.2:
    # acceptance then means "Mq's argmax is Mp's argmax")
    per_gamma_t0 = {}
    for gamma in gammas:
        urows = synth.uniform_stream(300 + gamma, 512 * (2 * gamma + 1)).reshape(512, -1)
        run_sequences(dec, gamma, 0.0, urows, restart, torch, n_steps=min(args.warmup, 4))
        t, per_seq = run_sequences(dec, gamma, 0.0, urows, restart, torch, n_sequences=2)
        per_gamma_t0[gamma] = {"tokens_per_s": t.tokens / t.secs, "ms_per_step": 1e3 * t.secs / t.steps,
                               "tokens_per_step": t.tokens / t.steps, "alpha": t.accepted / max(t.tested, 1),
                               "alpha_tests": t.tested}

    # plain Mp decoding: the denominator of the speedup.  One whole untimed sequence first: right
    # after the speculative runs the first ~100 plain steps are ~10 % slower than the steady state
    # (the chip's power management follows the change of load), which would flatter the speedup.
    ub = synth.uniform_stream(7, GEN_LEN)
    restart()
    for i in range(GEN_LEN - 1):
        dec.step_baseline(TEMPERATURE, ub[i])
    plain_runs = []
    for rep in range(3):
        restart()
        for i in range(args.warmup):
            dec.step_baseline(TEMPERATURE, ub[i])
        torch.cuda.synchronize()
        n_base = GEN_LEN - args.warmup - 1
        t0 = time.perf_counter()
        for i in range(n_base):
            dec.step_baseline(TEMPERATURE, ub[args.warmup + i])
        torch.cuda.synchronize()
        plain_runs.append(1e3 * (time.perf_counter() - t0) / n_base)
    base_ms = statistics.median(plain_runs)

    # Inside the graph: the cost coefficient c (Definition 3.7) from graph replays of one Mq step and
    # one Mp step; the whole verify forward and the share of each kind of launch in it, mid-sequence
    # (about 64 committed tokens), as differences of graph replays with that launch left out.
    def mid_sequence(gamma):
        restart()
        urows = synth.uniform_stream(200 + gamma, 64 * (2 * gamma + 1)).reshape(64, -1)
        got, i = 1, 0
        while got < GEN_LEN // 2:
            n, _ = dec.step(gamma, TEMPERATURE, urows[i]); got += n + 1; i += 1
        return got

    graph = {}
    for gamma in gammas:
        ctx_len = mid_sequence(gamma)
        mq_us, mp_us = dec.measure_cost(reps=20)
        verify_us = dec.time_forward(0, gamma + 1, 0, reps=20)
        kv_bytes = bytes_p["kv_per_pos"] * ctx_len
        b_verify = bytes_p["weights"] + bytes_p["cross_kv"] + kv_bytes + (gamma + 1) * cfg_p["vocab"] * 4
        graph[gamma] = {"c": mq_us / mp_us, "draft_step_us": mq_us, "plain_step_us": mp_us, "verify_us": verify_us,
                        "verify_bytes": b_verify, "verify_GBps": b_verify / verify_us / 1e3, "context": ctx_len}

    best = max(gammas, key=lambda g: per_gamma[g]["eq1_tokens_per_s"])
    d, ff, V, L = cfg_p["d_model"], cfg_p["d_ff"], cfg_p["vocab"], cfg_p["n_layers"]
    nq, enc = cfg_p["n_heads"] * cfg_p["d_head"], cfg_p["enc_len"]
    ctx_len = mid_sequence(best)
    full_us = dec.time_forward(0, best + 1, 0, reps=30)
    op_bytes = {"qkv": 3 * nq * d * 2, "attn": 2 * nq * 2 * ctx_len, "o": d * nq * 2, "cross_q": nq * d * 2,
                "cross_attn": 2 * enc * nq * 2, "cross_o": d * nq * 2, "ffn_in": 2 * ff * d * 2, "ffn_out": d * ff * 2,
                "head": V * d * 2}
    kernels = {}
    for name, bit in binding.SD_OP.items():
        us = (full_us - dec.time_forward(0, best + 1, bit, reps=30)) / (1 if name == "head" else L)
        kernels[name] = {"bytes": op_bytes[name], "us": us, "GBps": op_bytes[name] / us / 1e3,
                         "frac_of_hbm_peak": op_bytes[name] / us / 1e3 / HBM_PEAK_GBPS,
                         "launches_per_forward": 1 if name == "head" else L}

    # the draft model's step, launch by launch, the same way (a draft step that is not an iteration's first)
    draft_us = dec.time_forward(1, 1, 0, reps=30)
    bytes_q_ops = {"qkv": 3 * cfg_q["n_heads"] * cfg_q["d_head"] * cfg_q["d_model"] * 2, "attn": 2 * cfg_q["n_heads"] * cfg_q["d_head"] * 2 * ctx_len,
                   "o": cfg_q["d_model"] * cfg_q["n_heads"] * cfg_q["d_head"] * 2, "cross_q": cfg_q["n_heads"] * cfg_q["d_head"] * cfg_q["d_model"] * 2,
                   "cross_attn": 2 * cfg_q["enc_len"] * cfg_q["n_heads"] * cfg_q["d_head"] * 2, "cross_o": cfg_q["d_model"] * cfg_q["n_heads"] * cfg_q["d_head"] * 2,
                   "ffn_in": 2 * cfg_q["d_ff"] * cfg_q["d_model"] * 2, "ffn_out": cfg_q["d_model"] * cfg_q["d_ff"] * 2, "head": V * cfg_q["d_model"] * 2}
    draft_kernels = {}
    for name, bit in binding.SD_OP.items():
        us = (draft_us - dec.time_forward(1, 1, bit, reps=30)) / (1 if name == "head" else cfg_q["n_layers"])
        draft_kernels[name] = {"bytes": bytes_q_ops[name], "us": us, "launches_per_forward": 1 if name == "head" else cfg_q["n_layers"]}
    # what the chip gives a kernel that only reads (the GEMMs' access shape, no arithmetic)
    ceiling_GBps = dec.stream_read_GBps(0, reps=5)

    # phase timing with HIP events on the library's stream (eager launches; a few % slower than the graph)
    dec.set_flags(binding.SD_FLAG_PROFILE)
    prof = {}
    for gamma in gammas:
        restart()
        urows = synth.uniform_stream(200 + gamma, 64 * (2 * gamma + 1)).reshape(64, -1)
        dr = v = a = 0.0
        n_it = 0
        for i in range(20):
            dec.step(gamma, TEMPERATURE, urows[i])
            st = dec.stats()
            if i >= 4:
                dr += st["draft_ms"]; v += st["verify_ms"]; a += st["accept_ms"]; n_it += 1
        st = dec.stats()
        prof[gamma] = {"draft_ms": dr / n_it, "verify_ms": v / n_it, "accept_ms": a / n_it,
                       "ffn_in_us": 1e3 * st["ffn_in_ms_sum"] / max(st["ffn_in_launches"], 1)}
    dec.set_flags(binding.SD_FLAG_GRAPH)

    res = per_gamma[best]
    plain_tps = 1e3 / base_ms
    for g in gammas:
        pg, pr, gr = per_gamma[g], prof[g], graph[g]
        pg.update({"speedup_vs_plain": pg["tokens_per_s"] / plain_tps,
                   "thm38_predicted_speedup": expected_tokens(pg["alpha"], g) / (g * gr["c"] + 1.0),
                   "c": gr["c"], "draft_step_us": gr["draft_step_us"], "verify_us": gr["verify_us"],
                   "verify_GBps": gr["verify_GBps"], "verify_frac_of_hbm_peak": gr["verify_GBps"] / HBM_PEAK_GBPS,
                   "eager_phase_ms": {"draft": pr["draft_ms"], "verify": pr["verify_ms"], "accept": pr["accept_ms"]}})

    # Roofline of the dominant kernel: the gated FFN-in GEMM streams both d_ff x d_model matrices
    # of a layer exactly once (algorithmic bytes per launch = 2 * d_ff * d_model * 2).  Its launch
    # duration inside the step: (verify forward) - (verify forward without its FFN-in launches), both
    # as graph replays, per layer.  The back-to-back replay of the 24 FFN-in launches alone is kept as
    # a second figure.
    ffn_bytes = op_bytes["ffn_in"]
    ffn_us = kernels["ffn_in"]["us"]
    ffn_us_alone = dec.time_ffn_in(best + 1, reps=20)
    roofline = {"bound": "hbm", "kernel": "gemm_kernel<bf16, PRO_POST, EPI_GATED> (Mp FFN-in, gated GELU)",
                "achieved": ffn_bytes / ffn_us / 1e3, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": ffn_bytes / ffn_us / 1e3 / HBM_PEAK_GBPS, "bytes_per_launch": ffn_bytes,
                "us_per_launch": ffn_us, "us_per_launch_method": "in-step: difference of graph-replayed verify forwards with / without the launch",
                "us_per_launch_back_to_back_alone": ffn_us_alone,
                "us_per_launch_between_events_eager": prof[best]["ffn_in_us"],
                "rows": best + 1, "traffic": traffic_from_profile(),
                "traffic_source": "profiles/ffn_in_gemm_t5xxl_hbm_traffic.txt (rocprofv3 FETCH_SIZE / WRITE_SIZE, copy-calibrated)"}
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
        "value_definition": "mean tokens per run of Algorithm 1 (pooled over the timed runs and five more whole "
                            "sequences) / ms_per_step of the timed runs, at the gamma with the best Eq.-1 rate",
        "tokens_per_s_measured": res["tokens_per_s_measured"],
        "per_gamma": {str(g): per_gamma[g] for g in gammas},
        "per_gamma_temperature0": {str(g): per_gamma_t0[g] for g in gammas},
        "autotune": {"gamma": tuned["gamma"], "alpha": tuned["alpha"], "c": tuned["c"],
                     "thm38_predicted_speedup": tuned["improvement"],
                     "measured_speedup": per_gamma[tuned["gamma"]]["tokens_per_s"] / plain_tps},
        "plain_decode_tokens_per_s": plain_tps, "plain_decode_ms_per_token": base_ms,
        "plain_decode_ms_per_token_runs": plain_runs,
        "plain_decode_GBps": (bytes_p["weights"] + bytes_p["cross_kv"]) / base_ms / 1e6,
        "speedup_vs_plain": res["speedup_vs_plain"],
        "verify_GBps": res["verify_GBps"], "verify_frac_of_hbm_peak": res["verify_frac_of_hbm_peak"],
        "verify_kernels": {"rows": best + 1, "context": ctx_len, "forward_us": full_us, "per_launch": kernels},
        "draft_kernels": {"rows": 1, "context": ctx_len, "forward_us": draft_us, "per_launch": draft_kernels},
        "hbm_read_ceiling_GBps": ceiling_GBps, "hbm_read_ceiling_frac_of_peak": ceiling_GBps / HBM_PEAK_GBPS,
        "verify_frac_of_read_ceiling": res["verify_GBps"] / ceiling_GBps,
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    dec.close()


def sampler_workload(args):
    """The isolated accept / resample call (sd_spec_sample) as configured: 64 independent rows,
    vocabulary 32128, gamma 7, target logits N(0, 3^2), draft = target + N(0, sigma^2) for sigma in
    0.5 / 1 / 2.  Per sigma: microseconds per call (both launches: 64 x 15 statistics workgroups,
    then one tail workgroup per row), the rate against the one-pass bytes (2 gamma + 1 logits rows per
    sequence, read once), and the measured acceptance rate.  One JSON line."""
    import numpy as np
    import torch
    from paper_2211_17192_amd import binding, synth
    rows, gamma, V = 64, 7, 32128
    nbytes = rows * (2 * gamma + 1) * V * 4
    reps = max(20, args.steps)
    per_sigma = {}
    for sigma in (0.5, 1.0, 2.0):
        zp, zq, x, r, s = [torch.from_numpy(a).cuda() for a in synth.sampler_case(rows, gamma, V, sigma, int(sigma * 10))]
        scratch = binding.spec_sample_scratch(rows, gamma)
        out_n = torch.empty(rows, dtype=torch.int32, device="cuda")
        out_t = torch.empty(rows, dtype=torch.int32, device="cuda")
        call = lambda: binding.spec_sample(zp, zq, x, r, s, TEMPERATURE, scratch, out_n, out_t)
        for _ in range(max(args.warmup, 3)):
            call()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        runs = []
        for _ in range(5):
            e0.record()
            for _ in range(reps):
                call()
            e1.record()
            torch.cuda.synchronize()
            runs.append(1e3 * e0.elapsed_time(e1) / reps)
        n = out_n.cpu().numpy()
        tested = int(np.minimum(n + 1, gamma).sum())       # guesses up to and including the first rejection
        us = statistics.median(runs)
        per_sigma[str(sigma)] = {"us_per_call": us, "us_per_call_min": min(runs), "GBps": nbytes / us / 1e3,
                                 "frac_of_hbm_peak": nbytes / us / 1e3 / HBM_PEAK_GBPS,
                                 "alpha": float(n.sum()) / max(tested, 1), "alpha_tests": tested,
                                 "mean_accepted": float(n.mean())}
    mid = per_sigma["1.0"]
    print(json.dumps({
        "metric": "accept / resample calls per second (64 rows, gamma 7, vocabulary 32128)", "value": 1e6 / mid["us_per_call"],
        "unit": "calls/s", "n_gpus": 1, "steps": reps, "warmup": max(args.warmup, 3), "ms_per_step": mid["us_per_call"] / 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "isolated fused speculative-sampling kernel (configs[2]): 64 rows, vocab 32128, gamma 7, "
                               "target logits N(0,9), draft = target + N(0, sigma^2), sigma 0.5 / 1 / 2, temperature 1"},
        "per_sigma": per_sigma,
        "roofline": {"bound": "hbm", "kernel": "spec_verify_kernel<1> + <2> (statistics pass over 15 logits rows per sequence, then the tail)",
                     "achieved": mid["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": mid["frac_of_hbm_peak"],
                     "bytes_per_launch": nbytes, "us_per_launch": mid["us_per_call"], "traffic": None},
        "cpu_baseline": None}), flush=True)


def gpt97m_workload(args):
    """The GPT-like pair (Mp 12 layers, d_model 768, vocab 8192, ~97M parameters; Mq 2 layers, d_model
    256, ~6M), bf16, batch 1, 128-token random prompt, 256 generated tokens, temperature 1, gamma
    3 / 5 / 7: the launch-latency regime (Mp's weights are 23 us of HBM time).  One JSON line."""
    import torch
    from paper_2211_17192_amd import binding, synth
    gammas = [int(g) for g in args.gammas.split(",")]
    cfg_p, w_p, cfg_q, w_q = synth.gpt_pair("cuda", emb_rms=4.0, head_std=0.1)
    dec = binding.SpecDecoder(cfg_p, w_p, cfg_q, w_q, max_gamma=max(gammas), flags=binding.SD_FLAG_GRAPH)
    prompt = synth.random_tokens(5, 128, cfg_p["vocab"])
    gen = 256

    def restart():
        dec.reset()
        dec.prefill(prompt)

    per_gamma = {}
    for gamma in gammas:
        urows = synth.uniform_stream(100 + gamma, 1024 * (2 * gamma + 1)).reshape(1024, -1)
        run_sequences(dec, gamma, TEMPERATURE, urows, restart, torch, n_steps=args.warmup, gen_len=gen)
        timed, _ = run_sequences(dec, gamma, TEMPERATURE, urows, restart, torch, n_steps=args.steps, gen_len=gen)
        extra, per_seq = run_sequences(dec, gamma, TEMPERATURE, urows[256:], restart, torch, n_sequences=EXTRA_SEQUENCES, gen_len=gen)
        pool = Tally(); pool.add(timed); pool.add(extra)
        ms = 1e3 * timed.secs / args.steps
        mq_us, mp_us = dec.measure_cost(reps=20)
        alpha = pool.accepted / max(pool.tested, 1)
        per_gamma[gamma] = {"tokens_per_s": (pool.tokens / pool.steps) / ms * 1e3, "ms_per_step": ms,
                            "tokens_per_step": pool.tokens / pool.steps, "alpha": alpha, "alpha_tests": pool.tested,
                            "eq1_tokens_per_s": expected_tokens(alpha, gamma) / ms * 1e3,
                            "c": mq_us / mp_us, "draft_step_us": mq_us, "plain_step_us": mp_us,
                            "thm38_predicted_speedup": expected_tokens(alpha, gamma) / (gamma * mq_us / mp_us + 1.0),
                            "sequences": {"n": len(per_seq), "tokens": gen, "tokens_per_s_median": statistics.median(per_seq),
                                          "tokens_per_s_min": min(per_seq)}}
    ub = synth.uniform_stream(7, gen)
    plain_runs = []
    for rep in range(3):
        restart()
        for i in range(8):
            dec.step_baseline(TEMPERATURE, ub[i])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(8, gen - 1):
            dec.step_baseline(TEMPERATURE, ub[i])
        torch.cuda.synchronize()
        plain_runs.append(1e3 * (time.perf_counter() - t0) / (gen - 9))
    base_ms = statistics.median(plain_runs)
    best = max(gammas, key=lambda g: per_gamma[g]["eq1_tokens_per_s"])
    for g in gammas:
        per_gamma[g]["speedup_vs_plain"] = per_gamma[g]["tokens_per_s"] * base_ms / 1e3
    bytes_p = synth.model_bytes(cfg_p)
    r = per_gamma[best]
    dec.close()
    print(json.dumps({
        "metric": "generated tokens/s at batch 1 (GPT-like 97M / 6M pair, gamma=3/5/7)", "value": r["tokens_per_s"],
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "GPT-like pair (configs[1]): Mp 12L d768 12 heads ff3072 V8192, Mq 2L d256 4 heads ff1024; "
                               "batch 1, 128-token prompt, 256 generated tokens, temperature 1", "gamma": best, "gammas": gammas},
        "per_gamma": {str(g): per_gamma[g] for g in gammas},
        "plain_decode_tokens_per_s": 1e3 / base_ms, "plain_decode_ms_per_token": base_ms,
        "plain_decode_GBps": bytes_p["weights"] / base_ms / 1e6, "speedup_vs_plain": r["speedup_vs_plain"],
        "roofline": None, "cpu_baseline": None}), flush=True)


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
    """The NumPy oracle, as it stands, on the host cores, on the same T5-XXL-shaped pair: eight tokens
    of plain Mp decoding and three runs of Algorithm 1 (gamma = 3) from the start token.  `value` is the
    speculative rate, extrapolated from that sample to the 128-token sequences of the GPU figure."""
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
    gamma, n_plain, n_spec = 3, 8, 3
    t0 = time.perf_counter()
    decode.plain_decode(T.CachedScorer(mp), [0], n_plain, TEMPERATURE, synth.uniform_stream(6, n_plain))
    plain_s = time.perf_counter() - t0
    u = synth.uniform_stream(5, n_spec * (2 * gamma + 1)).reshape(n_spec, -1)
    sp, sq, prefix = T.CachedScorer(mp), T.CachedScorer(mq), [0]
    t0 = time.perf_counter()
    for i in range(n_spec):
        prefix, n, _ = decode.speculative_decoding_step(sp, sq, prefix, gamma, TEMPERATURE, u[i])
    spec_s = time.perf_counter() - t0
    tokens = len(prefix) - 1
    return {"value": tokens / spec_s, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"extrapolated from {n_spec} runs of Algorithm 1 at gamma={gamma} ({tokens} tokens in {spec_s:.1f} s) "
                      f"and {n_plain} tokens of plain decoding ({plain_s:.1f} s) on the full T5-XXL-shaped pair, float64 NumPy; "
                      f"cross-attention K/V set-up {t_enc:.1f} s not counted",
            "plain_tokens_per_s": n_plain / plain_s, "speculative_over_plain": (tokens / spec_s) / (n_plain / plain_s),
            "host_cpus": os.cpu_count()}


if __name__ == "__main__":
    main()
