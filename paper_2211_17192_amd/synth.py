"""Seeded synthetic inputs: model shapes, weights, prompts and uniform streams.

This module serves the GPU path and the CPU oracle alike and holds none of
the method's arithmetic: it only draws numbers.  Weights come from a
counter-based generator written in integer torch ops, so the same call
gives bit-identical tensors on the CPU and on the GPU.

The paper's experiments (section 4) use trained checkpoints and public
datasets that are not available here; these generators stand in for them
with the same shapes.
"""
from __future__ import annotations

import math

import numpy as np
import torch

GPT, T5DEC, GQA = 0, 1, 2

_M32 = 0xFFFFFFFF


# --------------------------------------------------------------------------
# uniform streams (host side)
# --------------------------------------------------------------------------
def uniform_stream(seed: int, n: int) -> np.ndarray:
    """n uniforms strictly inside (0,1), each (k+0.5)/2**24 with k from a
    seeded PCG64 stream; every value is exact in float32."""
    g = np.random.Generator(np.random.PCG64(seed))
    k = g.integers(0, 1 << 24, size=n, dtype=np.int64)
    return ((k.astype(np.float64) + 0.5) / float(1 << 24)).astype(np.float32)


def random_tokens(seed: int, n: int, vocab: int) -> np.ndarray:
    g = np.random.Generator(np.random.PCG64(seed))
    return g.integers(0, vocab, size=n, dtype=np.int64).astype(np.int32)


# --------------------------------------------------------------------------
# counter-based normal generator (torch integer ops; same bits on any device)
# --------------------------------------------------------------------------
def _mix32(x: torch.Tensor) -> torch.Tensor:
    """32-bit avalanche mix on int64 tensors holding values < 2**32."""
    x = x ^ (x >> 16)
    x = (x * 0x85EBCA6B) & _M32
    x = x ^ (x >> 13)
    x = (x * 0xC2B2AE35) & _M32
    x = x ^ (x >> 16)
    return x


def counter_normal(shape, seed: int, std: float = 1.0, mean: float = 0.0,
                   device="cpu", dtype=torch.float32, chunk: int = 1 << 24) -> torch.Tensor:
    """Approximately normal values (sum of eight 16-bit uniforms, unit
    variance after scaling) indexed by (seed, element index)."""
    n = int(np.prod(shape))
    out = torch.empty(n, dtype=dtype, device=device)
    key = _mix32(torch.tensor([(seed * 2654435761 + 12345) & _M32], dtype=torch.int64, device=device))
    scale = 1.0 / math.sqrt(8.0 * (65536.0 ** 2 - 1.0) / 12.0) / 2.0
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        idx = torch.arange(lo, hi, dtype=torch.int64, device=device)
        h = _mix32(((idx & _M32) ^ key) + ((idx >> 32) * 0x9E3779B1 & _M32) & _M32)
        acc = torch.zeros_like(idx)
        for j in range(4):
            h = _mix32((h + 0x9E3779B9 * (j + 1)) & _M32)
            acc = acc + (h & 0xFFFF) + (h >> 16)
        z = (acc * 2 - 8 * 65535).to(torch.float32) * scale      # integer -> one fp32 multiply
        out[lo:hi] = (z * std + mean).to(dtype)
    return out.reshape(shape)


# --------------------------------------------------------------------------
# model shapes
# --------------------------------------------------------------------------
def model_cfg(arch, n_layers, d_model, n_heads, d_ff, vocab, max_len, *, d_head=None,
              n_kv_heads=0, enc_len=0, logit_scale=1.0, norm_eps=1e-5, dtype="f32",
              rel_buckets=32, rel_max_dist=128, rope_theta=10000.0) -> dict:
    return dict(arch=arch, n_layers=n_layers, d_model=d_model, n_heads=n_heads,
                d_head=d_head or d_model // n_heads, d_ff=d_ff, vocab=vocab, max_len=max_len,
                n_kv_heads=n_kv_heads or n_heads, enc_len=enc_len, rel_buckets=rel_buckets,
                rel_max_dist=rel_max_dist, rope_theta=rope_theta, logit_scale=logit_scale,
                norm_eps=norm_eps, dtype=dtype)


def weight_shapes(cfg: dict) -> dict:
    """name -> (shape, kind); kind in {"w", "gain", "bias"}."""
    c = cfg
    d, H, Hk, dh, ff, V = c["d_model"], c["n_heads"], c["n_kv_heads"], c["d_head"], c["d_ff"], c["vocab"]
    s = {"tok_emb": ((V, d), "w"), "head": ((V, d), "w"), "lnf.g": ((d,), "gain")}
    if c["arch"] == GPT:
        s["pos_emb"] = ((c["max_len"], d), "w")
        s["lnf.b"] = ((d,), "bias")
    if c["arch"] == T5DEC:
        s["rel_bias"] = ((H, c["rel_buckets"]), "relb")
    for l in range(c["n_layers"]):
        p = f"l{l}."
        s[p + "ln1.g"] = ((d,), "gain")
        s[p + "ln2.g"] = ((d,), "gain")
        s[p + "wq"] = ((H * dh, d), "w")
        s[p + "wk"] = ((Hk * dh, d), "w")
        s[p + "wv"] = ((Hk * dh, d), "w")
        s[p + "wo"] = ((d, H * dh), "w")
        if c["arch"] == GPT:
            for b, n in (("ln1.b", d), ("ln2.b", d), ("bq", H * dh), ("bk", Hk * dh),
                         ("bv", Hk * dh), ("bo", d), ("b1", ff), ("b2", d)):
                s[p + b] = ((n,), "bias")
            s[p + "w1"] = ((ff, d), "w")
            s[p + "w2"] = ((d, ff), "w")
        else:
            s[p + "wg"] = ((ff, d), "w")
            s[p + "wu"] = ((ff, d), "w")
            s[p + "w2"] = ((d, ff), "w")
        if c["arch"] == T5DEC:
            s[p + "lnc.g"] = ((d,), "gain")
            s[p + "cq"] = ((H * dh, d), "w")
            s[p + "ck"] = ((H * dh, d), "w")
            s[p + "cv"] = ((H * dh, d), "w")
            s[p + "co"] = ((d, H * dh), "w")
    return s


def _tdtype(cfg):
    return torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32


def random_weights(cfg: dict, seed: int, device="cpu", w_std: float = 0.02,
                   std_overrides: dict | None = None) -> dict:
    """All weights ~ N(0, w_std^2); norm gains 1 + N(0, w_std^2); biases
    N(0, w_std^2); relative-position bias table N(0, 0.5^2).
    std_overrides maps a name suffix (e.g. "head") to another std."""
    out = {}
    dt = _tdtype(cfg)
    for i, (name, (shape, kind)) in enumerate(weight_shapes(cfg).items()):
        std = w_std
        if std_overrides:
            for suf, v in std_overrides.items():
                if name.endswith(suf):
                    std = v
        sd = seed * 100003 + i
        if kind == "gain":
            t = counter_normal(shape, sd, w_std, 1.0, device)
        elif kind == "relb":
            t = counter_normal(shape, sd, 0.5, 0.0, device)
        else:
            t = counter_normal(shape, sd, std, 0.0, device)
        out[name] = t.to(dt)
    return out


def truncated_noisy_copy(cfg_p: dict, w_p: dict, n_layers_q: int, seed: int, noise_std: float):
    """Draft model made of Mp's embeddings, its first n_layers_q layers, final
    norm and head, every tensor perturbed by N(0, noise_std^2)."""
    cfg_q = dict(cfg_p)
    cfg_q["n_layers"] = n_layers_q
    out = {}
    for i, name in enumerate(weight_shapes(cfg_q)):
        src = w_p[name]
        noise = counter_normal(tuple(src.shape), seed * 100003 + i, noise_std, 0.0, src.device)
        out[name] = (src.float() + noise).to(src.dtype)
    return cfg_q, out


# --------------------------------------------------------------------------
# the workloads
# --------------------------------------------------------------------------
def tiny_pair(device="cpu", seed: int = 1):
    """Tiny fp32 decoder-only pair: Mp 2 layers, d_model 64, 2 heads, d_ff 256,
    vocab 256, learned positions, max length 128, logits scaled by 20; Mq is
    Mp's first layer with N(0, 0.01^2) weight noise."""
    cfg_p = model_cfg(GPT, 2, 64, 2, 256, 256, 128, logit_scale=20.0, dtype="f32")
    w_p = random_weights(cfg_p, seed, device)
    cfg_q, w_q = truncated_noisy_copy(cfg_p, w_p, 1, seed + 1000, 0.01)
    return cfg_p, w_p, cfg_q, w_q


def to_numpy_weights(w: dict) -> dict:
    """torch weights -> numpy for the oracle: float32 as is, bf16 as uint16 bit patterns."""
    out = {}
    for k, t in w.items():
        t = t.detach().cpu().contiguous()
        if t.dtype == torch.bfloat16:
            out[k] = t.view(torch.int16).numpy().view(np.uint16)
        else:
            out[k] = t.numpy()
    return out


def sampler_case(rows: int, gamma: int, vocab: int, sigma: float, seed: int):
    """Inputs of the isolated accept / resample kernel: target logits
    N(0, 3^2) [rows, gamma+1, V]; draft logits = target logits of the first gamma
    positions + N(0, sigma^2); guesses x_i drawn from softmax(draft logits) with
    numpy's categorical sampler; uniforms r [rows, gamma], s [rows].  numpy arrays."""
    g = np.random.Generator(np.random.PCG64(seed))
    zp = (3.0 * g.standard_normal((rows, gamma + 1, vocab), dtype=np.float32)).astype(np.float32)
    zq = (zp[:, :gamma] + sigma * g.standard_normal((rows, gamma, vocab), dtype=np.float32)).astype(np.float32)
    x = np.zeros((rows, gamma), dtype=np.int32)
    for b in range(rows):
        for i in range(gamma):
            z = zq[b, i].astype(np.float64)
            q = np.exp(z - z.max())
            x[b, i] = g.choice(vocab, p=q / q.sum())
    u = uniform_stream(seed + 7919, rows * (gamma + 1)).reshape(rows, gamma + 1)
    return zp, zq, x, np.ascontiguousarray(u[:, :gamma]), np.ascontiguousarray(u[:, gamma])


def correlated_pair(cfg_p: dict, cfg_q: dict, seed: int, device="cpu", emb_rms: float = 1.0,
                    head_std: float = 0.02, w_std: float = 0.02, q_logit_gain: float = 1.0):
    """Random-init (Mp, Mq) whose next-token distributions agree to a tunable
    degree, standing in for a trained target / draft pair.

    Both models share a token table E [V, d_q] and an output table H [V, d_q];
    Mq uses them directly, Mp sees them through a random rotation P (d_q
    orthonormal rows in d_p dimensions): tok_emb_p = a E P, head_p = H P.  On
    the embedding -> head skip path the two models then give the same logits;
    the randomly initialised layers perturb them differently, so a larger
    emb_rms (embedding magnitude relative to the layers' output) gives a higher
    acceptance rate.  Iteration time does not depend on these values."""
    d_p, d_q, V = cfg_p["d_model"], cfg_q["d_model"], cfg_p["vocab"]
    assert cfg_q["vocab"] == V and d_q <= d_p
    cfg_q = dict(cfg_q)
    w_p = random_weights(cfg_p, seed, device, w_std)
    w_q = random_weights(cfg_q, seed + 1, device, w_std)
    E = counter_normal((V, d_q), seed * 7 + 1, 1.0, 0.0, device)
    H = counter_normal((V, d_q), seed * 7 + 2, head_std, 0.0, device)
    G = counter_normal((d_p, d_q), seed * 7 + 3, 1.0, 0.0, device)
    P = torch.linalg.qr(G)[0].T.contiguous()                 # [d_q, d_p], orthonormal rows
    dt = _tdtype(cfg_p)
    w_p["tok_emb"] = (emb_rms * math.sqrt(d_p / d_q) * (E @ P)).to(dt)
    w_p["head"] = (H @ P).to(dt)
    w_q["tok_emb"] = (emb_rms * E).to(dt)
    w_q["head"] = H.to(dt)
    cfg_q["logit_scale"] = cfg_p["logit_scale"] * math.sqrt(d_p / d_q) * q_logit_gain
    return w_p, cfg_q, w_q


def t5xxl_pair(device="cuda", seed: int = 4, gen_len: int = 128, emb_rms: float = 32.0,
               head_std: float = 0.1, logit_scale: float = 1.0, q_logit_gain: float = 1.0):
    """T5-XXL-shaped decoder (24 layers, d_model 4096, 64 heads x 64, d_ff 10240
    gated-GELU, vocab 32128, 512 encoder positions) with a T5-small-shaped draft
    (6 layers, d_model 512, 8 heads x 64, d_ff 2048), bf16, random init.  The
    encoder stack is not run: encoder outputs are N(0,1) tensors."""
    max_len = (gen_len + 1 + 16 + 15) // 16 * 16
    cfg_p = model_cfg(T5DEC, 24, 4096, 64, 10240, 32128, max_len, d_head=64, enc_len=512,
                      norm_eps=1e-6, dtype="bf16", logit_scale=logit_scale)
    cfg_q = model_cfg(T5DEC, 6, 512, 8, 2048, 32128, max_len, d_head=64, enc_len=512,
                      norm_eps=1e-6, dtype="bf16", logit_scale=logit_scale)
    w_p, cfg_q, w_q = correlated_pair(cfg_p, cfg_q, seed, device, emb_rms, head_std, 0.02, q_logit_gain)
    enc_p = counter_normal((512, 4096), seed * 7 + 5, 1.0, 0.0, device).to(torch.bfloat16)
    enc_q = counter_normal((512, 512), seed * 7 + 6, 1.0, 0.0, device).to(torch.bfloat16)
    return cfg_p, w_p, cfg_q, w_q, enc_p, enc_q


def gpt_pair(device="cuda", seed: int = 2, emb_rms: float = 1.0, head_std: float = 0.02,
             logit_scale: float = 1.0, q_logit_gain: float = 1.0):
    """GPT-like pair in bf16: Mp 12 layers, d_model 768, 12 heads, d_ff 3072,
    vocab 8192 (~97M parameters); Mq 2 layers, d_model 256, 4 heads, d_ff 1024
    (~6M).  Room for a 128-token prompt plus 256 generated tokens."""
    cfg_p = model_cfg(GPT, 12, 768, 12, 3072, 8192, 416, dtype="bf16", logit_scale=logit_scale)
    cfg_q = model_cfg(GPT, 2, 256, 4, 1024, 8192, 416, dtype="bf16", logit_scale=logit_scale)
    w_p, cfg_q, w_q = correlated_pair(cfg_p, cfg_q, seed, device, emb_rms, head_std, 0.02, q_logit_gain)
    return cfg_p, w_p, cfg_q, w_q


def gqa8b_pair(device="cuda", seed: int = 6, max_len: int = 2336, emb_rms: float = 32.0,
               head_std: float = 0.1, logit_scale: float = 1.0, q_logit_gain: float = 1.0):
    """8B-class decoder-only target in bf16 (32 layers, d_model 4096, 32 query / 8 KV heads x 128,
    d_ff 14336 SwiGLU, vocab 32000, rotary positions) with a 2-layer draft (d_model 1024,
    8 heads x 128, d_ff 4096: the width is given, the rest is this build's choice), random init,
    correlated like the other pairs.  max_len 2336 = 2048 context + 256 generated + slack."""
    cfg_p = model_cfg(GQA, 32, 4096, 32, 14336, 32000, max_len, d_head=128, n_kv_heads=8,
                      norm_eps=1e-5, dtype="bf16", logit_scale=logit_scale)
    cfg_q = model_cfg(GQA, 2, 1024, 8, 4096, 32000, max_len, d_head=128, n_kv_heads=8,
                      norm_eps=1e-5, dtype="bf16", logit_scale=logit_scale)
    w_p, cfg_q, w_q = correlated_pair(cfg_p, cfg_q, seed, device, emb_rms, head_std, 0.02, q_logit_gain)
    return cfg_p, w_p, cfg_q, w_q


def model_bytes(cfg: dict) -> dict:
    """Bytes one forward has to read: layer + head weights (every row of them),
    and per cached position the self-attention keys / values."""
    e = 2 if cfg["dtype"] == "bf16" else 4
    shapes = weight_shapes(cfg)
    w = sum(int(np.prod(s)) for n, (s, k) in shapes.items()
            if k == "w" and n not in ("tok_emb", "pos_emb") and not n.endswith((".ck", ".cv")))
    cross = 2 * cfg["n_layers"] * cfg["enc_len"] * cfg["n_heads"] * cfg["d_head"] * e
    kv_per_pos = 2 * cfg["n_layers"] * cfg["n_kv_heads"] * cfg["d_head"] * e
    return {"weights": w * e, "cross_kv": cross, "kv_per_pos": kv_per_pos}
