"""Seeded small model pairs shared by the CPU and GPU tests (inputs only: no method arithmetic)."""
from oracle import transformer as T
from paper_2211_17192_amd import synth

# Weight scale of the small bf16 pairs.  With w_std = 0.1 the T5DEC toy model (unscaled attention
# scores) is ill-conditioned in bf16 whoever evaluates it: the oracle's own bf16 model and its own
# unrounded model then differ by 12 % of a row's largest logit (tests/test_oracle_transformer.py
# measures it), so no 2e-2 comparison between two bf16 implementations means anything there.
# 0.06 keeps that gap below 2e-2 for every block type.  fp32 pairs use 0.1.
W_STD = {"f32": 0.1, "bf16": 0.06}


def small_cfg(arch, dtype, d_head=32):
    """d_head 32: two heads of 32 (GQA: four); d_head 64: two heads of 64 (GQA: four query, two KV heads),
    the head size the bf16 matrix-core attention kernel takes."""
    kw = dict(dtype=dtype, logit_scale=4.0)
    if d_head == 64:
        if arch == T.GPT:
            return synth.model_cfg(T.GPT, 3, 128, 2, 128, 512, 160, **kw)
        if arch == T.T5DEC:
            return synth.model_cfg(T.T5DEC, 3, 128, 2, 96, 512, 160, enc_len=72, norm_eps=1e-6, **kw)
        return synth.model_cfg(T.GQA, 3, 128, 4, 160, 512, 160, d_head=64, n_kv_heads=2, **kw)
    assert d_head == 32
    if arch == T.GPT:
        return synth.model_cfg(T.GPT, 3, 64, 2, 128, 512, 160, **kw)
    if arch == T.T5DEC:
        return synth.model_cfg(T.T5DEC, 3, 64, 2, 96, 512, 160, enc_len=40, norm_eps=1e-6, **kw)
    return synth.model_cfg(T.GQA, 3, 128, 4, 160, 512, 160, d_head=32, n_kv_heads=2, **kw)


def small_pair(arch, dtype, seed=3, w_std=None, d_head=32):
    """(cfg_p, w_p, cfg_q, w_q, enc_p, enc_q): a 3-layer target of the given block type and its
    1-layer noisy copy as the approximation model."""
    cfg = small_cfg(arch, dtype, d_head)
    w = synth.random_weights(cfg, seed, w_std=W_STD[dtype] if w_std is None else w_std)
    cfg_q, w_q = synth.truncated_noisy_copy(cfg, w, 1, seed + 50, 0.02)
    enc_p = enc_q = None
    if arch == T.T5DEC:
        enc_p = synth.counter_normal((cfg["enc_len"], cfg["d_model"]), 91, 1.0).to(w["head"].dtype)
        enc_q = enc_p.clone()
    return cfg, w, cfg_q, w_q, enc_p, enc_q


def unrounded(cfg):
    """The same model evaluated without any bf16 rounding of activations (weights keep their values)."""
    c = dict(cfg)
    c["dtype"] = "f32"
    return c


def row_rel_err(got, ref):
    """max over rows of (max_k |got - ref| of the row) / (max_k |ref| of the row)."""
    import numpy as np
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return float(np.max(np.abs(got - ref).max(axis=-1) / np.abs(ref).max(axis=-1)))
