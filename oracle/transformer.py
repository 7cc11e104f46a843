"""Oracle: the decoder models Mp / Mq of the synthetic workloads (float64 NumPy).

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

The paper treats Mp and Mq as black boxes that map a prefix to a next-token
distribution (section 2.1) and only gives sizes for its experiments
(section 4).  The internals below are therefore this build's own written
model specification; the GPU path implements the same prose independently.

Three block types ("arch"):

  GPT    pre-LayerNorm (gain + bias), learned absolute positions, linear
         layers with bias, tanh-GELU MLP, attention scale 1/sqrt(d_head).
  T5DEC  RMSNorm (gain only), no biases, unscaled attention with one
         relative-position bias table [n_heads, rel_buckets] shared by all
         layers, cross-attention over a fixed encoder output (no bias),
         gated tanh-GELU MLP.
  GQA    RMSNorm, rotary positions on adjacent pairs (2i, 2i+1), grouped
         key/value heads, attention scale 1/sqrt(d_head), SwiGLU MLP.

All linear weights are stored [out_features, in_features].  Logits are
logit_scale * (final_norm(x) @ head^T).

Precision model.  dtype "f32": every step in float64 on the float32 weight
values.  dtype "bf16": weights are bf16 values; the residual stream and all
accumulations stay wide, and a tensor is rounded to bf16 (nearest-even)
exactly where the GPU path stores or feeds one in bf16: the normed GEMM
input, q / k / v (after rotary), the attention output, the MLP hidden
activation and the final normed row.  For RMSNorm the rounded GEMM input is
x * gain and the division by rms(x) is applied to the GEMM output rows (the
same product; only the place of the rounding is fixed by this convention).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

GPT, T5DEC, GQA = 0, 1, 2


@dataclass
class ModelConfig:
    arch: int
    n_layers: int
    d_model: int
    n_heads: int
    d_head: int
    d_ff: int
    vocab: int
    max_len: int
    n_kv_heads: int = 0            # 0 -> n_heads
    enc_len: int = 0
    rel_buckets: int = 32
    rel_max_dist: int = 128
    rope_theta: float = 10000.0
    logit_scale: float = 1.0
    norm_eps: float = 1e-5
    dtype: str = "f32"             # "f32" | "bf16"

    def __post_init__(self):
        if self.n_kv_heads == 0:
            self.n_kv_heads = self.n_heads


# --------------------------------------------------------------------------
# number formats
# --------------------------------------------------------------------------
def bf16_round(a) -> np.ndarray:
    """Round float64 values to the nearest bf16 (ties to even), return float64."""
    f = np.ascontiguousarray(np.asarray(a, dtype=np.float64).astype(np.float32))
    bits = f.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(a))


def bf16_bits_to_f64(u16) -> np.ndarray:
    """Decode an array of bf16 bit patterns (uint16) to float64 (exact).  Large
    arrays go through torch's CPU conversion, which is multi-threaded."""
    u = np.ascontiguousarray(np.asarray(u16, dtype=np.uint16))
    if u.size >= (1 << 20):
        import torch
        return torch.from_numpy(u.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    return (u.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def to_f64(a) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return bf16_bits_to_f64(a)
    return a.astype(np.float64)


# --------------------------------------------------------------------------
# elementary layers (textbook definitions)
# --------------------------------------------------------------------------
def layer_norm(x, gain, bias, eps):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * gain + bias


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def softmax_rows(s):
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def rel_bucket(rel: int, n_buckets: int, max_dist: int) -> int:
    """Bucket of the causal distance rel = query_pos - key_pos >= 0.

    The first half of the buckets hold one distance each; the second half is
    spaced logarithmically up to max_dist; anything farther shares the last
    bucket (the unidirectional bucketing of the T5 paper).
    """
    half = n_buckets // 2
    if rel < half:
        return int(rel)
    b = half + int(np.floor(np.log(rel / half) / np.log(max_dist / half) * (n_buckets - half)))
    return min(b, n_buckets - 1)


def rotate_pairs(v, pos, theta):
    """Rotary embedding on adjacent pairs: (v[2i], v[2i+1]) is rotated by the
    angle pos * theta**(-2i/d).  v: [..., d] for one position."""
    d = v.shape[-1]
    i = np.arange(d // 2, dtype=np.float64)
    ang = float(pos) * theta ** (-2.0 * i / d)
    c, s = np.cos(ang), np.sin(ang)
    out = np.empty_like(v)
    a, b = v[..., 0::2], v[..., 1::2]
    out[..., 0::2] = a * c - b * s
    out[..., 1::2] = a * s + b * c
    return out


# --------------------------------------------------------------------------
# the model
# --------------------------------------------------------------------------
class KVCache:
    """Per-layer key / value rows for positions 0..max_len-1 (float64)."""

    def __init__(self, cfg: ModelConfig):
        w = cfg.n_kv_heads * cfg.d_head
        self.k = np.zeros((cfg.n_layers, cfg.max_len, w))
        self.v = np.zeros((cfg.n_layers, cfg.max_len, w))


class Transformer:
    """weights: dict name -> ndarray; float32 for dtype "f32", bf16 bit
    patterns as uint16 (or float32 holding bf16 values) for dtype "bf16"."""

    def __init__(self, cfg: ModelConfig, weights: dict):
        self.cfg = cfg
        self.wt = weights
        self.cross_k = None
        self.cross_v = None
        self._small = {}

    # -- helpers -----------------------------------------------------------
    def R(self, a):
        return bf16_round(a) if self.cfg.dtype == "bf16" else a

    def W(self, name):
        """Weight as float64.  Big matrices are decoded on every use so that a
        multi-gigabyte model never exists twice in memory."""
        a = self.wt[name]
        if a.size <= (1 << 22):
            if name not in self._small:
                self._small[name] = to_f64(a)
            return self._small[name]
        return to_f64(a)

    def linear(self, x, wname, bname=None):
        """x @ W^T (+ bias).  A big weight is decoded and multiplied in blocks of
        output features, so its float64 copy never exists as a whole; every
        output element is still one full-length dot product."""
        a = self.wt[wname]
        if a.size <= (1 << 22):
            y = x @ self.W(wname).T
        else:
            y = np.empty((x.shape[0], a.shape[0]))
            for r0 in range(0, a.shape[0], 2048):
                y[:, r0:r0 + 2048] = x @ to_f64(a[r0:r0 + 2048]).T
        if bname is not None:
            y = y + self.W(bname)
        return y

    def normed(self, x, prefix):
        """(h, rs): the rows fed to the linear layers after a norm and the per-row
        factor their outputs are multiplied by.  LayerNorm: h = R(LN(x)), rs = 1.
        RMSNorm: h = R(x * gain), rs = 1 / sqrt(mean(x^2) + eps), so that
        (h @ W^T) * rs = rms_norm(x) @ W^T up to the rounding R."""
        c = self.cfg
        if c.arch == GPT:
            return self.R(layer_norm(x, self.W(prefix + ".g"), self.W(prefix + ".b"), c.norm_eps)), 1.0
        rs = 1.0 / np.sqrt((x ** 2).mean(axis=-1, keepdims=True) + c.norm_eps)
        return self.R(x * self.W(prefix + ".g")), rs

    # -- encoder side (T5DEC) ------------------------------------------------
    def set_encoder_output(self, enc_out):
        """Cross-attention keys / values of every layer from a fixed encoder
        output [enc_len, d_model]; computed once per sequence."""
        c = self.cfg
        e = to_f64(enc_out)
        assert e.shape == (c.enc_len, c.d_model)
        self.cross_k = [self.R(self.linear(e, f"l{l}.ck")) for l in range(c.n_layers)]
        self.cross_v = [self.R(self.linear(e, f"l{l}.cv")) for l in range(c.n_layers)]

    # -- attention over explicit key / value rows -----------------------------
    def _attend(self, q, keys, vals, scale, bias=None, causal_pos=None):
        """q [M, H*dh]; keys, vals [L, Hkv*dh]; bias [H, M, L] or None;
        causal_pos[m] = last visible key index of row m (None: all visible)."""
        c = self.cfg
        M, L = q.shape[0], keys.shape[0]
        group = c.n_heads // c.n_kv_heads
        out = np.zeros((M, c.n_heads * c.d_head))
        for h in range(c.n_heads):
            g = h // group
            qh = q[:, h * c.d_head:(h + 1) * c.d_head]
            kh = keys[:, g * c.d_head:(g + 1) * c.d_head]
            vh = vals[:, g * c.d_head:(g + 1) * c.d_head]
            s = scale * (qh @ kh.T)
            if bias is not None:
                s = s + bias[h]
            if causal_pos is not None:
                for m in range(M):
                    s[m, causal_pos[m] + 1:] = -np.inf
            out[:, h * c.d_head:(h + 1) * c.d_head] = softmax_rows(s) @ vh
        return out

    # -- forward -------------------------------------------------------------
    def forward(self, tokens, start_pos: int, cache: KVCache) -> np.ndarray:
        """Process tokens at positions start_pos .. start_pos+M-1 given cached
        keys / values for positions < start_pos.  Appends the new rows to the
        cache and returns logits [M, vocab] (float64); row m is the
        distribution of the token following position start_pos+m."""
        c = self.cfg
        tokens = np.asarray(tokens, dtype=np.int64)
        M = tokens.shape[0]
        pos = np.arange(start_pos, start_pos + M)
        if start_pos + M > c.max_len:
            raise ValueError("sequence exceeds max_len")
        x = to_f64(np.asarray(self.wt["tok_emb"])[tokens])          # decode only the rows that are used
        if c.arch == GPT:
            x = x + to_f64(np.asarray(self.wt["pos_emb"])[pos])
        scale = 1.0 if c.arch == T5DEC else 1.0 / np.sqrt(c.d_head)
        L = start_pos + M
        bias = None
        if c.arch == T5DEC:
            tab = self.W("rel_bias")                        # [H, buckets]
            bucket = np.zeros((M, L), dtype=np.int64)
            for m in range(M):
                for j in range(pos[m] + 1):
                    bucket[m, j] = rel_bucket(pos[m] - j, c.rel_buckets, c.rel_max_dist)
            bias = tab[:, bucket]                           # [H, M, L]
        for l in range(c.n_layers):
            p = f"l{l}"
            h, rs = self.normed(x, p + ".ln1")
            if c.arch == GPT:
                q = self.linear(h, p + ".wq", p + ".bq")
                k = self.linear(h, p + ".wk", p + ".bk")
                v = self.linear(h, p + ".wv", p + ".bv")
            else:
                q = self.linear(h, p + ".wq") * rs
                k = self.linear(h, p + ".wk") * rs
                v = self.linear(h, p + ".wv") * rs
            if c.arch == GQA:
                q = q.reshape(M, c.n_heads, c.d_head)
                k = k.reshape(M, c.n_kv_heads, c.d_head)
                for m in range(M):
                    q[m] = rotate_pairs(q[m], pos[m], c.rope_theta)
                    k[m] = rotate_pairs(k[m], pos[m], c.rope_theta)
                q = q.reshape(M, -1)
                k = k.reshape(M, -1)
            q, k, v = self.R(q), self.R(k), self.R(v)
            cache.k[l, start_pos:L] = k
            cache.v[l, start_pos:L] = v
            a = self.R(self._attend(q, cache.k[l, :L], cache.v[l, :L], scale, bias, pos))
            x = x + self.linear(a, p + ".wo", p + ".bo" if c.arch == GPT else None)
            if c.arch == T5DEC:
                hc, rsc = self.normed(x, p + ".lnc")
                qc = self.R(self.linear(hc, p + ".cq") * rsc)
                ac = self.R(self._attend(qc, self.cross_k[l], self.cross_v[l], 1.0))
                x = x + self.linear(ac, p + ".co")
            h2, rs2 = self.normed(x, p + ".ln2")
            if c.arch == GPT:
                f = self.R(gelu_tanh(self.linear(h2, p + ".w1", p + ".b1")))
                x = x + self.linear(f, p + ".w2", p + ".b2")
            else:
                act = gelu_tanh if c.arch == T5DEC else silu
                f = self.R(act(self.linear(h2, p + ".wg") * rs2) * (self.linear(h2, p + ".wu") * rs2))
                x = x + self.linear(f, p + ".w2")
        hf, rsf = self.normed(x, "lnf")
        return c.logit_scale * (self.linear(hf, "head") * rsf)


class CachedScorer:
    """Prefix -> next-token logits with a KV cache that is reused for the
    longest common prefix of consecutive calls (stale rows are recomputed).
    use_cache=False recomputes every call from position 0: the plain
    definition M(prefix) of section 2.1."""

    def __init__(self, model: Transformer, use_cache: bool = True):
        self.model = model
        self.use_cache = use_cache
        self.cache = KVCache(model.cfg)
        self.cached = []

    def score(self, prefix, k: int) -> np.ndarray:
        """Logits rows for the last k positions of prefix: row j is the
        next-token distribution given prefix[: len(prefix)-k+1+j]."""
        prefix = [int(t) for t in prefix]
        n = len(prefix)
        common = 0
        if self.use_cache:
            lim = min(len(self.cached), n - k)
            while common < lim and self.cached[common] == prefix[common]:
                common += 1
        logits = self.model.forward(prefix[common:], common, self.cache)
        self.cached = prefix
        return logits[-k:]
