"""Oracle: Algorithm 1 (SpeculativeDecodingStep) and the decoding loops.

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

A "scorer" is anything with score(prefix, k) -> logits rows [k, V] for the
last k positions of prefix (oracle.transformer.CachedScorer, or the table
models the tests use).  Uniforms for one step are laid out as
[d_1..d_gamma | r_1..r_gamma | s]: draft draws, acceptance tests, final draw.
"""
from __future__ import annotations

import numpy as np

from .sampling import accept_and_resample, accept_and_resample_argmax_lenient, icdf, standardise


def speculative_decoding_step(mp, mq, prefix, gamma: int, temperature: float, uniforms, lenience: float = 1.0,
                              top_k: int = 0, top_p: float = 0.0):
    """One run of Algorithm 1.  Returns (new_prefix, n, info).

    1. for i = 1..gamma: q_i = Mq(prefix + x_<i), x_i ~ q_i        (serial)
    2. p_1..p_{gamma+1} = Mp on prefix, prefix+[x_1], ..., prefix+[x_1..x_gamma]
    3. n = number of guesses before the first r_i > p_i(x_i)/q_i(x_i)
    4. t ~ p_{n+1}, replaced by norm(max(0, p_{n+1}-q_{n+1})) when n < gamma
    5. return prefix + [x_1..x_n, t]

    lenience < 1 relaxes step 3 as appendix A.5 describes (q multiplied by l; at
    temperature 0 the argmax variant).  top_k / top_p select the section 2.2
    standardisation, the same for both models.
    """
    u = np.asarray(uniforms, dtype=np.float64)
    if u.shape != (2 * gamma + 1,):
        raise ValueError("need 2*gamma+1 uniforms")
    if np.any(u <= 0) or np.any(u >= 1):
        raise ValueError("uniforms must lie in the open interval (0,1)")
    d, r, s = u[:gamma], u[gamma:2 * gamma], u[2 * gamma]
    prefix = [int(t) for t in prefix]
    x, q_rows, q_logits = [], [], []
    for i in range(gamma):
        zq = mq.score(prefix + x, 1)[0]
        qi = standardise(zq, temperature, top_k, top_p)
        x.append(icdf(qi, d[i]))
        q_rows.append(qi)
        q_logits.append(zq)
    zp = mp.score(prefix + x, gamma + 1)
    p_rows = np.stack([standardise(z, temperature, top_k, top_p) for z in zp])
    if temperature == 0 and lenience < 1.0:
        n, t = accept_and_resample_argmax_lenient(zp, x, lenience)
        info = {"fallback": False, "ratios": None, "margins": None}
    else:
        n, t, info = accept_and_resample(p_rows, np.stack(q_rows), x, r, s,
                                         lenience=float(np.float32(lenience)))
    info.update({"x": list(x), "p_logits": zp, "q_logits": np.stack(q_logits),
                 "p_rows": p_rows, "q_rows": np.stack(q_rows)})
    return prefix + x[:n] + [t], n, info


def speculative_decode(mp, mq, prompt, n_new: int, gamma: int, temperature: float, uniform_rows,
                       lenience: float = 1.0, top_k: int = 0, top_p: float = 0.0):
    """Repeat Algorithm 1 until n_new tokens exist; the surplus of the last
    run is dropped.  uniform_rows yields one [2*gamma+1] row per run.
    Returns (tokens, records) with one record (n, emitted tokens, info) per run."""
    prefix = [int(t) for t in prompt]
    target = len(prefix) + n_new
    records = []
    it = iter(uniform_rows)
    while len(prefix) < target:
        new_prefix, n, info = speculative_decoding_step(mp, mq, prefix, gamma, temperature, next(it), lenience, top_k, top_p)
        records.append((n, new_prefix[len(prefix):], info))
        prefix = new_prefix
    return prefix[:target], records


def plain_decode(mp, prompt, n_new: int, temperature: float, uniforms, top_k: int = 0, top_p: float = 0.0):
    """Standard autoregressive decoding from Mp alone: one token per run."""
    prefix = [int(t) for t in prompt]
    it = iter(uniforms)
    for _ in range(n_new):
        z = mp.score(prefix, 1)[0]
        prefix.append(icdf(standardise(z, temperature, top_k, top_p), float(next(it))))
    return prefix
