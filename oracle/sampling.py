"""Oracle: standardised sampling and the accept / resample part of Algorithm 1.

TEST INFRASTRUCTURE ONLY -- never imported by the product path.

Everything is float64 NumPy, written as the paper states it:

* section 2.2 (standardised sampling): temperature and argmax are folded
  into an ordinary probability vector;
* section 2.3 (speculative sampling) and Algorithm 1: the acceptance test
  r_i <= p_i(x_i)/q_i(x_i), n = index of the first rejection, the adjusted
  distribution norm(max(0, p_{n+1} - q_{n+1})) and the final draw.

Readings where the paper is silent:
* a guess is accepted when r <= p/q (the algorithm rejects when r > p/q);
  callers supply uniforms from the open interval (0, 1);
* "x ~ dist" is realised by inverse-CDF sampling in vocabulary-index order
  from a caller supplied uniform: the smallest k whose cumulative weight
  exceeds u times the total weight;
* argmax ties go to the lowest index;
* if the residual max(0, p - q) has zero total weight in floating point, the
  draw falls back to p_{n+1} itself.
"""
from __future__ import annotations

import numpy as np


def standardise(logits, temperature: float, top_k: int = 0, top_p: float = 0.0) -> np.ndarray:
    """Section 2.2: turn one logits row into the distribution that is sampled.

    temperature > 0: softmax(logits / temperature).
    temperature == 0: argmax sampling, i.e. all mass on the (lowest-index)
    maximum -- "zeroing out non-max elements and normalizing".
    top_k > 0: only the k most probable tokens keep their mass (top-k sampling);
    0 < top_p < 1: then only the smallest set of most probable tokens whose mass
    reaches top_p keeps its mass (nucleus sampling); the rest is renormalised.
    The section names both as samplers that become plain sampling from an
    adjusted distribution but does not define them; the definitions used here:
    a token is kept by top-k when its logit is >= the k-th largest logit, and by
    the nucleus when its logit is >= the logit of the token at which the
    descending cumulative mass first reaches top_p -- so tokens tied with the
    last kept one are kept with it.  Argmax sampling ignores both.
    """
    z = np.asarray(logits, dtype=np.float64)
    if z.ndim != 1:
        raise ValueError("standardise takes one logits row")
    if temperature < 0:
        raise ValueError("temperature must be >= 0")
    if temperature == 0:
        out = np.zeros_like(z)
        out[int(np.argmax(z))] = 1.0          # np.argmax returns the first maximum
        return out
    y = z / float(temperature)
    e = np.exp(y - np.max(y))
    if top_k > 0:
        kth = np.sort(z)[::-1][min(int(top_k), z.size) - 1]
        e = np.where(z >= kth, e, 0.0)
    if 0.0 < top_p < 1.0:
        order = np.argsort(-z, kind="stable")
        cum = np.cumsum(e[order])
        first = int(np.nonzero(cum >= top_p * cum[-1])[0][0])
        e = np.where(z >= z[order[first]], e, 0.0)
    return e / np.sum(e)


def nucleus_margin(logits, temperature: float, top_k: int, top_p: float) -> float:
    """How close the nucleus decision of standardise() is to flipping: the smallest
    distance, in units of total mass, between top_p and the descending cumulative
    mass at a boundary between distinct logit values.  Tests use it to recognise
    rows where fp32 and fp64 arithmetic may legitimately choose different sets."""
    z = np.asarray(logits, dtype=np.float64)
    y = z / float(temperature)
    e = np.exp(y - np.max(y))
    if top_k > 0:
        kth = np.sort(z)[::-1][min(int(top_k), z.size) - 1]
        e = np.where(z >= kth, e, 0.0)
    order = np.argsort(-z, kind="stable")
    cum = np.cumsum(e[order]) / np.sum(e)
    return float(np.min(np.abs(cum - top_p)))


def icdf(weights, u: float) -> int:
    """Inverse-CDF draw from unnormalised non-negative weights.

    Returns the smallest index k with sum_{j<=k} w_j > u * sum_j w_j, sums
    taken in index order.  If round-off leaves no such k, the last index with
    a positive weight is returned.
    """
    w = np.asarray(weights, dtype=np.float64)
    if np.any(w < 0):
        raise ValueError("negative weight")
    c = np.cumsum(w)
    total = c[-1]
    if not total > 0:
        raise ValueError("weights sum to zero")
    k = int(np.searchsorted(c, u * total, side="right"))
    if k >= w.size:
        k = int(np.nonzero(w > 0)[0][-1])
    return k


def beta(p, q) -> float:
    """Acceptance probability of one guess: sum_x min(p(x), q(x)) (Theorem 3.5)."""
    return float(np.sum(np.minimum(np.asarray(p, np.float64), np.asarray(q, np.float64))))


def d_lk(p, q) -> float:
    """Definition 3.2: sum_x |p(x) - M(x)| with M = (p + q)/2."""
    p = np.asarray(p, np.float64)
    q = np.asarray(q, np.float64)
    m = 0.5 * (p + q)
    return float(np.sum(np.abs(p - m)))


def adjusted_distribution(p, q) -> np.ndarray:
    """Unnormalised residual max(0, p - q) of section 2.3 / Algorithm 1."""
    return np.maximum(0.0, np.asarray(p, np.float64) - np.asarray(q, np.float64))


def accept_and_resample(p_rows, q_rows, x, r, s, lenience: float = 1.0):
    """Second half of Algorithm 1, on explicit distributions.

    p_rows : [gamma+1, V] target distributions p_1..p_{gamma+1}
    q_rows : [gamma, V]   draft distributions q_1..q_gamma
    x      : [gamma]      draft tokens x_i ~ q_i
    r      : [gamma]      uniforms of the acceptance tests
    s      : uniform of the final draw
    lenience : the factor l of appendix A.5 (q is multiplied by l before the
               comparison with p; 1 gives the exact algorithm).

    Returns (n, t, info): n accepted guesses, the extra token t, and a dict
    with the per-decision ratios p_i(x_i)/q_i(x_i), margins |r_i - ratio| and
    whether the zero-residual fallback was taken.
    """
    p_rows = np.asarray(p_rows, np.float64)
    q_rows = np.asarray(q_rows, np.float64)
    gamma = q_rows.shape[0]
    if p_rows.shape[0] != gamma + 1 or len(x) != gamma or len(r) != gamma:
        raise ValueError("shape mismatch")
    ratios = np.empty(gamma)
    for i in range(gamma):
        qi = q_rows[i, x[i]] * lenience
        pi = p_rows[i, x[i]]
        ratios[i] = np.inf if qi == 0 else pi / qi
    n = gamma
    for i in range(gamma):
        if r[i] > ratios[i]:                   # first rejected guess
            n = i
            break
    fallback = False
    if n < gamma:
        w = adjusted_distribution(p_rows[n], lenience * q_rows[n])
        if not np.sum(w) > 0:
            w = p_rows[n]
            fallback = True
    else:
        w = p_rows[gamma]
    t = icdf(w, s)
    info = {"ratios": ratios, "margins": np.abs(np.asarray(r, np.float64) - ratios),
            "fallback": fallback}
    return n, t, info


def accept_and_resample_argmax_lenient(p_logits, x, lenience: float):
    """Appendix A.5, last paragraph: lenience under argmax sampling (temperature 0).

    The one-hot distributions leave the ordinary test nothing to relax, so the
    lenience is applied before standardising: guess x_i is kept when
    p_i(x_i) >= l * max p_i, where p_i is the softmax of the unscaled logits (the
    paper prints "<=", which would keep exactly the unlikely tokens; read as a
    misprint).  In logits: z[x_i] - max z >= ln l.  The extra token is the argmax
    of the row after the kept guesses.  Returns (n, t).
    """
    z = np.asarray(p_logits, np.float64)
    gamma = len(x)
    if z.shape[0] != gamma + 1:
        raise ValueError("shape mismatch")
    log_l = np.log(np.float64(np.float32(lenience)))
    n = gamma
    for i in range(gamma):
        if z[i, x[i]] - np.max(z[i]) < log_l:
            n = i
            break
    return n, int(np.argmax(z[n]))


def accept_and_resample_from_logits(p_logits, q_logits, x, r, s, temperature: float, lenience: float = 1.0,
                                    top_k: int = 0, top_p: float = 0.0):
    """Same as accept_and_resample, starting from logits rows (section 2.2 first; the same
    standardisation for both models).  With temperature 0 and lenience < 1 the argmax
    variant of the lenient test applies."""
    if temperature == 0 and lenience < 1.0:
        n, t = accept_and_resample_argmax_lenient(p_logits, x, lenience)
        return n, t, {"fallback": False, "ratios": None, "margins": None}
    p_rows = np.stack([standardise(z, temperature, top_k, top_p) for z in p_logits])
    q_rows = np.stack([standardise(z, temperature, top_k, top_p) for z in q_logits])
    return accept_and_resample(p_rows, q_rows, x, r, s, lenience=np.float64(np.float32(lenience)))


def icdf_edge_distance(weights, u: float, k: int) -> float:
    """Distance, in normalised CDF units, from u to the nearer edge of token k's
    CDF interval.  Used by parity tests to recognise draws that a different
    summation order may legitimately flip."""
    w = np.asarray(weights, np.float64)
    c = np.cumsum(w) / np.sum(w)
    lo = 0.0 if k == 0 else c[k - 1]
    hi = c[k]
    return float(min(abs(u - lo), abs(u - hi)))
