"""Pins for oracle/sampling.py and oracle/decode.py (CPU only).

The pins are facts the paper fixes, checked through the oracle's own entry
points by exact enumeration: all uniforms run over midpoint grids chosen so
that, for the dyadic distributions used, no grid point ever coincides with a
decision threshold.  Counting grid points then gives exact probabilities.
"""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import analysis, decode, drafts, sampling


def grid(n):
    return [(k + 0.5) / n for k in range(n)]


class TableScorer:
    """Next-token distribution = table(prefix); logits = log(prob), so that at
    temperature 1 the standardised distribution is the table row itself."""

    def __init__(self, fn):
        self.fn = fn

    def score(self, prefix, k):
        rows = []
        for j in range(k):
            ctx = prefix[: len(prefix) - k + 1 + j]
            with np.errstate(divide="ignore"):
                rows.append(np.log(np.asarray(self.fn(ctx), dtype=np.float64)))
        return np.stack(rows)


P1 = [3 / 16, 5 / 16, 1 / 16, 7 / 16]
Q1 = [1 / 2, 1 / 4, 1 / 8, 1 / 8]
# second-position tables, depending on the previous token
P2 = {0: [1 / 4, 1 / 4, 1 / 4, 1 / 4], 1: [1 / 2, 0, 1 / 4, 1 / 4], 2: [0, 0, 1 / 2, 1 / 2], 3: [1 / 8, 3 / 8, 1 / 4, 1 / 4]}
Q2 = {0: [1 / 2, 1 / 2, 0, 0], 1: [1 / 4, 1 / 4, 1 / 4, 1 / 4], 2: [1 / 2, 0, 0, 1 / 2], 3: [1 / 4, 1 / 8, 1 / 8, 1 / 2]}


def table_models():
    mp = TableScorer(lambda ctx: P1 if len(ctx) == 1 else P2[ctx[-1]])
    mq = TableScorer(lambda ctx: Q1 if len(ctx) == 1 else Q2[ctx[-1]])
    return mp, mq


def test_standardise_matches_library_softmax_and_argmax():
    rng = np.random.default_rng(0)
    z = rng.normal(0, 3, size=50)
    for T in (1.0, 0.7, 2.5):
        np.testing.assert_allclose(sampling.standardise(z, T), scipy.special.softmax(z / T), rtol=1e-13)
    z[7] = z[30] = z.max() + 1.0                     # tie -> lowest index
    one = sampling.standardise(z, 0.0)
    assert one[7] == 1.0 and one.sum() == 1.0


def test_icdf_counts_equal_probabilities():
    w = np.array([3, 0, 5, 1, 0, 7], dtype=float)    # total 16
    counts = np.zeros(6, dtype=int)
    for u in grid(32):
        counts[sampling.icdf(w, u)] += 1
    assert list(counts) == [6, 0, 10, 2, 0, 14]


def test_single_token_speculative_sampling_is_distributed_as_p():
    """Appendix A.1: P(x = x') = p(x'), by exact enumeration with gamma = 1; the
    acceptance frequency equals sum min(p, q) (Theorem 3.5) and, given that
    the guess is kept, the bonus token follows p_2(. | x_1)."""
    mp, mq = table_models()
    first = np.zeros(4, dtype=int)
    accepted = 0
    second = {a: np.zeros(4, dtype=int) for a in range(4)}
    gd, gr, gs = grid(8), grid(16), grid(48)
    for d, r, s in itertools.product(gd, gr, gs):
        out, n, _ = decode.speculative_decoding_step(mp, mq, [0], 1, 1.0, [d, r, s])
        first[out[1]] += 1
        if n == 1:
            accepted += 1
            second[out[1]][out[2]] += 1
        else:
            assert len(out) == 2
    total = len(gd) * len(gr) * len(gs)
    assert [Fraction(int(c), total) for c in first] == [Fraction(p).limit_denominator(64) for p in P1]
    assert Fraction(accepted, total) == Fraction(10, 16) == Fraction(sampling.beta(P1, Q1)).limit_denominator(64)
    for a in range(4):
        na = second[a].sum()
        # P(first = a and kept) = min(p, q)(a)
        assert Fraction(int(na), total) == Fraction(min(P1[a], Q1[a])).limit_denominator(64)
        assert [Fraction(int(c), int(na)) for c in second[a]] == [Fraction(p).limit_denominator(64) for p in P2[a]]


def test_two_guess_step_joint_distribution():
    """gamma = 2 with context-dependent tables: first token ~ p_1; given the
    first guess a is kept, the second token ~ p_2(.|a); given both kept, the
    third ~ p_3 (here the uniform table)."""
    mp0, mq0 = table_models()
    P3 = [1 / 4, 1 / 4, 1 / 4, 1 / 4]
    mp = TableScorer(lambda ctx: P3 if len(ctx) == 3 else mp0.fn(ctx))
    mq = TableScorer(lambda ctx: P3 if len(ctx) == 3 else mq0.fn(ctx))
    first = np.zeros(4, dtype=int)
    pair = np.zeros((4, 4), dtype=int)
    third = np.zeros(4, dtype=int)
    gd, gr, gs = grid(8), grid(8), grid(12)
    total = 0
    for d1, d2, r1, r2 in itertools.product(gd, gd, gr, gr):
        for s in gs:
            out, n, _ = decode.speculative_decoding_step(mp, mq, [0], 2, 1.0, [d1, d2, r1, r2, s])
            total += 1
            assert len(out) == 1 + n + 1 and 0 <= n <= 2
            first[out[1]] += 1
            if n >= 1:
                pair[out[1], out[2]] += 1
            if n == 2:
                third[out[3]] += 1
    np.testing.assert_allclose(first / total, P1, atol=1e-12)
    for a in range(4):
        np.testing.assert_allclose(pair[a] / total, min(P1[a], Q1[a]) * np.array(P2[a]), atol=1e-12)
    np.testing.assert_allclose(third / third.sum(), P3, atol=1e-12)


def test_tokens_per_run_is_the_capped_geometric_of_equation_1():
    """Context-free tables (the i.i.d. assumption of section 3.1 holds exactly):
    the distribution of n and its mean match the capped geometric / Equation 1."""
    p, q = [3 / 4, 1 / 4], [1 / 2, 1 / 2]
    alpha = sampling.beta(p, q)
    assert alpha == 0.75
    mp, mq = TableScorer(lambda ctx: p), TableScorer(lambda ctx: q)
    gamma = 3
    hist = np.zeros(gamma + 1, dtype=int)
    g2 = grid(2)
    for u in itertools.product(*([g2] * (2 * gamma)), grid(4)):
        _, n, _ = decode.speculative_decoding_step(mp, mq, [0], gamma, 1.0, list(u))
        hist[n] += 1
    pmf = hist / hist.sum()
    np.testing.assert_allclose(pmf, analysis.capped_geometric_pmf(alpha, gamma), atol=1e-12)
    mean_tokens = float(np.sum((np.arange(gamma + 1) + 1) * pmf))
    assert abs(mean_tokens - (1 - 0.75 ** 4) / (1 - 0.75)) < 1e-12
    assert abs(mean_tokens - analysis.expected_tokens(alpha, gamma)) < 1e-12


def test_monte_carlo_output_distribution_chi_square():
    """Non-dyadic p, q on 8 tokens: tokens decoded by repeated runs of Algorithm 1
    from a context-free pair follow p (chi-square, fixed seed)."""
    rng = np.random.default_rng(5)
    p = rng.dirichlet(np.ones(8))
    q = rng.dirichlet(np.ones(8))
    mp, mq = TableScorer(lambda ctx: p), TableScorer(lambda ctx: q)
    gamma = 3
    counts = np.zeros(8)
    acc = tot = 0
    for _ in range(6000):
        u = (rng.integers(0, 1 << 24, size=2 * gamma + 1) + 0.5) / (1 << 24)
        out, n, _ = decode.speculative_decoding_step(mp, mq, [0], gamma, 1.0, u)
        for t in out[1:]:
            counts[t] += 1
        acc += n
        tot += min(n + 1, gamma)                    # guesses actually tested
    chi2, pval = scipy.stats.chisquare(counts, p * counts.sum())
    assert pval > 1e-3
    rate = acc / tot
    b = sampling.beta(p, q)
    assert abs(rate - b) < 4 * np.sqrt(b * (1 - b) / tot)


def test_dlk_identities():
    rng = np.random.default_rng(1)
    for _ in range(20):
        p, q = rng.dirichlet(np.ones(9)), rng.dirichlet(np.ones(9))
        assert abs(sampling.d_lk(p, q) - (1 - sampling.beta(p, q))) < 1e-14      # Lemma 3.3
        assert abs(sampling.d_lk(p, q) - sampling.d_lk(q, p)) < 1e-14
        # normaliser of the adjusted distribution is 1 - beta (appendix A.1)
        assert abs(sampling.adjusted_distribution(p, q).sum() - (1 - sampling.beta(p, q))) < 1e-14
    assert sampling.d_lk([1, 0, 0], [0, .5, .5]) == 1.0 and sampling.d_lk([.2, .8], [.2, .8]) == 0.0


def test_degenerate_cases():
    rng = np.random.default_rng(2)
    p = rng.dirichlet(np.ones(6), size=4)
    x = [int(np.argmax(p[i])) for i in range(3)]
    # q == p: every guess is kept whatever the uniforms (Corollary 3.4, D_LK = 0)
    for r in ([0.999] * 3, [0.5] * 3):
        n, t, info = sampling.accept_and_resample(p, p[:3], x, r, 0.3)
        assert n == 3 and not info["fallback"] and t == sampling.icdf(p[3], 0.3)
    # disjoint supports: first guess always rejected, t ~ p_1 unchanged
    pp = np.array([[.5, .5, 0, 0], [.25, .75, 0, 0]])
    qq = np.array([[0, 0, .5, .5]])
    for s in grid(4):
        n, t, _ = sampling.accept_and_resample(pp, qq, [2], [1e-7], s)
        assert n == 0 and t == sampling.icdf(pp[0], s)
    # rejected although p == q numerically impossible; zero residual -> fall back to p
    n, t, info = sampling.accept_and_resample(pp, pp[:1] * 1.0, [0], [0.5], 0.9)
    assert n == 1
    same = np.array([[.5, .5], [.5, .5]])
    bigger_q = np.array([[.5 + 1e-17, .5]])
    n, t, info = sampling.accept_and_resample(same, bigger_q, [0], [0.5], 0.9)
    assert n == 1                                     # ratio rounds to 1: kept
    # a rejection whose residual vanishes in floating point falls back to p itself
    q_eps = np.array([[.5 * (1 + 2.0 ** -52), .5]])
    n, t, info = sampling.accept_and_resample(same, q_eps, [0], [1 - 2.0 ** -53], 0.75)
    assert n == 0 and info["fallback"] and t == 1


def test_temperature_zero_is_argmax_logic():
    zp = np.array([[0., 2., 1.], [3., 0., 0.], [0., 0., 5.]])
    zq = np.array([[0., 1., 0.5], [0., 4., 0.]])
    # q argmaxes: 1, 1 ; p argmaxes: 1, 0, 2  -> first kept, second rejected, t = argmax p_2 = 0
    n, t, _ = sampling.accept_and_resample_from_logits(zp, zq, [1, 1], [0.99, 0.01], 0.5, 0.0)
    assert (n, t) == (1, 0)
    n, t, _ = sampling.accept_and_resample_from_logits(zp, np.array([[0., 1., 0.], [9., 0., 0.]]), [1, 0], [0.99, 0.99], 0.5, 0.0)
    assert (n, t) == (2, 2)


def test_lenient_alpha_formula_against_enumeration():
    """Appendix A.5: with lenience l the acceptance rate is sum min(p/l, q)."""
    l = 0.5
    acc = 0
    gd, gr = grid(8), grid(32)
    p_rows = np.array([P1, P1])
    for d, r in itertools.product(gd, gr):
        x = sampling.icdf(Q1, d)
        n, _, _ = sampling.accept_and_resample(p_rows, np.array([Q1]), [x], [r], 0.5, lenience=l)
        acc += n
    assert abs(acc / (len(gd) * len(gr)) - analysis.lenient_alpha(P1, Q1, l)) < 1e-12


def test_lenient_output_distribution_closed_form_and_bound():
    """Appendix A.5: with lenience l no token comes out with more than p(x)/l.  By exact
    enumeration over (draft draw, test uniform, final draw) the one-guess output
    distribution is min(q, p/l) + (1 - alpha_l) * max(0, p - l q) / (1 - l alpha_l)."""
    for l in (0.5, 0.25):
        p, q = np.array(P1), np.array(Q1)
        gd, gr, gs = grid(8), grid(64), grid(512)
        counts = np.zeros(4)
        p_rows = np.array([P1, P1])
        for d, r in itertools.product(gd, gr):
            x = sampling.icdf(Q1, d)
            n, _, _ = sampling.accept_and_resample(p_rows, np.array([Q1]), [x], [r], 0.5, lenience=l)
            if n == 1:
                counts[x] += len(gs)
            else:
                for sv in gs:
                    _, t, _ = sampling.accept_and_resample(p_rows, np.array([Q1]), [x], [r], sv, lenience=l)
                    counts[t] += 1
        out = counts / (len(gd) * len(gr) * len(gs))
        alpha = analysis.lenient_alpha(P1, Q1, l)
        closed = np.minimum(q, p / l) + (1 - alpha) * np.maximum(0, p - l * q) / (1 - l * alpha)
        # the final-draw grid resolves the residual only to 1/512 per reject case
        np.testing.assert_allclose(out, closed, atol=2e-3)
        assert abs(out.sum() - 1) < 1e-12
        assert np.all(out <= p / l + 2e-3) and np.all(closed <= p / l + 1e-15)


def test_argmax_lenience_special_cases():
    """Appendix A.5, temperature 0: l = 1 is the exact argmax test (no ties), a tiny l
    keeps every guess, kept guesses grow as l shrinks, and a hand-worked row."""
    rng = np.random.default_rng(5)
    for _ in range(50):
        zp = rng.normal(0, 2, size=(4, 9))
        zq = rng.normal(0, 2, size=(3, 9))
        x = [int(np.argmax(zq[i])) if rng.random() < 0.5 else int(np.argmax(zp[i])) for i in range(3)]
        n1, t1, _ = sampling.accept_and_resample_from_logits(zp, zq, x, [0.5] * 3, 0.5, 0.0)
        n2, t2 = sampling.accept_and_resample_argmax_lenient(zp, x, 1.0)
        assert (n1, t1) == (n2, t2)
        ns = [sampling.accept_and_resample_argmax_lenient(zp, x, l)[0] for l in (1.0, 0.5, 0.1, 1e-3, 1e-30)]
        assert ns == sorted(ns) and ns[-1] == 3
    # softmax([0, ln 2, ln 4]) = [1/7, 2/7, 4/7]: token 1 has half the top probability
    z = np.log(np.array([[1.0, 2.0, 4.0], [1.0, 1.0, 8.0]]))
    assert sampling.accept_and_resample_argmax_lenient(z, [1], 0.51) == (0, 2)
    assert sampling.accept_and_resample_argmax_lenient(z, [1], 0.49) == (1, 2)
    assert sampling.accept_and_resample_argmax_lenient(z, [0], 0.26) == (0, 2)
    assert sampling.accept_and_resample_argmax_lenient(z, [0], 0.24) == (1, 2)


def test_top_k_and_nucleus_standardisation():
    """Section 2.2: top-k and nucleus sampling as plain sampling from an adjusted distribution.
    Hand-worked dyadic rows, reductions to argmax / plain sampling, and a brute-force
    restatement (smallest prefix of the descending order whose mass reaches top_p)."""
    z = np.log(np.array([1 / 2, 1 / 4, 1 / 8, 1 / 8]))
    np.testing.assert_allclose(sampling.standardise(z, 1.0, top_k=2), [2 / 3, 1 / 3, 0, 0], atol=1e-15)
    np.testing.assert_allclose(sampling.standardise(z, 1.0, top_k=3), [1 / 2, 1 / 4, 1 / 8, 1 / 8], atol=1e-15)  # tie kept
    np.testing.assert_allclose(sampling.standardise(z, 1.0, top_p=0.4), [1, 0, 0, 0], atol=1e-15)
    np.testing.assert_allclose(sampling.standardise(z, 1.0, top_p=0.7), [2 / 3, 1 / 3, 0, 0], atol=1e-15)
    np.testing.assert_allclose(sampling.standardise(z, 1.0, top_p=0.8), [1 / 2, 1 / 4, 1 / 8, 1 / 8], atol=1e-15)
    # top-k first, nucleus on what is left: {1/2, 1/4} -> {2/3, 1/3}; 0.6 needs only the first
    np.testing.assert_allclose(sampling.standardise(z, 1.0, top_k=2, top_p=0.6), [1, 0, 0, 0], atol=1e-15)
    np.testing.assert_allclose(sampling.standardise(z, 1.0, top_k=2, top_p=0.7), [2 / 3, 1 / 3, 0, 0], atol=1e-15)
    rng = np.random.default_rng(11)
    for _ in range(40):
        v = int(rng.integers(5, 60))
        z = rng.normal(0, 2.5, size=v)
        T = float(rng.choice([0.5, 1.0, 1.7]))
        plain = sampling.standardise(z, T)
        np.testing.assert_array_equal(sampling.standardise(z, T, top_k=v + 3), plain)
        np.testing.assert_array_equal(sampling.standardise(z, T, top_p=1.0), plain)
        np.testing.assert_array_equal(sampling.standardise(z, T, top_k=1), sampling.standardise(z, 0.0))
        np.testing.assert_array_equal(sampling.standardise(z, T, top_p=1e-9), sampling.standardise(z, 0.0))
        k = int(rng.integers(1, v + 1))
        top_p = float(rng.uniform(0.05, 0.95))
        # brute force, top-k: exactly the k largest survive, with their softmax ratios
        got = sampling.standardise(z, T, top_k=k)
        keep = sorted(range(v), key=lambda i: -z[i])[:k]
        want = np.zeros(v); want[keep] = plain[keep] / plain[keep].sum()
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=0)
        # brute force, nucleus: grow the set one token at a time in descending probability
        got = sampling.standardise(z, T, top_p=top_p)
        order = sorted(range(v), key=lambda i: -plain[i])
        mass, m = 0.0, 0
        while mass < top_p:
            mass += plain[order[m]]; m += 1
        if sampling.nucleus_margin(z, T, 0, top_p) > 1e-9:
            want = np.zeros(v); want[order[:m]] = plain[order[:m]] / plain[order[:m]].sum()
            np.testing.assert_allclose(got, want, rtol=1e-12, atol=0)


def test_speculative_sampling_with_top_k_is_distributed_as_the_adjusted_p():
    """Section 2.2 + appendix A.1: with the same standardisation applied to both models the
    one-guess output is distributed as the standardised p (exact enumeration)."""
    mp, mq = table_models()
    want = sampling.standardise(np.log(np.array(P1)), 1.0, top_k=2)      # {5/16, 7/16} renormalised
    np.testing.assert_allclose(want, [0, 5 / 12, 0, 7 / 12], atol=1e-15)
    counts = np.zeros(4)
    gd, gr, gs = grid(12), grid(8), grid(8)
    for d, r, sv in itertools.product(gd, gr, gs):
        out, n, _ = decode.speculative_decoding_step(mp, mq, [0], 1, 1.0, [d, r, sv], top_k=2)
        counts[out[1]] += 1
    # q keeps {1/2, 1/4} -> {2/3, 1/3} (draw threshold 8/12); token 0 is always dropped, token 1 always
    # kept; the residual {0, 1/12, 0, 7/12} normalises to {0, 1/8, 0, 7/8} (threshold 1/8)
    np.testing.assert_allclose(counts / counts.sum(), want, atol=1e-12)


def test_table_drafts_leave_the_output_distribution_at_p():
    """Section 3.6: a unigram or bigram table as the approximation model.  Whatever q is, the
    first emitted token is distributed as p_1 and (given it was a kept guess) the second as
    p_2 (appendix A.1); the acceptance rate is sum min(p, q) of the table row (Cor. 3.6)."""
    mp, _ = table_models()
    with np.errstate(divide="ignore"):
        bigram = drafts.TableDraft(np.log(np.array([Q2[0], Q2[1], Q2[2], Q2[3]])), row_of=[0, 1, 2, 3])
        unigram = drafts.TableDraft(np.log(np.array([Q1])))
    np.testing.assert_array_equal(unigram.score([2, 0, 3], 2), np.log(np.array([Q1, Q1])))
    with np.errstate(divide="ignore"):
        np.testing.assert_array_equal(bigram.score([2, 0, 3], 2), np.log(np.array([Q2[0], Q2[3]])))
    gd, gr, gs = grid(8), grid(16), grid(24)        # thresholds: draws k/8, tests 3/8 and 1/2, residual 1/6 and 1/8
    # unigram, one guess: output ~ P1, acceptance rate = sum min(P1, Q1)
    counts, kept = np.zeros(4), 0
    for d, r, sv in itertools.product(gd, gr, gs):
        out, n, _ = decode.speculative_decoding_step(mp, unigram, [0], 1, 1.0, [d, r, sv])
        counts[out[1]] += 1
        kept += n
    np.testing.assert_allclose(counts / counts.sum(), P1, atol=1e-12)
    assert abs(kept / counts.sum() - sampling.beta(P1, Q1)) < 1e-12
    # bigram (context token 0 -> row Q2[0] = [1/2, 1/2, 0, 0]), target P1: output ~ P1 again
    counts = np.zeros(4)
    for d, r, sv in itertools.product(grid(2), gr, gs):
        out, n, _ = decode.speculative_decoding_step(mp, bigram, [0], 1, 1.0, [d, r, sv])
        counts[out[1]] += 1
    np.testing.assert_allclose(counts / counts.sum(), P1, atol=1e-12)


def test_copy_draft_match_rule_on_worked_contexts():
    """Section 3.6, copying model: the last `match` tokens are looked up among their earlier
    occurrences, the most recent one that has a successor wins (contexts worked by hand)."""
    two = drafts.CopyDraft(8, 2)
    assert two.copied_token([5, 6, 7, 5, 6]) == 7
    assert two.copied_token([1, 2, 3, 1, 2, 4, 1, 2]) == 4          # occurrences at 0 (-> 3) and 3 (-> 4)
    assert two.copied_token([7, 7, 7]) == 7                          # overlapping occurrence at 0
    assert two.copied_token([7, 7]) is None                          # only the tail itself
    assert two.copied_token([1, 2, 3, 2, 1]) is None
    assert two.copied_token([4]) is None
    one = drafts.CopyDraft(8, 1)
    assert one.copied_token([3, 5, 3, 6, 3]) == 6
    rows = two.score([5, 6, 7, 5, 6], 2)                             # contexts [5,6,7,5] and [5,6,7,5,6]
    np.testing.assert_array_equal(rows[0], np.zeros(8))              # (7,5) never seen: uniform
    assert rows[1][7] == 0.0 and np.all(np.isneginf(np.delete(rows[1], 7)))


def test_copy_draft_leaves_the_output_distribution_at_p():
    """A one-hot q on token x keeps x with probability p(x) (Cor. 3.6: sum min(p, q) = p(x)) and
    otherwise draws from p with x removed, so the output is distributed as p (appendix A.1)."""
    mp = TableScorer(lambda ctx: P2[ctx[-1]])
    copy = drafts.CopyDraft(4, 2)
    prefix = [0, 3, 1, 0, 3]                                         # copied guess 1; p = P2[3] = [1/8, 3/8, 1/4, 1/4]
    counts, kept = np.zeros(4), 0
    for d, r, sv in itertools.product(grid(2), grid(8), grid(10)):  # test threshold 3/8; residual [1/5, 0, 2/5, 2/5]
        out, n, info = decode.speculative_decoding_step(mp, copy, prefix, 1, 1.0, [d, r, sv])
        assert info["x"] == [1]
        counts[out[len(prefix)]] += 1
        kept += n
    np.testing.assert_allclose(counts / counts.sum(), P2[3], atol=1e-12)
    assert abs(kept / counts.sum() - 3 / 8) < 1e-12
    # no earlier occurrence: the uniform model, acceptance rate sum min(p, 1/4)
    counts, kept = np.zeros(4), 0
    for d, r, sv in itertools.product(grid(4), grid(8), grid(8)):
        out, n, _ = decode.speculative_decoding_step(mp, copy, [0, 1, 2], 1, 1.0, [d, r, sv])
        counts[out[3]] += 1
        kept += n
    np.testing.assert_allclose(counts / counts.sum(), P2[2], atol=1e-12)
    assert abs(kept / counts.sum() - sampling.beta(P2[2], [1 / 4] * 4)) < 1e-12
    # ... or the fallback model when one is given
    with np.errstate(divide="ignore"):
        bigram = drafts.TableDraft(np.log(np.array([Q2[0], Q2[1], Q2[2], Q2[3]])), row_of=[0, 1, 2, 3])
    both = drafts.CopyDraft(4, 2, fallback=bigram)
    with np.errstate(divide="ignore"):
        np.testing.assert_array_equal(both.score([0, 1, 2], 1)[0], np.log(np.array(Q2[2])))
    assert both.score([0, 3, 1, 0, 3], 1)[0][1] == 0.0


def test_copy_draft_on_a_periodic_target_keeps_every_guess():
    """Closed form: when Mp continues a cycle with certainty and the context already holds one
    period, every copied guess is Mp's own token, so each run of Algorithm 1 emits gamma + 1
    tokens (the guesses extend the context they are matched in)."""
    with np.errstate(divide="ignore"):
        mp = TableScorer(lambda ctx: [1.0 if t == (ctx[-1] + 1) % 4 else 0.0 for t in range(4)])
        copy = drafts.CopyDraft(4, 2)
        for T in (0.0, 1.0):
            rng = np.random.default_rng(5)
            rows = (rng.uniform(0.01, 0.99, 7) for _ in range(10))
            toks, recs = decode.speculative_decode(mp, copy, [0, 1, 2, 3, 0, 1], 12, 3, T, rows)
            assert toks[6:] == [(2 + i) % 4 for i in range(12)]
            assert [n for n, _, _ in recs] == [3, 3, 3]


def test_uniform_validation():
    mp, mq = table_models()
    with pytest.raises(ValueError):
        decode.speculative_decoding_step(mp, mq, [0], 1, 1.0, [0.0, 0.5, 0.5])
    with pytest.raises(ValueError):
        decode.speculative_decoding_step(mp, mq, [0], 2, 1.0, [0.5, 0.5, 0.5])


def test_icdf_edge_distance_on_hand_worked_cdfs():
    """The helper that decides which draw disagreements the GPU tests excuse.  Weights (1, 1, 2)
    have the CDF edges 0.25, 0.5, 1: token 1 owns [0.25, 0.5)."""
    w = [1.0, 1.0, 2.0]
    assert sampling.icdf_edge_distance(w, 0.3, 1) == pytest.approx(0.05)      # nearer edge 0.25
    assert sampling.icdf_edge_distance(w, 0.45, 1) == pytest.approx(0.05)     # nearer edge 0.5
    assert sampling.icdf_edge_distance(w, 0.2, 0) == pytest.approx(0.05)      # token 0: edges 0 and 0.25
    assert sampling.icdf_edge_distance(w, 0.9, 2) == pytest.approx(0.1)
    assert sampling.icdf_edge_distance([4.0, 4.0, 8.0], 0.3, 1) == pytest.approx(0.05)   # scale-free
    # a zero-weight token has an empty interval: its distance is the distance to that single edge
    assert sampling.icdf_edge_distance([1.0, 0.0, 1.0], 0.6, 1) == pytest.approx(0.1)
    # meaning: moving u by more than the distance towards the nearer edge changes the drawn token,
    # moving it by less does not
    rng = np.random.default_rng(5)
    for _ in range(200):
        w = rng.random(9) + 0.01
        u = float(rng.random() * 0.98 + 0.01)
        k = sampling.icdf(w, u)
        d = sampling.icdf_edge_distance(w, u, k)
        c = np.concatenate([[0.0], np.cumsum(w) / np.sum(w)])
        assert c[k] <= u < c[k + 1] and d == pytest.approx(min(u - c[k], c[k + 1] - u))
        towards = -1.0 if (u - c[k]) <= (c[k + 1] - u) else 1.0
        assert sampling.icdf(w, u + towards * 0.5 * d) == k
        moved = u + towards * (d + 1e-9)
        if 0.0 < moved < 1.0:
            assert sampling.icdf(w, moved) != k


def test_nucleus_margin_on_hand_worked_rows():
    """The helper that recognises rows whose nucleus could legitimately come out differently in
    fp32.  Probabilities (0.5, 0.3, 0.2): the descending cumulative mass passes 0.5, 0.8, 1."""
    z = np.log([0.3, 0.5, 0.2])
    assert sampling.nucleus_margin(z, 1.0, 0, 0.75) == pytest.approx(0.05)    # |0.8 - 0.75|
    assert sampling.nucleus_margin(z, 1.0, 0, 0.55) == pytest.approx(0.05)    # |0.5 - 0.55|
    assert sampling.nucleus_margin(z, 1.0, 0, 0.8) == pytest.approx(0.0, abs=1e-15)
    # after top-2 the masses are 0.625, 0.375: cumulative 0.625, 1
    assert sampling.nucleus_margin(z, 1.0, 2, 0.6) == pytest.approx(0.025)
    # temperature 0.5 squares the probabilities: (0.25, 0.09, 0.04) / 0.38
    assert sampling.nucleus_margin(z, 0.5, 0, 0.9) == pytest.approx(abs(0.34 / 0.38 - 0.9))
    # meaning: the kept set of standardise() changes exactly where the margin reaches zero
    kept = lambda top_p: int(np.count_nonzero(sampling.standardise(z, 1.0, 0, top_p)))
    assert (kept(0.8 - 1e-9), kept(0.8 + 1e-9)) == (2, 3)
    assert (kept(0.5 - 1e-9), kept(0.5 + 1e-9)) == (1, 2)
    for top_p in (0.3, 0.6, 0.79, 0.81, 0.95):
        m = sampling.nucleus_margin(z, 1.0, 0, top_p)
        assert m > 0 and kept(top_p - 0.5 * m) == kept(top_p) == kept(top_p + 0.5 * m)
