"""GPU parity: the fused accept / resample kernel against the oracle's
Algorithm-1 arithmetic on the same seeded logits, guesses and uniforms.

Bar: n and t bit-exact, except acceptance decisions with |r - p/q| < 1e-3 and
draws whose uniform lies within 1e-5 (normalised CDF units) of an edge of the
chosen token's CDF interval; such tolerated events are counted and must be rare.
"""
import numpy as np
import pytest
import torch

from oracle import sampling
from paper_2211_17192_amd import synth

pytestmark = pytest.mark.gpu


def run_case(rows, gamma, vocab, sigma, seed, temperature):
    from paper_2211_17192_amd import binding
    zp, zq, x, r, s = synth.sampler_case(rows, gamma, vocab, sigma, seed)
    dev = "cuda"
    n_d, t_d = binding.spec_sample(torch.from_numpy(zp).to(dev), torch.from_numpy(zq).to(dev),
                                   torch.from_numpy(x).to(dev), torch.from_numpy(r).to(dev),
                                   torch.from_numpy(s).to(dev), temperature)
    torch.cuda.synchronize()
    n_g, t_g = n_d.cpu().numpy(), t_d.cpu().numpy()
    tolerated = 0
    for b in range(rows):
        if temperature == 0:
            xb = [int(np.argmax(zq[b, i])) for i in range(gamma)]      # x_i ~ one-hot q_i
        else:
            xb = list(x[b])
        n_o, t_o, info = sampling.accept_and_resample_from_logits(zp[b], zq[b], xb, r[b], s[b], temperature)
        if temperature == 0:
            continue_check = True
        if (n_g[b], t_g[b]) == (n_o, t_o):
            continue
        # a tolerated disagreement must be explained by a near-threshold decision
        if n_g[b] != n_o:
            first = min(n_g[b], n_o)
            assert info["margins"][first] < 1e-3, (b, n_g[b], n_o, info["margins"])
        else:
            p_rows = np.stack([sampling.standardise(z, temperature) for z in zp[b]])
            q_rows = np.stack([sampling.standardise(z, temperature) for z in zq[b]])
            w = p_rows[n_o] if n_o == gamma else sampling.adjusted_distribution(p_rows[n_o], q_rows[n_o])
            assert sampling.icdf_edge_distance(w, s[b], int(t_g[b])) < 1e-5, (b, t_g[b], t_o)
        tolerated += 1
    return tolerated, n_g


@pytest.mark.parametrize("sigma", [0.5, 1.0, 2.0])
def test_spec_sample_matches_oracle_full_vocab(sigma):
    """The isolated-sampler workload as configured: 64 independent rows, vocabulary 32128,
    gamma = 7, target logits N(0, 3^2), draft = target + N(0, sigma^2), through plain
    sd_spec_sample (64 x 15 statistics workgroups, then one tail workgroup per row)."""
    tol, n = run_case(64, 7, 32128, sigma, seed=int(sigma * 10), temperature=1.0)
    assert tol <= 2
    assert n.min() >= 0 and n.max() <= 7
    print(f"sigma {sigma}: mean accepted {n.mean():.2f} of 7, tolerated {tol}")


@pytest.mark.parametrize("rows,gamma,vocab,temperature", [
    (5, 1, 256, 1.0), (3, 4, 50, 1.0), (4, 15, 1000, 0.7), (2, 3, 4099, 2.0),   # ragged / odd vocab
    (6, 5, 8192, 0.0), (3, 7, 32128, 0.0),
])
def test_spec_sample_shapes_and_temperatures(rows, gamma, vocab, temperature):
    if temperature == 0.0:
        from paper_2211_17192_amd import binding
        zp, zq, x, r, s = synth.sampler_case(rows, gamma, vocab, 0.5, 3)
        xg = np.argmax(zq, axis=-1).astype(np.int32)
        n_d, t_d = binding.spec_sample(torch.from_numpy(zp).cuda(), torch.from_numpy(zq).cuda(),
                                       torch.from_numpy(xg).cuda(), torch.from_numpy(r).cuda(),
                                       torch.from_numpy(s).cuda(), 0.0)
        for b in range(rows):
            n_o, t_o, _ = sampling.accept_and_resample_from_logits(zp[b], zq[b], list(xg[b]), r[b], s[b], 0.0)
            assert (int(n_d[b]), int(t_d[b])) == (n_o, t_o)
    else:
        tol, _ = run_case(rows, gamma, vocab, 1.0, 11, temperature)
        assert tol <= 1


def test_spec_sample_degenerate_inputs():
    """q == p keeps every guess; a guess the target gives (almost) no mass is dropped
    and the residual draw can never return it when q > p there."""
    from paper_2211_17192_amd import binding
    rows, gamma, V = 4, 3, 512
    zp, _, _, r, s = synth.sampler_case(rows, gamma, V, 1.0, 5)
    zq = zp[:, :gamma].copy()
    x = np.argmax(zq, axis=-1).astype(np.int32)
    n_d, t_d = binding.spec_sample(torch.from_numpy(zp).cuda(), torch.from_numpy(zq).cuda(),
                                   torch.from_numpy(x).cuda(), torch.from_numpy(r).cuda(),
                                   torch.from_numpy(s).cuda(), 1.0)
    assert n_d.cpu().tolist() == [gamma] * rows
    for b in range(rows):
        assert int(t_d[b]) == sampling.icdf(sampling.standardise(zp[b, gamma], 1.0), s[b])
    # second scenario: the first guess has target probability ~ e^-60 -> rejected at once
    zp2 = zp.copy()
    for b in range(rows):
        zp2[b, 0, x[b, 0]] = -60.0
    n_d, t_d = binding.spec_sample(torch.from_numpy(zp2).cuda(), torch.from_numpy(zq).cuda(),
                                   torch.from_numpy(x).cuda(), torch.from_numpy(r).cuda(),
                                   torch.from_numpy(s).cuda(), 1.0)
    assert n_d.cpu().tolist() == [0] * rows
    assert all(int(t_d[b]) != x[b, 0] for b in range(rows))


def test_spec_sample_rejects_bad_arguments():
    from paper_2211_17192_amd import binding
    assert binding.lib.sd_spec_sample_scratch_bytes(0, 3) == 0
    assert binding.lib.sd_spec_sample_scratch_bytes(4, 16) == 0
    z = torch.zeros(1, 2, 8, device="cuda")
    with pytest.raises(binding.SdError):
        binding.spec_sample(z, z[:, :1].contiguous(), torch.zeros(1, 1, dtype=torch.int32, device="cuda"),
                            None, None, 1.0)


@pytest.mark.parametrize("rows,gamma,vocab,lenience,sigma", [
    (16, 7, 32128, 0.5, 1.0), (70, 5, 32128, 0.3, 2.0), (6, 4, 4099, 0.1, 2.0), (3, 3, 257, 1.0, 1.0),
])
def test_lenient_acceptance_and_beta_match_oracle(rows, gamma, vocab, lenience, sigma):
    """Appendix A.5 in the kernel: test r <= p/(l q), residual max(0, p - l q), and the
    side output beta_i = sum_x min(p_i/l, q_i).  70 rows take the two-launch path."""
    from oracle import analysis
    from paper_2211_17192_amd import binding
    zp, zq, x, r, s = synth.sampler_case(rows, gamma, vocab, sigma, 21)
    beta = torch.full((rows, gamma), -1.0, device="cuda")
    n_d, t_d = binding.spec_sample(torch.from_numpy(zp).cuda(), torch.from_numpy(zq).cuda(),
                                   torch.from_numpy(x).cuda(), torch.from_numpy(r).cuda(),
                                   torch.from_numpy(s).cuda(), 1.0, lenience=lenience, beta=beta)
    torch.cuda.synchronize()
    n_g, t_g, beta_g = n_d.cpu().numpy(), t_d.cpu().numpy(), beta.cpu().numpy()
    l64 = float(np.float32(lenience))
    tolerated, more_kept = 0, 0
    for b in range(rows):
        p_rows = np.stack([sampling.standardise(z, 1.0) for z in zp[b]])
        q_rows = np.stack([sampling.standardise(z, 1.0) for z in zq[b]])
        n_o, t_o, info = sampling.accept_and_resample(p_rows, q_rows, list(x[b]), r[b], s[b], lenience=l64)
        n_strict, _, _ = sampling.accept_and_resample(p_rows, q_rows, list(x[b]), r[b], s[b])
        more_kept += n_o - n_strict
        for i in range(gamma):
            want = analysis.lenient_alpha(p_rows[i], q_rows[i], l64)
            assert abs(beta_g[b, i] - want) <= 2e-6 * max(want, 1e-3), (b, i, beta_g[b, i], want)
        if (n_g[b], t_g[b]) == (n_o, t_o):
            continue
        if n_g[b] != n_o:
            assert info["margins"][min(n_g[b], n_o)] < 1e-3
        else:
            w = p_rows[n_o] if n_o == gamma else sampling.adjusted_distribution(p_rows[n_o], l64 * q_rows[n_o])
            assert sampling.icdf_edge_distance(w, s[b], int(t_g[b])) < 1e-5
        tolerated += 1
    assert tolerated <= 1
    if lenience < 1.0:
        assert more_kept > 0            # the relaxed test really keeps more guesses on these inputs


@pytest.mark.parametrize("lenience", [0.5, 0.05])
def test_lenient_argmax_sampling_matches_oracle(lenience):
    """Temperature 0 with lenience: keep x_i iff z[x_i] - max z >= ln l (double), t = argmax."""
    from paper_2211_17192_amd import binding
    rows, gamma, vocab = 12, 6, 8192
    zp, zq, _, r, s = synth.sampler_case(rows, gamma, vocab, 3.0, 33)
    xg = np.argmax(zq, axis=-1).astype(np.int32)
    beta = torch.full((rows, gamma), -1.0, device="cuda")
    n_d, t_d = binding.spec_sample(torch.from_numpy(zp).cuda(), torch.from_numpy(zq).cuda(),
                                   torch.from_numpy(xg).cuda(), torch.from_numpy(r).cuda(),
                                   torch.from_numpy(s).cuda(), 0.0, lenience=lenience, beta=beta)
    torch.cuda.synchronize()
    kept = 0
    for b in range(rows):
        n_o, t_o = sampling.accept_and_resample_argmax_lenient(zp[b], list(xg[b]), lenience)
        assert (int(n_d[b]), int(t_d[b])) == (n_o, t_o)
        kept += n_o
        for i in range(gamma):      # beta of a one-hot q: 1 if its token passes the test, else 0
            ok = sampling.accept_and_resample_argmax_lenient(zp[b, i:i + 2], [int(xg[b, i])], lenience)[0] == 1
            assert float(beta[b, i]) == (1.0 if ok else 0.0)
    assert 0 < kept < rows * gamma


@pytest.mark.parametrize("rows,gamma,vocab,temperature,top_k,top_p", [
    (16, 5, 32128, 1.0, 40, 0.0), (16, 5, 32128, 1.0, 0, 0.9), (70, 3, 32128, 0.7, 50, 0.8),
    (8, 4, 4096, 1.0, 1, 0.0), (8, 4, 1000, 1.3, 0, 0.5), (4, 2, 256, 1.0, 300, 0.999),
])
def test_top_k_and_nucleus_match_oracle(rows, gamma, vocab, temperature, top_k, top_p):
    """Section 2.2 standardisation with top-k / nucleus inside the kernel, the same for p and q
    rows: n, t and beta against the oracle.  The guesses are drawn from the filtered q, as
    Algorithm 1 does.  Rows whose nucleus boundary lies within 1e-5 of top_p (fp32 vs fp64
    exponentials may then choose different sets) are skipped and counted."""
    from paper_2211_17192_amd import binding
    zp, zq, _, r, s = synth.sampler_case(rows, gamma, vocab, 1.0, 44)
    # peaked rows (logit std 7.5): with flatter ones the tokens at a nucleus boundary carry ~1e-5
    # of the mass each over 32128 entries, and most boundaries would sit inside the skip margin
    zp, zq = (zp * np.float32(2.5)).astype(np.float32), (zq * np.float32(2.5)).astype(np.float32)
    tp = float(np.float32(top_p))
    d = synth.uniform_stream(45, rows * gamma).reshape(rows, gamma)
    q_rows = [[sampling.standardise(zq[b, i], temperature, top_k, tp) for i in range(gamma)] for b in range(rows)]
    x = np.array([[sampling.icdf(q_rows[b][i], d[b, i]) for i in range(gamma)] for b in range(rows)], dtype=np.int32)
    beta = torch.full((rows, gamma), -1.0, device="cuda")
    n_d, t_d = binding.spec_sample(torch.from_numpy(zp).cuda(), torch.from_numpy(zq).cuda(),
                                   torch.from_numpy(x).cuda(), torch.from_numpy(r).cuda(),
                                   torch.from_numpy(s).cuda(), temperature, beta=beta, top_k=top_k, top_p=top_p)
    torch.cuda.synchronize()
    n_g, t_g, beta_g = n_d.cpu().numpy(), t_d.cpu().numpy(), beta.cpu().numpy()
    skipped, tolerated, rejected = 0, 0, 0
    for b in range(rows):
        if 0.0 < tp < 1.0:
            margin = min(sampling.nucleus_margin(z, temperature, top_k, tp) for z in list(zp[b]) + list(zq[b]))
            if margin < 1e-5:
                skipped += 1
                continue
        p_rows = np.stack([sampling.standardise(z, temperature, top_k, tp) for z in zp[b]])
        qr = np.stack(q_rows[b])
        n_o, t_o, info = sampling.accept_and_resample(p_rows, qr, list(x[b]), r[b], s[b])
        rejected += int(n_o < gamma)
        for i in range(gamma):
            want = sampling.beta(p_rows[i], qr[i])
            assert abs(beta_g[b, i] - want) <= 2e-6 * max(want, 1e-3), (b, i, beta_g[b, i], want)
        if (n_g[b], t_g[b]) == (n_o, t_o):
            continue
        if n_g[b] != n_o:
            assert info["margins"][min(n_g[b], n_o)] < 1e-3
        else:
            w = p_rows[n_o] if n_o == gamma else sampling.adjusted_distribution(p_rows[n_o], qr[n_o])
            assert sampling.icdf_edge_distance(w, s[b], int(t_g[b])) < 1e-5
        tolerated += 1
    assert tolerated <= 1 and skipped <= rows // 4
    if top_k != 1:
        assert rejected > 0


def test_filters_refuse_vocabularies_they_cannot_hold():
    from paper_2211_17192_amd import binding
    z = torch.zeros(1, 2, 40000, device="cuda")
    with pytest.raises(binding.SdError):
        binding.spec_sample(z, z[:, :1].contiguous(), torch.zeros(1, 1, dtype=torch.int32, device="cuda"),
                            torch.full((1, 1), 0.5, device="cuda"), torch.full((1,), 0.5, device="cuda"), 1.0, top_k=5)
    z = torch.zeros(1, 2, 1001, device="cuda")
    with pytest.raises(binding.SdError):
        binding.spec_sample(z, z[:, :1].contiguous(), torch.zeros(1, 1, dtype=torch.int32, device="cuda"),
                            torch.full((1, 1), 0.5, device="cuda"), torch.full((1,), 0.5, device="cuda"), 1.0, top_p=0.5)
