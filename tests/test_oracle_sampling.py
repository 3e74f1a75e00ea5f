"""Pins for the oracle's sampler: RNG constants, nucleus definition, limits, statistics."""
import math

import numpy as np
import pytest
import torch
from scipy import stats

from oracle import sampling as S


def test_mix64_matches_published_splitmix64_stream():
    # The splitmix64 generator seeded with 0 emits mix(0 + k*golden) for k = 1, 2, 3, ...;
    # its first outputs are widely published test vectors.
    golden = 0x9E3779B97F4A7C15
    outs = [S.mix64((k * golden) & ((1 << 64) - 1)) for k in range(3)]
    assert outs == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_uniform_is_reproducible_in_range_and_uniform():
    us = np.array([S.uniform(42, b, t) for b in range(64) for t in range(256)])
    assert us.min() >= 0.0 and us.max() < 1.0
    assert S.uniform(42, 3, 9) == S.uniform(42, 3, 9)
    assert S.uniform(42, 3, 9) != S.uniform(42, 9, 3) and S.uniform(42, 3, 9) != S.uniform(43, 3, 9)
    assert np.all(us * 2 ** 24 == np.round(us * 2 ** 24))          # exactly 24 bits
    assert stats.kstest(us, "uniform").pvalue > 1e-3
    # successive steps of one row are not correlated
    a = us.reshape(64, 256)
    assert abs(np.corrcoef(a[:, :-1].ravel(), a[:, 1:].ravel())[0, 1]) < 0.03


def _row(seed=0, V=512, scale=2.0):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(V, generator=g, dtype=torch.float64) * scale


def test_softmax_rows_sum_to_one_and_logprobs_nonpositive():
    z = _row(1)
    lsm = S.log_softmax(z)
    assert abs(float(torch.exp(lsm).sum()) - 1.0) < 1e-12
    assert (lsm <= 0).all()
    assert (lsm - torch.log_softmax(z, 0)).abs().max() < 1e-12


def test_nucleus_is_the_shortest_prefix():
    p = torch.softmax(_row(2), 0)
    for top_p in (0.1, 0.5, 0.9, 0.999):
        keep = S.nucleus(p, top_p)
        mass = float(p[keep].sum())
        smallest = float(p[keep].min())
        assert mass >= top_p - 1e-15
        assert mass - smallest < top_p                     # dropping its smallest member falls short
        assert float(p[~keep].max()) <= smallest           # nothing outside beats a member
    assert S.nucleus(p, 1.0).all()
    # hand example, crossing token included, ties broken towards the lower index
    q = torch.tensor([0.1, 0.3, 0.3, 0.2, 0.1], dtype=torch.float64)
    assert S.nucleus(q, 0.5).tolist() == [False, True, True, False, False]
    assert S.nucleus(q, 0.3).tolist() == [False, True, False, False, False]
    assert S.nucleus(q, 0.61).tolist() == [False, True, True, True, False]


def test_limits_reduce_to_greedy():
    z = _row(3)
    best = int(torch.argmax(z))
    for b in range(4):
        for t in range(4):
            assert S.sample(z, S.Sampling(temperature=1.0, top_p=1e-9, seed=7), b, t)[0] == best
            assert S.sample(z, S.Sampling(temperature=1e-4, top_p=1.0, seed=7), b, t)[0] == best
    tied = torch.tensor([0.0, 2.0, 2.0, 1.0], dtype=torch.float64)
    assert S.sample(tied, S.Sampling(greedy=True), 0, 0)[0] == 1  # lowest index among exact ties


def test_sampled_token_follows_the_cdf_by_hand():
    z = torch.log(torch.tensor([0.1, 0.2, 0.3, 0.4], dtype=torch.float64))
    s = S.Sampling(temperature=1.0, top_p=1.0)
    for u, want in ((0.0, 0), (0.0999, 0), (0.1001, 1), (0.2999, 1), (0.3001, 2), (0.61, 3), (0.9999, 3)):
        tok, lp, _ = S.sample(z, s, 0, 0, u=u)
        assert tok == want and abs(lp - math.log([0.1, 0.2, 0.3, 0.4][want])) < 1e-12
    # top_p = 0.65 keeps {3, 2} (0.4 + 0.3); renormalised to 3/7 and 4/7 in index order 2, 3
    s = S.Sampling(temperature=1.0, top_p=0.65, logprob_mode=1)
    assert S.sample(z, s, 0, 0, u=0.42)[0] == 2 and S.sample(z, s, 0, 0, u=0.43)[0] == 3
    assert abs(S.sample(z, s, 0, 0, u=0.9)[1] - math.log(4 / 7)) < 1e-12
    s0 = S.Sampling(temperature=1.0, top_p=0.65, logprob_mode=0)
    assert abs(S.sample(z, s0, 0, 0, u=0.9)[1] - math.log(0.4)) < 1e-12
    # temperature 0.5 squares the probabilities
    s = S.Sampling(temperature=0.5, top_p=1.0, logprob_mode=1)
    sq = np.array([0.01, 0.04, 0.09, 0.16]) / 0.30
    assert abs(S.sample(z, s, 0, 0, u=0.99)[1] - math.log(sq[3])) < 1e-12


def test_empirical_frequencies_match_softmax():
    z = _row(4, V=24, scale=1.0)
    p = torch.softmax(z, 0).numpy()
    s = S.Sampling(temperature=1.0, top_p=1.0, seed=123)
    n = 20000
    counts = np.zeros(24)
    for i in range(n):
        counts[S.sample(z, s, i % 64, i // 64)[0]] += 1
    assert stats.chisquare(counts, p * n).pvalue > 1e-3


def test_cdf_margin():
    z = torch.log(torch.tensor([0.25, 0.25, 0.5], dtype=torch.float64))
    tok, _, info = S.sample(z, S.Sampling(), 0, 0, u=0.3)
    assert tok == 1 and abs(S.cdf_margin(info, tok) - 0.05) < 1e-12
