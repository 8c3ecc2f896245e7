"""Pins for the oracle's drafting step and for the outer loop (Alg. 3) built on the oracle, against what
the paper and the mathematics fix for context-independent toy models (Sec. 2)."""
from __future__ import annotations

import itertools

import numpy as np
import scipy.special

import oracle
import workloads
from tests import toy_loop

PAPER_MB = np.array([1 / 3, 2 / 3])       # eq. (toy models): M_b(a), M_b(b)
PAPER_MS = np.array([2 / 3, 1 / 3])       # M_s(a), M_s(b)


def test_sample_rows_is_the_inverse_cdf_of_the_softmax():
    rng = np.random.default_rng(5)
    for V, T in ((1, 1.0), (2, 0.7), (17, 1.3), (1000, 0.8)):
        logits = (rng.standard_normal((64, V)) * 3).astype(np.float32)
        u = workloads.philox_uniforms(77 + V, (64,))
        tok, margins = oracle.sample_rows(logits, u, T)
        p = scipy.special.softmax(logits.astype(np.float64) / T, axis=1)
        cdf = np.cumsum(p, axis=1)
        want = np.array([np.searchsorted(cdf[r], u[r] * cdf[r, -1], side="right") for r in range(64)])
        want = np.minimum(want, V - 1)
        safe = margins > 1e-9
        assert safe.mean() > 0.9
        assert np.array_equal(tok[safe], want[safe])


def test_sample_rows_extremes_and_bf16():
    logits = np.array([[0.0, -np.inf if False else -80.0, 1.0, -80.0]], dtype=np.float32)   # tokens 1, 3 have weight ~1e-35
    tok, _ = oracle.sample_rows(logits, np.array([0.0], dtype=np.float32), 1.0)
    assert tok[0] == 0                       # u = 0 takes the first token of positive weight
    tok, _ = oracle.sample_rows(logits, np.array([1.0 - 2.0 ** -24], dtype=np.float32), 1.0)
    assert tok[0] == 2                       # u -> 1 takes the last token that carries mass at this resolution
    # bf16 rows are upcast exactly: same draw as the float32 row holding the same values
    rng = np.random.default_rng(6)
    f = (rng.standard_normal((32, 50)) * 2).astype(np.float32)
    bits = (f.view(np.uint32) >> 16).astype(np.uint16)
    f_exact = (bits.astype(np.uint32) << 16).view(np.float32)
    u = workloads.philox_uniforms(3, (32,))
    a, _ = oracle.sample_rows(bits, u, 0.9, dtype=oracle.BF16)
    b, _ = oracle.sample_rows(f_exact, u, 0.9)
    assert np.array_equal(a, b)


def test_sample_rows_frequencies_follow_the_distribution():
    logits = np.log(np.array([0.5, 0.25, 0.125, 0.125]))[None, :].repeat(40000, axis=0).astype(np.float32)
    tok, _ = oracle.sample_rows(logits, workloads.philox_uniforms(11, (40000,)), 1.0)
    freq = np.bincount(tok, minlength=4) / 40000
    assert np.abs(freq - [0.5, 0.25, 0.125, 0.125]).max() < 0.01


def _loop(algo, gamma, B=4096, iters=50, seed=1):
    return toy_loop.oracle_loop(algo, np.log(PAPER_MB), np.log(PAPER_MS), gamma, B, iters, 1.0, seed)


def test_paper_toy_expected_accepted_tokens_gamma_2():
    # Sec. 2: E[tau] = 10/9 under token verification, 11/9 under block verification (gamma = 2)
    n = 4096 * 50
    for algo, want in (("token", 10 / 9), ("block", 11 / 9)):
        tau = _loop(algo, 2)["tau"]
        assert abs(tau.mean() - want) < 4.0 / np.sqrt(n), (algo, tau.mean())


def _exact_ccdf_block(gamma):
    # Pr(tau >= k) = E_{X^k ~ M_s} w_k(X^k), w_k = min(w_{k-1} M_b(X_k)/M_s(X_k), 1)  (Lemma on the acceptance
    # probability of a sub-block); enumeration over the 2^k draft prefixes
    out = [1.0]
    for k in range(1, gamma + 1):
        total = 0.0
        for xs in itertools.product((0, 1), repeat=k):
            w, prob = 1.0, 1.0
            for x in xs:
                w = min(w * PAPER_MB[x] / PAPER_MS[x], 1.0)
                prob *= PAPER_MS[x]
            total += prob * w
        out.append(total)
    return np.array(out)


def test_paper_toy_ccdf_of_tau_gamma_10():
    # the experiment behind the paper's figure of the complementary CDF of tau (gamma = 10)
    gamma, n = 10, 4096 * 50
    token = toy_loop.ccdf(_loop("token", gamma)["tau"], gamma)
    block = toy_loop.ccdf(_loop("block", gamma)["tau"], gamma)
    exact_token = (2 / 3) ** np.arange(gamma + 1)       # each draft token survives with sum_x min(M_b, M_s) = 2/3
    exact_block = _exact_ccdf_block(gamma)
    tol = 4.0 * 0.5 / np.sqrt(n)
    assert np.abs(token - exact_token).max() < tol
    assert np.abs(block - exact_block).max() < tol
    assert np.all(exact_block >= exact_token - 1e-15) and exact_block[gamma] > exact_token[gamma]


def test_block_efficiency_grows_with_gamma_and_block_beats_token():
    be = {}
    for gamma in (4, 6, 8, 10):
        for algo in ("token", "block", "greedy"):
            be[algo, gamma] = 1.0 + _loop(algo, gamma, B=2048, iters=20)["tau"].mean()
    for algo in ("token", "block", "greedy"):
        assert be[algo, 4] < be[algo, 6] < be[algo, 8] < be[algo, 10]
    for gamma in (4, 6, 8, 10):
        assert be["block", gamma] > be["token", gamma] + 0.02
        assert be["greedy", gamma] > be["token", gamma] + 0.02
    # closed forms: token 1 + sum_k (2/3)^k; block 1 + sum_k Pr(tau >= k)
    for gamma in (4, 10):
        assert abs(be["token", gamma] - (1 + ((2 / 3) ** np.arange(1, gamma + 1)).sum())) < 0.03
        assert abs(be["block", gamma] - (1 + _exact_ccdf_block(gamma)[1:].sum())) < 0.03
