"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests re-types the oracle's arithmetic to compare against itself: each
one checks a printed value, a theorem, a closed form or a library routine.
"""
from __future__ import annotations

import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle
from tests import tiny

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "toy_example.txt")


def _golden():
    vals = {}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = [s.strip() for s in line.split("=")]
            vals[k] = Fraction(v)
    return vals


def _toy(gamma):
    # Section 2: two tokens a=0, b=1, M_b = (1/3, 2/3), M_s = (2/3, 1/3), context-independent
    Mb = tiny.constant_tables([1 / 3, 2 / 3], 2, gamma)
    Ms = tiny.constant_tables([2 / 3, 1 / 3], 2, gamma)
    return Mb, Ms


def _expected_tau(law):
    return sum(m * tau for (_, tau, _), m in law.items())


def _cond(law, Ms, xs):
    """Law of (tau, Y) given the draft block xs."""
    ms = tiny.joint(Ms, xs)
    out = {}
    for (x, tau, y), m in law.items():
        if x == tuple(xs):
            out[(tau, y)] = out.get((tau, y), 0.0) + m / ms
    return out


# ---------------------------------------------------------------- printed values (Sec. 2)
def test_toy_example_token_matches_printed_values():
    g = _golden()
    Mb, Ms = _toy(2)
    law, dbg, skipped = tiny.output_law(oracle.TOKEN, Mb, Ms, 2, 2)
    assert skipped < 1e-9
    assert abs(sum(law.values()) - 1.0) < 1e-12
    assert _expected_tau(law) == pytest.approx(float(g["token_expected_tau"]), abs=1e-6)
    # per-token acceptance probabilities: h_i depends only on the token at position i
    for xs, d in dbg.items():
        for i, x in enumerate(xs, start=1):
            want = g["token_accept_a"] if x == 0 else g["token_accept_b"]
            assert d[i, 2] == pytest.approx(float(want), abs=1e-6)


def test_toy_example_block_matches_printed_values():
    g = _golden()
    Mb, Ms = _toy(2)
    law, _, skipped = tiny.output_law(oracle.BLOCK, Mb, Ms, 2, 2)
    assert skipped < 1e-9
    assert _expected_tau(law) == pytest.approx(float(g["block_expected_tau"]), abs=1e-6)
    a, b = 0, 1
    for xs, key in (((a, b), "block_accept_all_ab"), ((b, b), "block_accept_all_bb"),
                    ((a, a), "block_accept_all_aa"), ((b, a), "block_accept_all_ba")):
        c = _cond(law, Ms, xs)
        p_all = sum(m for (tau, _), m in c.items() if tau == 2)
        assert p_all == pytest.approx(float(g[key]), abs=1e-6)
    # aa rejected: nothing is kept and the correction is b
    c = _cond(law, Ms, (a, a))
    rejected = {k: m for k, m in c.items() if k[0] != 2}
    assert set(rejected) == {(int(g["block_aa_rejected_tau"]), int(g["block_aa_rejected_Y"]))}
    # ba: b is always kept; when a is dropped the correction is b
    c = _cond(law, Ms, (b, a))
    assert min(tau for (tau, _) in c) == int(g["block_ba_min_tau"])
    assert {y for (tau, y) in c if tau == 1} == {int(g["block_ba_rejected_Y"])}
    # the printed ordering token < block < ideal
    assert float(g["token_expected_tau"]) < _expected_tau(law) < float(g["ideal_expected_tau"])


# ---------------------------------------------------------------- Theorem 1 (lossless), exact
CASES = [(2, 1), (2, 2), (2, 3), (3, 2), (3, 3), (4, 2), (4, 3)]


@pytest.mark.parametrize("V,gamma", CASES)
@pytest.mark.parametrize("algo", [oracle.BLOCK, oracle.TOKEN])
def test_lossless_by_enumeration(V, gamma, algo):
    """(X^tau, Y, Z^{gamma-tau}) with Z ~ M_b has law M_b^{gamma+1} (Lemma on valid
    verification + Theorem 1; token verification is valid too)."""
    rng = np.random.default_rng(1000 * V + gamma)
    Mb = tiny.random_tables(rng, V, gamma)
    Ms = tiny.random_tables(rng, V, gamma)
    law, _, skipped = tiny.output_law(algo, Mb, Ms, V, gamma)
    assert skipped < 1e-9
    out = tiny.emitted_law(law, Mb, V, gamma)
    worst = 0.0
    for seq in itertools.product(range(V), repeat=gamma + 1):
        worst = max(worst, abs(out.get(seq, 0.0) - tiny.joint(Mb, seq)))
    assert worst < 1e-12 + skipped


@pytest.mark.parametrize("V,gamma", [(3, 2), (4, 2), (3, 3), (4, 3)])
@pytest.mark.parametrize("algo", [oracle.BLOCK, oracle.TOKEN])
def test_lossless_with_masked_tokens(V, gamma, algo):
    """The same with conditionals in which tokens are masked out (logit -inf, as top-k / top-p warping
    leaves them), independently in the two models: a drafted token the target excludes has ratio 0 and
    must never survive, and the output law must still be M_b^{gamma+1}."""
    rng = np.random.default_rng(77 * V + gamma)
    Mb = tiny.sparse_tables(rng, V, gamma)
    Ms = tiny.sparse_tables(rng, V, gamma)
    law, _, skipped = tiny.output_law(algo, Mb, Ms, V, gamma)
    assert skipped < 1e-9
    out = tiny.emitted_law(law, Mb, V, gamma)
    worst = 0.0
    for seq in itertools.product(range(V), repeat=gamma + 1):
        worst = max(worst, abs(out.get(seq, 0.0) - tiny.joint(Mb, seq)))
    assert worst < 1e-12 + skipped
    # no accepted prefix contains a token of target probability zero
    for (xs, tau, y), pr in law.items():
        if pr > 0:
            assert all(Mb[xs[:i]][xs[i]] > 0 for i in range(tau)) and Mb[xs[:tau]][y] > 0


# ------------------------------------------- Lemma "accept_prob": Pr(tau >= i | X^i) = w_i(x^i)
def _w_from_definition(Mb, Ms, xs):
    """eq. (def_as) evaluated on the tables: the quantity the lemma speaks about."""
    w = [1.0]
    for i in range(1, len(xs) + 1):
        r = Mb[xs[:i - 1]][xs[i - 1]] / Ms[xs[:i - 1]][xs[i - 1]]
        w.append(min(w[-1] * r, 1.0))
    return w


@pytest.mark.parametrize("V,gamma", [(2, 3), (3, 3), (4, 2)])
def test_block_prefix_acceptance_equals_w(V, gamma):
    rng = np.random.default_rng(77 + V * 10 + gamma)
    Mb = tiny.random_tables(rng, V, gamma)
    Ms = tiny.random_tables(rng, V, gamma)
    law, _, _ = tiny.output_law(oracle.BLOCK, Mb, Ms, V, gamma)
    for i in range(1, gamma + 1):
        for prefix in itertools.product(range(V), repeat=i):
            num = sum(m for (xs, tau, _), m in law.items() if xs[:i] == prefix and tau >= i)
            den = tiny.joint(Ms, prefix)
            assert num / den == pytest.approx(_w_from_definition(Mb, Ms, prefix)[i], abs=1e-12)


@pytest.mark.parametrize("V,gamma", [(2, 3), (3, 3), (4, 2)])
def test_tau_equals_l_probability_is_residual_mass(V, gamma):
    """Proof of Theorem 1: Pr(tau = l | X^l = x^l) = S_l (the residual mass the oracle reports)."""
    rng = np.random.default_rng(5 + V * 10 + gamma)
    Mb = tiny.random_tables(rng, V, gamma)
    Ms = tiny.random_tables(rng, V, gamma)
    law, dbg, _ = tiny.output_law(oracle.BLOCK, Mb, Ms, V, gamma)
    for l in range(0, gamma):
        for prefix in itertools.product(range(V), repeat=l):
            num = sum(m for (xs, tau, _), m in law.items() if xs[:l] == prefix and tau == l)
            den = tiny.joint(Ms, prefix)
            some_draft = prefix + (0,) * (gamma - l)
            assert num / den == pytest.approx(dbg[some_draft][l, 1], abs=1e-12)


# ------------------------------------------------- closed forms and orderings of E[tau]
@pytest.mark.parametrize("V,gamma", CASES)
def test_expected_accept_length_closed_forms_and_ordering(V, gamma):
    rng = np.random.default_rng(31 * V + gamma)
    Mb = tiny.random_tables(rng, V, gamma)
    Ms = tiny.random_tables(rng, V, gamma)
    e_block = _expected_tau(tiny.output_law(oracle.BLOCK, Mb, Ms, V, gamma)[0])
    e_token = _expected_tau(tiny.output_law(oracle.TOKEN, Mb, Ms, V, gamma)[0])
    e_greedy = _expected_tau(tiny.output_law(oracle.GREEDY, Mb, Ms, V, gamma)[0])
    # token: Pr(tau >= i) = sum_{x^i} prod_j min(M_s, M_b)(x_j | x^{j-1})  (Leviathan et al.; Sec. 2)
    tok = 0.0
    blk = 0.0
    bound = 0.0
    for i in range(1, gamma + 1):
        for xs in itertools.product(range(V), repeat=i):
            pr = 1.0
            for j in range(i):
                pr *= min(Ms[xs[:j]][xs[j]], Mb[xs[:j]][xs[j]])
            tok += pr
            blk += tiny.joint(Ms, xs) * _w_from_definition(Mb, Ms, xs)[i]
            bound += min(tiny.joint(Ms, xs), tiny.joint(Mb, xs))
    assert e_token == pytest.approx(tok, abs=1e-12)
    assert e_block == pytest.approx(blk, abs=1e-12)            # Lemma accept_prob
    assert e_block >= e_token - 1e-12                          # Theorem 2
    assert e_block <= bound + 1e-12                            # coupling upper bound (App. C)
    assert e_greedy == pytest.approx(bound, abs=1e-12)         # Lemma block-accept (greedy attains it)
    assert e_greedy >= e_block - 1e-12                         # greedy >= block in one iteration


def test_toy_gamma3_context_independent_token_closed_form():
    # context-independent: E_token[tau] = sum_i (1 - d_TV)^i with d_TV = 1/3 (Sec. 2)
    Mb, Ms = _toy(3)
    law, _, _ = tiny.output_law(oracle.TOKEN, Mb, Ms, 2, 3)
    assert _expected_tau(law) == pytest.approx(sum((2 / 3) ** i for i in (1, 2, 3)), abs=1e-6)


# ----------------------------------------- greedy: Lemma block-accept and the modified target
@pytest.mark.parametrize("V,gamma", [(2, 2), (3, 2), (3, 3)])
def test_greedy_joint_acceptance_is_min_of_joints(V, gamma):
    rng = np.random.default_rng(9 * V + gamma)
    Mb = tiny.random_tables(rng, V, gamma)
    Ms = tiny.random_tables(rng, V, gamma)
    law, _, _ = tiny.output_law(oracle.GREEDY, Mb, Ms, V, gamma)
    for l in range(1, gamma + 1):
        for prefix in itertools.product(range(V), repeat=l):
            got = sum(m for (xs, tau, _), m in law.items() if xs[:l] == prefix and tau >= l)
            assert got == pytest.approx(min(tiny.joint(Mb, prefix), tiny.joint(Ms, prefix)), abs=1e-12)


@pytest.mark.parametrize("V,gamma", [(2, 2), (3, 2), (3, 3)])
def test_greedy_is_lossless_with_distribution_modification(V, gamma):
    """Lemma greedy_block_identical: (X^tau, Y, Z^{gamma-tau-1}) ~ M_b^gamma when Z follows the
    modified target (normalised max(M_b - M_s, 0) on JOINT probabilities, Alg. 5)."""
    rng = np.random.default_rng(123 + 9 * V + gamma)
    Mb = tiny.random_tables(rng, V, gamma)
    Ms = tiny.random_tables(rng, V, gamma)
    law, _, _ = tiny.output_law(oracle.GREEDY, Mb, Ms, V, gamma)
    out = {}
    for (xs, tau, y), m in law.items():
        prefix = tuple(xs[:tau]) + (y,)
        if tau == gamma:              # gamma+1 tokens emitted: marginalise Y away
            seq = tuple(xs)
            out[seq] = out.get(seq, 0.0) + m
            continue
        for z in itertools.product(range(V), repeat=gamma - len(prefix)):
            seq = prefix + z
            pm = m
            for j in range(len(prefix), gamma):
                res = np.array([max(tiny.joint(Mb, seq[:j] + (x,)) - tiny.joint(Ms, seq[:j] + (x,)), 0.0)
                                for x in range(V)])
                pm *= res[seq[j]] / res.sum() if res.sum() > 0 else 0.0
            out[seq] = out.get(seq, 0.0) + pm
    for seq in itertools.product(range(V), repeat=gamma):
        assert out.get(seq, 0.0) == pytest.approx(tiny.joint(Mb, seq), abs=1e-12)


# ---------------------------------------------------------------- special cases
def _random_call(rng, B, gamma, V, sigma=2.0, noise=0.7):
    tl = (rng.standard_normal((B, gamma + 1, V)) * sigma).astype(np.float32)
    dl = (tl[:, :gamma] + rng.standard_normal((B, gamma, V)) * noise).astype(np.float32)
    tok = rng.integers(0, V, size=(B, gamma)).astype(np.int32)
    uni = (rng.integers(0, 1 << 24, size=(B, gamma + 1)) * 2.0 ** -24).astype(np.float32)
    return tl, dl, tok, uni


def test_gamma_one_block_equals_token():
    # Section 5: with gamma = 1 the two algorithms are the same
    rng = np.random.default_rng(3)
    tl, dl, tok, uni = _random_call(rng, 400, 1, 50)
    a = oracle.verify(oracle.BLOCK, tl, dl, tok, uni, 0.9)
    b = oracle.verify(oracle.TOKEN, tl, dl, tok, uni, 0.9)
    assert np.array_equal(a["accept_len"], b["accept_len"])
    assert np.array_equal(a["next_token"], b["next_token"])
    assert 0 < a["accept_len"].sum() < 400


@pytest.mark.parametrize("algo", [oracle.BLOCK, oracle.TOKEN, oracle.GREEDY])
def test_identical_models_accept_everything_and_sample_target(algo):
    """draft == target: every ratio is 1, tau = gamma, and Y is a plain inverse-CDF draw of
    softmax(target row gamma / T) -- compared with scipy softmax + numpy cumsum/searchsorted."""
    rng = np.random.default_rng(11)
    B, gamma, V, T = 64, 3, 97, 0.7
    tl, _, tok, uni = _random_call(rng, B, gamma, V)
    dl = tl[:, :gamma].copy()
    out = oracle.verify(algo, tl, dl, tok, uni, T)
    assert np.all(out["accept_len"] == gamma)
    probs = scipy.special.softmax(tl[:, gamma].astype(np.float64) / T, axis=-1)
    cdf = np.cumsum(probs, axis=-1)
    want = np.array([np.searchsorted(cdf[b], float(uni[b, gamma]) * cdf[b, -1], side="right") for b in range(B)])
    assert np.array_equal(out["next_token"], want)


def test_log_normalisers_match_scipy_logsumexp():
    rng = np.random.default_rng(12)
    tl, dl, tok, uni = _random_call(rng, 5, 4, 333, sigma=6.0)
    T = 0.55
    out = oracle.verify(oracle.BLOCK, tl, dl, tok, uni, T)
    want_t = scipy.special.logsumexp(tl.astype(np.float64) / T, axis=-1)
    want_d = scipy.special.logsumexp(dl.astype(np.float64) / T, axis=-1)
    assert np.allclose(out["dbg"][:, :, 3], want_t, rtol=0, atol=1e-11)
    assert np.allclose(out["dbg"][:, :4, 4], want_d, rtol=0, atol=1e-11)
    # log r_i = log p_{i-1}(X_i) - log q_{i-1}(X_i) with scipy's log_softmax
    lp = scipy.special.log_softmax(tl.astype(np.float64) / T, axis=-1)
    lq = scipy.special.log_softmax(dl.astype(np.float64) / T, axis=-1)
    for b in range(5):
        for i in range(1, 5):
            want = lp[b, i - 1, tok[b, i - 1]] - lq[b, i - 1, tok[b, i - 1]]
            assert out["dbg"][b, i, 5] == pytest.approx(want, abs=1e-11)


def test_residual_mass_identities():
    """S_i = w_i - sum_x min(w_i p_i, q_i) (proof of Lemma accept_prob), h_i = (w_i - m_i)/(1 - m_i),
    S_0 = d_TV(p_0, q_0) = 0.5 * ||p_0 - q_0||_1 (Sec. 2), and w_i >= prod_j min(1, r_j) pointwise."""
    rng = np.random.default_rng(13)
    B, gamma, V, T = 40, 5, 211, 1.3
    tl, dl, tok, uni = _random_call(rng, B, gamma, V, noise=1.0)
    # draw the draft tokens from the draft model so that ratios are typical
    q = scipy.special.softmax(dl.astype(np.float64) / T, axis=-1)
    p = scipy.special.softmax(tl.astype(np.float64) / T, axis=-1)
    for b in range(B):
        for i in range(gamma):
            tok[b, i] = rng.choice(V, p=q[b, i])
    out = oracle.verify(oracle.BLOCK, tl, dl, tok, uni, T)
    tk = oracle.verify(oracle.TOKEN, tl, dl, tok, uni, T)
    w, S, h = out["dbg"][..., 0], out["dbg"][..., 1], out["dbg"][..., 2]
    for b in range(B):
        assert S[b, 0] == pytest.approx(0.5 * np.abs(p[b, 0] - q[b, 0]).sum(), abs=1e-13)
        run = 1.0
        for i in range(gamma):
            m = np.minimum(w[b, i] * p[b, i], q[b, i]).sum()
            assert S[b, i] == pytest.approx(w[b, i] - m, abs=1e-13)
            if 1 <= i and w[b, i] < 1.0:
                assert h[b, i] == pytest.approx((w[b, i] - m) / (1.0 - m), abs=1e-11)
        for i in range(1, gamma + 1):
            run *= tk["dbg"][b, i, 2]
            assert w[b, i] >= run - 1e-15
        assert S[b, gamma] == w[b, gamma] == h[b, gamma]
    # token verification's residual masses are the w == 1 case
    assert np.allclose(tk["dbg"][:, :gamma, 1], 0.5 * np.abs(p[:, :gamma] - q).sum(-1), atol=1e-13)


def test_residual_sample_never_returns_a_zero_weight_token_and_follows_the_weights():
    rng = np.random.default_rng(14)
    gamma, V, T = 2, 12, 1.0
    tl, dl, tok, _ = _random_call(rng, 1, gamma, V, noise=1.5)
    # draft tokens the target likes least relative to the draft: every h_i < 1
    lr = (scipy.special.log_softmax(tl[0, :gamma].astype(np.float64) / T, axis=-1)
          - scipy.special.log_softmax(dl[0].astype(np.float64) / T, axis=-1))
    tok[0] = lr.argmin(-1)
    n = 20000
    uni = np.zeros((n, gamma + 1), np.float32)
    uni[:, :gamma] = 0.999999          # reject everything: tau = 0 for both algorithms
    uni[:, gamma] = ((np.arange(n) + 0.5) / n).astype(np.float32)
    out = oracle.verify(oracle.BLOCK, np.repeat(tl, n, 0), np.repeat(dl, n, 0), np.repeat(tok, n, 0), uni, T)
    keep = out["accept_len"] == 0
    assert keep.sum() > n // 2
    p0 = scipy.special.softmax(tl[0, 0].astype(np.float64) / T)
    q0 = scipy.special.softmax(dl[0, 0].astype(np.float64) / T)
    rho = np.maximum(p0 - q0, 0.0)
    freq = np.bincount(out["next_token"][keep], minlength=V) / keep.sum()
    assert np.all(freq[rho == 0.0] == 0.0)
    assert np.allclose(freq, rho / rho.sum(), atol=2.0 / n * V)


def test_bf16_inputs_are_upcast_exactly():
    import torch
    rng = np.random.default_rng(15)
    tl, dl, tok, uni = _random_call(rng, 6, 3, 130)
    tb = torch.from_numpy(tl).to(torch.bfloat16)
    db = torch.from_numpy(dl).to(torch.bfloat16)
    a = oracle.verify(oracle.BLOCK, tb.view(torch.int16).numpy().view(np.uint16),
                      db.view(torch.int16).numpy().view(np.uint16), tok, uni, 0.8, dtype=oracle.BF16)
    b = oracle.verify(oracle.BLOCK, tb.float().numpy(), db.float().numpy(), tok, uni, 0.8, dtype=oracle.F32)
    assert np.array_equal(a["accept_len"], b["accept_len"])
    assert np.array_equal(a["next_token"], b["next_token"])
    assert np.array_equal(a["dbg"], b["dbg"], equal_nan=True)


def test_margins_flag_a_uniform_on_a_boundary():
    rng = np.random.default_rng(16)
    tl, dl, tok, uni = _random_call(rng, 1, 3, 40)
    base = oracle.verify(oracle.BLOCK, tl, dl, tok, uni, 1.0)
    h = base["dbg"][0, :, 2]
    uni2 = uni.copy()
    uni2[0, 2] = np.float32(h[3])        # eta_3 on top of h_3 (to float32 rounding)
    out = oracle.verify(oracle.BLOCK, tl, dl, tok, uni2, 1.0)
    assert out["margins"][0, 0] < 1e-7
    assert base["margins"][0, 1] > 0.0


def test_bad_arguments_are_rejected():
    rng = np.random.default_rng(17)
    tl, dl, tok, uni = _random_call(rng, 2, 2, 10)
    with pytest.raises(RuntimeError):
        oracle.verify(oracle.BLOCK, tl, dl, tok, uni, 0.0)
    bad = tok.copy()
    bad[0, 0] = 10
    with pytest.raises(RuntimeError):
        oracle.verify(oracle.BLOCK, tl, dl, bad, uni, 1.0)


def test_greedy_rejected_mass_equals_residual_mass_plus_one_minus_w():
    """For rows that sum to one, sum_x max(q - w p, 0) = sum_x max(w p - q, 0) - sum_x (w p - q) = S + 1 - w, so the
    ratio of Alg. 4 (which the oracle forms from the two sums, each taken directly) is S / (S + 1 - w) wherever
    w < 1, and at least 1 wherever w >= 1.  The kernels rely on this to skip the second sum."""
    rng = np.random.default_rng(99)
    tl, dl, tok, uni = _random_call(rng, 50, 6, 400)
    out = oracle.verify(oracle.GREEDY, tl, dl, tok, uni, 0.9)
    w, S, h = out["dbg"][:, 1:6, 0], out["dbg"][:, 1:6, 1], out["dbg"][:, 1:6, 2]      # positions 1 .. gamma - 1
    below = w < 1.0
    assert below.any() and (~below).any()
    np.testing.assert_allclose(h[below], np.minimum(S[below] / (S[below] + 1.0 - w[below]), 1.0), rtol=1e-9, atol=1e-12)
    assert np.all(h[~below] == 1.0)


@pytest.mark.parametrize("algo", [oracle.BLOCK, oracle.GREEDY])
def test_acceptance_probability_never_exceeds_w(algo):
    """S_i = sum_x max(w_i p_i - q_i, 0) <= sum_x w_i p_i = w_i, and S / (S + 1 - w) grows with S, so
    h_i <= w_i / (w_i + 1 - w_i) = w_i (Alg. 2; Alg. 4 with its unclipped weight, where h_i = 1 <= w_i once w_i >= 1).
    A test with eta_i >= w_i therefore fails whatever S_i is - what lets the kernels leave such a position's
    residual mass unformed.  Checked on the oracle's own w, S and h, and on its decisions: no position whose
    uniform is at or above w_i is ever the accepted length."""
    rng = np.random.default_rng(1234)
    tl, dl, tok, uni = _random_call(rng, 200, 6, 300)
    out = oracle.verify(algo, tl, dl, tok, uni, 0.8)
    w, S, h = out["dbg"][:, 1:, 0], out["dbg"][:, 1:, 1], out["dbg"][:, 1:, 2]         # positions 1 .. gamma
    assert np.all(S <= w * (1 + 1e-12))
    assert np.all(h <= np.maximum(w, 0.0) * (1 + 1e-12) + 1e-300)
    hopeless = uni[:, :6] >= w                                  # eta_i >= w_i
    assert hopeless.any() and (~hopeless).any()
    tau = out["accept_len"]
    for b in range(len(tau)):
        if tau[b] >= 1:
            assert not hopeless[b, tau[b] - 1]


@pytest.mark.parametrize("algo", [oracle.BLOCK, oracle.GREEDY])
def test_a_position_before_a_weight_of_one_is_never_the_accepted_length(algo):
    """Alg. 2 / 4 keep the LAST position whose test passes.  Where w_{i+1} >= 1 the acceptance probability of position
    i + 1 is 1 (h = 1 at w >= 1; the last test is eta < min(w_gamma, 1)) and its test passes whatever its uniform in
    [0, 1) is, so tau >= i + 1 and position i is never the accepted length - what lets the kernels leave position i's
    residual mass unformed once they know w_{i+1}.  Checked on the oracle's own w and decisions, with drafts close enough
    to the target for weights of one to be common."""
    rng = np.random.default_rng(4321)
    B, gamma, V = 300, 6, 200
    tl = rng.normal(0.0, 2.0, (B, gamma + 1, V)).astype(np.float32)
    dl = (tl[:, :gamma] + rng.normal(0.0, 0.4, (B, gamma, V))).astype(np.float32)
    q = np.exp(dl.astype(np.float64) / 0.8)
    q /= q.sum(-1, keepdims=True)
    tok = np.array([[rng.choice(V, p=q[b, i]) for i in range(gamma)] for b in range(B)], dtype=np.int32)
    uni = rng.random((B, gamma + 1)).astype(np.float32)
    out = oracle.verify(algo, tl, dl, tok, uni, 0.8)
    w = out["dbg"][:, :, 0]                                     # w_0 .. w_gamma
    sure = w[:, 1:] >= 1.0                                      # position i + 1 surely passes, i = 0 .. gamma - 1
    assert sure.any() and (~sure).any()
    tau = out["accept_len"]
    for b in range(B):
        if tau[b] < gamma:
            assert not sure[b, tau[b]]
    # and the position behind such a weight has acceptance probability one
    h = out["dbg"][:, 1:, 2]
    assert np.all(h[sure] == 1.0)
