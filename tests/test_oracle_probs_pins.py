"""Pins of the oracle's probability-input form (the ps / qs arrays of App. A) against what the paper
and the mathematics fix: the printed values of the worked example with its tables typed in directly,
the exact output law on tiny vocabularies (Theorem 1), the prefix-acceptance lemma, a hand-computed
case with rows that do not sum to one, and agreement with the logit form on softmax rows computed
by a library routine.
"""
from __future__ import annotations

import itertools
from fractions import Fraction

import numpy as np
import pytest
import scipy.special

import oracle
from tests import tiny
from tests.test_oracle_pins import _cond, _expected_tau, _golden, _toy, CASES


# ---------------------------------------------------------------- printed values (Sec. 2)
def test_toy_example_printed_values_from_probability_tables():
    g = _golden()
    Mb, Ms = _toy(2)
    tok_law, dbg, skipped = tiny.output_law(oracle.TOKEN, Mb, Ms, 2, 2, form="probs")
    assert skipped < 1e-9
    assert _expected_tau(tok_law) == pytest.approx(float(g["token_expected_tau"]), abs=1e-6)
    for xs, d in dbg.items():
        for i, x in enumerate(xs, start=1):
            want = g["token_accept_a"] if x == 0 else g["token_accept_b"]
            assert d[i, 2] == pytest.approx(float(want), abs=1e-6)
    law, _, skipped = tiny.output_law(oracle.BLOCK, Mb, Ms, 2, 2, form="probs")
    assert skipped < 1e-9
    assert _expected_tau(law) == pytest.approx(float(g["block_expected_tau"]), abs=1e-6)
    for xs, key in (((0, 1), "block_accept_all_ab"), ((1, 1), "block_accept_all_bb"),
                    ((0, 0), "block_accept_all_aa"), ((1, 0), "block_accept_all_ba")):
        c = _cond(law, Ms, xs)
        assert sum(m for (tau, _), m in c.items() if tau == 2) == pytest.approx(float(g[key]), abs=1e-6)


# ---------------------------------------------------------------- Theorem 1 (lossless), exact
@pytest.mark.parametrize("V,gamma", CASES)
@pytest.mark.parametrize("algo", [oracle.BLOCK, oracle.TOKEN])
def test_lossless_by_enumeration_probability_form(V, gamma, algo):
    rng = np.random.default_rng(2000 * V + gamma)
    Mb = tiny.random_tables(rng, V, gamma)
    Ms = tiny.random_tables(rng, V, gamma)
    law, _, skipped = tiny.output_law(algo, Mb, Ms, V, gamma, form="probs")
    assert skipped < 1e-9
    out = tiny.emitted_law(law, Mb, V, gamma)
    worst = max(abs(out.get(seq, 0.0) - tiny.joint(Mb, seq)) for seq in itertools.product(range(V), repeat=gamma + 1))
    assert worst < 1e-12 + skipped


@pytest.mark.parametrize("V,gamma", [(3, 2), (4, 3)])
@pytest.mark.parametrize("algo", [oracle.BLOCK, oracle.TOKEN])
def test_lossless_with_zero_probabilities_probability_form(V, gamma, algo):
    """Rows with exact zeros (tokens outside a model's support) in both models."""
    rng = np.random.default_rng(91 * V + gamma)
    Mb = tiny.sparse_tables(rng, V, gamma)
    Ms = tiny.sparse_tables(rng, V, gamma)
    law, _, skipped = tiny.output_law(algo, Mb, Ms, V, gamma, form="probs")
    assert skipped < 1e-9
    out = tiny.emitted_law(law, Mb, V, gamma)
    worst = max(abs(out.get(seq, 0.0) - tiny.joint(Mb, seq)) for seq in itertools.product(range(V), repeat=gamma + 1))
    assert worst < 1e-12 + skipped
    for (xs, tau, y), pr in law.items():
        if pr > 0:
            assert all(Mb[xs[:i]][xs[i]] > 0 for i in range(tau)) and Mb[xs[:tau]][y] > 0


# ---------------------------------------------------------------- Lemma: Pr(tau >= i | X^i) = w_i
@pytest.mark.parametrize("V,gamma", [(3, 3), (4, 2)])
def test_block_prefix_acceptance_equals_w_probability_form(V, gamma):
    rng = np.random.default_rng(5 * V + gamma)
    Mb = tiny.random_tables(rng, V, gamma)
    Ms = tiny.random_tables(rng, V, gamma)
    law, _, _ = tiny.output_law(oracle.BLOCK, Mb, Ms, V, gamma, form="probs")
    for i in range(1, gamma + 1):
        for prefix in itertools.product(range(V), repeat=i):
            w = 1.0                                          # the definition of w_i, from the tables
            for j in range(i):
                w = min(w * Mb[prefix[:j]][prefix[j]] / Ms[prefix[:j]][prefix[j]], 1.0)
            got = sum(m for (xs, tau, _), m in law.items() if xs[:i] == prefix and tau >= i) / tiny.joint(Ms, prefix)
            assert got == pytest.approx(w, abs=1e-11)


# ---------------------------------------------------------------- rows are used as given
def test_unnormalised_rows_are_used_as_given_hand_computed():
    """gamma = 1, V = 3, rows that do not sum to one, every quantity worked out by hand in exact
    fractions: X_1 = 0, r_1 = p_0(0) / q_0(0) = (1/8) / (1/2) = 1/4 = w_1 = h_1 (block, last position).
    eta = 0.3 rejects; the residual at row 0 is max(p_0 - q_0, 0) = (0, 3/8, 1/8), total 1/2;
    u = 0.8 -> t = 0.4 > 3/8 -> Y = 2;  u = 0.7 -> t = 0.35 < 3/8 -> Y = 1.
    eta = 0.2 accepts; Y is drawn from p_1 = (1/4, 1/4, 1/4) (sum 3/4): u = 0.7 -> t = 0.525 -> Y = 2."""
    p = np.array([[[1 / 8, 5 / 8, 1 / 4], [1 / 4, 1 / 4, 1 / 4]]], dtype=np.float32)
    q = np.array([[[1 / 2, 1 / 4, 1 / 8]]], dtype=np.float32)
    tok = np.array([[0]], dtype=np.int32)
    for algo in (oracle.BLOCK, oracle.TOKEN):
        for eta, u, tau, y in ((0.3, 0.8, 0, 2), (0.3, 0.7, 0, 1), (0.2, 0.7, 1, 2), (0.2, 0.1, 1, 0)):
            out = oracle.verify_probs(algo, p, q, tok, np.array([[eta, u]], dtype=np.float32))
            assert (int(out["accept_len"][0]), int(out["next_token"][0])) == (tau, y), (algo, eta, u)
            assert out["dbg"][0, 1, 2] == pytest.approx(float(Fraction(1, 4)), abs=1e-15)
    out = oracle.verify_probs(oracle.BLOCK, p, q, tok, np.array([[0.3, 0.8]], dtype=np.float32))
    assert out["dbg"][0, 0, 1] == pytest.approx(0.5, abs=1e-15)        # S_0 = 3/8 + 1/8


# ---------------------------------------------------------------- agreement with the logit form
@pytest.mark.parametrize("algo", [oracle.BLOCK, oracle.TOKEN, oracle.GREEDY])
def test_probability_form_agrees_with_logit_form_on_library_softmax_rows(algo):
    """Softmax rows from scipy, handed over as float64 probabilities, must give the decisions and the
    w, S, h of the logit form on the same logits (wherever no uniform sits on a boundary)."""
    rng = np.random.default_rng(17)
    B, gamma, V, T = 40, 5, 300, 0.7
    tl = (rng.standard_normal((B, gamma + 1, V)) * 2).astype(np.float32)
    dl = (tl[:, :gamma] + rng.standard_normal((B, gamma, V)) * 0.8).astype(np.float32)
    P = scipy.special.softmax(tl.astype(np.float64) / T, axis=-1)
    Q = scipy.special.softmax(dl.astype(np.float64) / T, axis=-1)
    tok = np.stack([[rng.choice(V, p=Q[b, i]) for i in range(gamma)] for b in range(B)]).astype(np.int32)
    uni = rng.random((B, gamma + 1)).astype(np.float32)
    a = oracle.verify(algo, tl, dl, tok, uni, T)
    b = oracle.verify_probs(algo, P, Q, tok, uni, dtype=oracle.F64)
    safe = a["margins"].min(axis=1) > 1e-9
    assert safe.sum() >= B - 2
    assert np.array_equal(a["accept_len"][safe], b["accept_len"][safe])
    assert np.array_equal(a["next_token"][safe], b["next_token"][safe])
    np.testing.assert_allclose(b["dbg"][:, :, :3], a["dbg"][:, :, :3], rtol=1e-10, atol=1e-13)


def test_float32_and_bf16_probability_rows_are_upcast_exactly():
    import torch
    g = torch.Generator().manual_seed(3)
    P = torch.softmax(torch.randn(3, 4, 50, generator=g) * 2, -1).to(torch.bfloat16)
    Q = torch.softmax(torch.randn(3, 3, 50, generator=g) * 2, -1).to(torch.bfloat16)
    tok = torch.multinomial(Q.float().reshape(-1, 50), 1).reshape(3, 3).numpy().astype(np.int32)
    uni = np.random.default_rng(5).random((3, 4)).astype(np.float32)
    a = oracle.verify_probs(oracle.BLOCK, P.view(torch.int16).numpy().view(np.uint16),
                            Q.view(torch.int16).numpy().view(np.uint16), tok, uni, dtype=oracle.BF16)
    b = oracle.verify_probs(oracle.BLOCK, P.float().numpy(), Q.float().numpy(), tok, uni, dtype=oracle.F32)
    c = oracle.verify_probs(oracle.BLOCK, P.double().numpy(), Q.double().numpy(), tok, uni, dtype=oracle.F64)
    for other in (b, c):
        assert np.array_equal(a["accept_len"], other["accept_len"]) and np.array_equal(a["next_token"], other["next_token"])
        assert np.array_equal(a["dbg"][:, :, :3], other["dbg"][:, :, :3])


# ---------------------------------------------------------------- greedy block verification (Alg. 4)
@pytest.mark.parametrize("V,gamma", [(2, 2), (3, 2), (3, 3)])
def test_greedy_joint_acceptance_is_min_of_joints_probability_form(V, gamma):
    """Lemma on greedy block verification: Pr(X^l = x^l, tau >= l) = min{M_b(x^l), M_s(x^l)}."""
    rng = np.random.default_rng(31 * V + gamma)
    Mb = tiny.random_tables(rng, V, gamma)
    Ms = tiny.random_tables(rng, V, gamma)
    law, _, skipped = tiny.output_law(oracle.GREEDY, Mb, Ms, V, gamma, form="probs")
    assert skipped < 1e-9
    for l in range(1, gamma + 1):
        for prefix in itertools.product(range(V), repeat=l):
            got = sum(m for (xs, tau, _), m in law.items() if xs[:l] == prefix and tau >= l)
            assert got == pytest.approx(min(tiny.joint(Mb, prefix), tiny.joint(Ms, prefix)), abs=1e-12)


@pytest.mark.parametrize("V,gamma", CASES)
def test_expected_accept_length_ordering_probability_form(V, gamma):
    """Theorem 2 (block >= token in expected accepted length) and the greedy upper bound sum_l sum_x min{M_s, M_b}."""
    rng = np.random.default_rng(400 * V + gamma)
    Mb = tiny.random_tables(rng, V, gamma)
    Ms = tiny.random_tables(rng, V, gamma)
    e = {a: _expected_tau(tiny.output_law(a, Mb, Ms, V, gamma, form="probs")[0])
         for a in (oracle.BLOCK, oracle.TOKEN, oracle.GREEDY)}
    bound = sum(min(tiny.joint(Mb, x), tiny.joint(Ms, x))
                for l in range(1, gamma + 1) for x in itertools.product(range(V), repeat=l))
    assert e[oracle.TOKEN] <= e[oracle.BLOCK] + 1e-12
    assert e[oracle.BLOCK] <= e[oracle.GREEDY] + 1e-12
    assert e[oracle.GREEDY] == pytest.approx(bound, abs=1e-11)
