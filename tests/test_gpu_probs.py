"""GPU parity of `spec_verify_probs` (distributions handed over as probabilities, App. A's arrays) with the
oracle's probability form on the same values: the probabilities are made on the device from the seeded
synthetic logits (softmax at the workload's temperature, rounded to the input dtype) and the oracle reads
exactly those rounded values."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import workloads
from tests import parity
from tests.test_gpu_parity import _custom, _say

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _probs_inputs(cfg, seed, top_k=0):
    inp = workloads.generate(cfg, seed=seed, device=DEV, top_k_target=top_k, top_k_draft=top_k and 3 * top_k)
    dt = inp["target_logits"].dtype
    P = torch.softmax(inp["target_logits"].float() / cfg.temperature, -1).to(dt)
    Q = torch.softmax(inp["draft_logits"].float() / cfg.temperature, -1).to(dt)
    # the drafter produced X_i, so q(X_i) > 0 even after rounding to the input dtype
    q_tok = torch.gather(Q.float(), 2, inp["draft_tokens"].long().unsqueeze(-1))
    assert bool((q_tok > 0).all())
    return P, Q, inp


def _host(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16), oracle.BF16
    return t.cpu().numpy(), oracle.F32


def _run_gpu(sv, algo, P, Q, inp, **kw):
    B, g1, _ = P.shape
    dbg = torch.full((B, g1, 3), float("nan"), dtype=torch.float32, device=DEV)
    tau, y = sv.spec_verify_probs(algo, P, Q, inp["draft_tokens"], inp["uniforms"], debug_out=dbg, **kw)
    torch.cuda.synchronize()
    return {"accept_len": tau.cpu().numpy(), "next_token": y.cpu().numpy(), "dbg": dbg.cpu().numpy()}


def _run_oracle(algo, P, Q, inp):
    hp, dt = _host(P)
    hq, _ = _host(Q)
    return oracle.verify_probs(parity.ALGOS[algo][0], hp, hq, inp["draft_tokens"].cpu().numpy(),
                               inp["uniforms"].cpu().numpy(), dtype=dt)


SHAPES = [
    (1, 4, 1000, "f32"),
    (8, 8, 32000, "f32"),
    (16, 8, 128256, "bf16"),
    (4, 2, 8200, "bf16"),        # a chunk and a ragged tail, aligned
    (5, 3, 8191, "f32"),         # odd V: scalar loads
    (3, 1, 50257, "bf16"),       # gamma = 1, odd V
    (2, 64, 2000, "bf16"),       # the largest gamma
    (300, 3, 700, "f32"),
]


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("B,gamma,V,dtype", SHAPES)
def test_probs_parity(algo, B, gamma, V, dtype):
    import paper_2403_10444_amd as sv
    cfg = _custom(B, gamma, V, dtype, sigma_t=2.5, sigma_d=1.0, T=0.8)
    P, Q, inp = _probs_inputs(cfg, seed=900 + B + gamma)
    rep = parity.compare(_run_gpu(sv, algo, P, Q, inp), _run_oracle(algo, P, Q, inp),
                         label=f"probs {B}x{gamma}x{V} {dtype} {algo}", greedy=(algo == "greedy"))
    _say(rep)


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_probs_with_zero_probabilities(algo):
    """Top-k warped rows: most tokens have probability exactly zero, independently in the two models."""
    import paper_2403_10444_amd as sv
    cfg = _custom(16, 6, 20000, "bf16", sigma_t=3.0, sigma_d=1.0, T=0.9)
    P, Q, inp = _probs_inputs(cfg, seed=321, top_k=40)
    assert float((P == 0).float().mean()) > 0.9
    rep = parity.compare(_run_gpu(sv, algo, P, Q, inp), _run_oracle(algo, P, Q, inp),
                         label=f"probs top-k {algo}", greedy=(algo == "greedy"))
    _say(rep)


@pytest.mark.parametrize("algo", ["block", "token"])
def test_probs_with_draft_lengths_and_padded_rows(algo):
    """Per-sequence draft lengths and padded rows (NaN in everything that must not be read): sequence b must come
    out as the oracle gives it on its leading rows."""
    import paper_2403_10444_amd as sv
    B, gamma, V = 20, 6, 12000
    cfg = _custom(B, gamma, V, "bf16", sigma_t=2.5, sigma_d=1.0, T=1.0)
    P, Q, inp = _probs_inputs(cfg, seed=55)
    lens = np.array([1 + (b * 5) % gamma for b in range(B)], dtype=np.int32)
    Pb = torch.full((B, gamma + 1, V + 24), float("nan"), dtype=P.dtype, device=DEV)
    Qb = torch.full((B, gamma, V + 8), float("nan"), dtype=Q.dtype, device=DEV)
    Pb[..., :V] = P
    Qb[..., :V] = Q
    for b in range(B):
        Pb[b, lens[b] + 1:] = float("nan")
        Qb[b, lens[b]:] = float("nan")
    got = _run_gpu(sv, algo, Pb[..., :V], Qb[..., :V], inp, draft_lens=torch.as_tensor(lens, device=DEV))
    hp, dt = _host(P)
    hq, _ = _host(Q)
    tok, uni = inp["draft_tokens"].cpu().numpy(), inp["uniforms"].cpu().numpy()
    n_safe = 0
    for g in np.unique(lens):
        sel = np.nonzero(lens == g)[0]
        ref = oracle.verify_probs(parity.ALGOS[algo][0], hp[sel, :g + 1], hq[sel, :g], tok[sel, :g], uni[sel, :g + 1], dtype=dt)
        safe = ref["margins"].min(axis=1) >= parity.MARGIN
        n_safe += int(safe.sum())
        assert np.array_equal(got["accept_len"][sel][safe], ref["accept_len"][safe])
        assert np.array_equal(got["next_token"][sel][safe], ref["next_token"][safe])
    assert n_safe >= 0.8 * B


def test_probs_unnormalised_rows_are_used_as_given():
    """The hand-computed case of the oracle's pins (gamma = 1, V = 3, rows that do not sum to one)."""
    import paper_2403_10444_amd as sv
    p = torch.tensor([[[1 / 8, 5 / 8, 1 / 4], [1 / 4, 1 / 4, 1 / 4]]], dtype=torch.float32, device=DEV)
    q = torch.tensor([[[1 / 2, 1 / 4, 1 / 8]]], dtype=torch.float32, device=DEV)
    tok = torch.zeros((1, 1), dtype=torch.int32, device=DEV)
    for algo in ("block", "token"):
        for eta, u, tau, y in ((0.3, 0.8, 0, 2), (0.3, 0.7, 0, 1), (0.2, 0.7, 1, 2), (0.2, 0.1, 1, 0)):
            uni = torch.tensor([[eta, u]], dtype=torch.float32, device=DEV)
            a, b = sv.spec_verify_probs(algo, p, q, tok, uni)
            torch.cuda.synchronize()
            assert (int(a[0]), int(b[0])) == (tau, y), (algo, eta, u)
