"""Seeded random shapes and options against the oracle: batch, draft length, vocabulary (tiny, odd, chunk
boundaries, wide rows), dtype, algorithm, temperature, kernel path, top-k masking, per-sequence draft
lengths and padded rows (everything that must not be read is NaN), two calls in a row on one workspace.
Sequences are compared with the oracle's result on their own leading rows."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import oracle
import paper_2403_10444_amd as sv
import workloads
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
PATHS = {"default": 0, "staged": 1, "fused": 3, "fused-large": 4}


def _draw_case(rng, it, probs):
    B = int(rng.integers(1, 40))
    gamma = int(rng.integers(1, 13))
    V = int(rng.choice([rng.integers(2, 300), rng.integers(300, 9000), rng.integers(9000, 70000),
                        rng.integers(70000, 300000), 8192, 16384, 131072, 131080, 8 * rng.integers(100, 6000)]))
    dtype = str(rng.choice(["bf16", "f32"]))
    T = float(rng.choice([0.5, 0.8, 1.0, 1.5]))
    cfg = workloads.Config(f"random{it}", B, gamma, V, dtype, float(rng.choice([1.0, 3.0, 6.0])),
                           float(rng.choice([0.3, 1.0, 2.5])), T, bool(rng.integers(0, 2)), 1)
    return dict(cfg=cfg, algo=str(rng.choice(["block", "token", "greedy"])), path=str(rng.choice(list(PATHS))),
                top_k=int(rng.choice([0, 0, 0, 5, 50])) if V > 200 else 0, use_lens=bool(rng.integers(0, 2)),
                pad_t=int(rng.choice([0, 0, 8, 3, 24])), pad_d=int(rng.choice([0, 0, 8, 5, 16])),
                lens_seed=int(rng.integers(1 << 30)))


def _host(t):
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16), oracle.BF16
    return t.cpu().numpy(), oracle.F32


def _check(case, it, probs):
    cfg, algo = case["cfg"], case["algo"]
    B, gamma, V, T = cfg.B, cfg.gamma, cfg.V, cfg.temperature
    inp = workloads.generate(cfg, seed=1000 + it, device=DEV, top_k_target=case["top_k"], top_k_draft=3 * case["top_k"])
    rows_t, rows_d = inp["target_logits"], inp["draft_logits"]
    if probs:
        rows_t = torch.softmax(rows_t.float() / T, -1).to(rows_t.dtype)
        rows_d = torch.softmax(rows_d.float() / T, -1).to(rows_d.dtype)
        if not bool((torch.gather(rows_d.float(), 2, inp["draft_tokens"].long().unsqueeze(-1)) > 0).all()):
            return                                   # a drafted token's probability rounded to zero: outside the contract
    lens = (np.random.default_rng(case["lens_seed"]).integers(1, gamma + 1, size=B).astype(np.int32)
            if case["use_lens"] else np.full(B, gamma, np.int32))
    tb = torch.full((B, gamma + 1, V + case["pad_t"]), float("nan"), dtype=rows_t.dtype, device=DEV)
    db = torch.full((B, gamma, V + case["pad_d"]), float("nan"), dtype=rows_d.dtype, device=DEV)
    tb[..., :V] = rows_t
    db[..., :V] = rows_d
    for b in range(B):
        tb[b, lens[b] + 1:] = float("nan")
        db[b, lens[b]:] = float("nan")
    dbg = torch.full((B, gamma + 1, 3), float("nan"), dtype=torch.float32, device=DEV)
    ws = sv.alloc_workspace(B, gamma, V, DEV)
    dl = torch.as_tensor(lens, device=DEV) if case["use_lens"] else None
    sv.spec_verify_debug_config(PATHS[case["path"]], -1)
    try:
        for _ in range(2):
            if probs:
                tau, y = sv.spec_verify_probs(algo, tb[..., :V], db[..., :V], inp["draft_tokens"], inp["uniforms"],
                                              draft_lens=dl, debug_out=dbg, workspace=ws)
            else:
                tau, y = sv.spec_verify_ex(algo, tb[..., :V], db[..., :V], inp["draft_tokens"], inp["uniforms"], T,
                                           draft_lens=dl, debug_out=dbg, workspace=ws)
        # the same without the debug block: residual masses that cannot matter are then left out, and the
        # decisions must not change
        if probs:
            tau2, y2 = sv.spec_verify_probs(algo, tb[..., :V], db[..., :V], inp["draft_tokens"], inp["uniforms"],
                                            draft_lens=dl, workspace=ws)
        else:
            tau2, y2 = sv.spec_verify_ex(algo, tb[..., :V], db[..., :V], inp["draft_tokens"], inp["uniforms"], T,
                                         draft_lens=dl, workspace=ws)
        torch.cuda.synchronize()
        assert torch.equal(tau, tau2) and torch.equal(y, y2), case
    finally:
        sv.spec_verify_debug_config(0, -1)
    assert sv.spec_verify_workspace_check(ws, B, gamma, V) == 0
    tau, y, dbg = tau.cpu().numpy(), y.cpu().numpy(), dbg.cpu().numpy()
    ht, odt = _host(rows_t)
    hd, _ = _host(rows_d)
    tok, uni = inp["draft_tokens"].cpu().numpy(), inp["uniforms"].cpu().numpy()
    for g in np.unique(lens):
        sel = np.nonzero(lens == g)[0]
        args = (parity.ALGOS[algo][0], ht[sel, :g + 1], hd[sel, :g], tok[sel, :g], uni[sel, :g + 1])
        ref = oracle.verify_probs(*args, dtype=odt) if probs else oracle.verify(*args, T, dtype=odt)
        m = ref["margins"]
        tau_bad = tau[sel] != ref["accept_len"]
        y_bad = (y[sel] != ref["next_token"]) & ~tau_bad
        unexcused = (tau_bad & ~(m[:, 0] < parity.MARGIN)) | (y_bad & ~(m[:, 1] < parity.MARGIN))
        assert not unexcused.any(), (case, int(g), sel[unexcused].tolist())
        S, w = ref["dbg"][:, :, 1], ref["dbg"][:, :, 0]
        tol = parity.S_RTOL * S + parity.S_FLOOR * np.maximum(w, 1e-30)
        assert np.all(np.abs(dbg[sel, :g + 1, 1].astype(np.float64) - S) <= tol), (case, int(g))


@pytest.mark.parametrize("probs", [False, True], ids=["logits", "probs"])
@pytest.mark.parametrize("block", range(4))
def test_random_shapes_and_options(block, probs):
    rng = np.random.default_rng(7000 + 10 * block + (1 if probs else 0))
    for j in range(25):
        it = 100 * block + j
        _check(_draw_case(rng, it, probs), it, probs)
