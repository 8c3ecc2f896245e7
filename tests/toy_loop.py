"""The outer loop of speculative decoding (Alg. 3) around the ORACLE, for context-independent toy models
(Sec. 2: both models ignore the context, so every row of a model's logits is the same vector).

One iteration per sequence: draft gamma tokens from M_s, score them with both models (here: repeat the two
logit vectors), verify, emit X^tau and Y.  With context-independent models the iterations are independent,
which is what lets B sequences x `iters` iterations stand for B * iters draws of (tau, Y).
The uniforms of iteration `it` come from `workloads.philox_uniforms`, so the GPU loop gets the same ones.
"""
from __future__ import annotations

import numpy as np

import oracle
import workloads

ALGO = {"block": oracle.BLOCK, "token": oracle.TOKEN, "greedy": oracle.GREEDY}


def iteration_uniforms(seed: int, it: int, B: int, gamma: int):
    """(draft uniforms [B, gamma], verification uniforms [B, gamma+1]) of iteration `it`."""
    u = workloads.philox_uniforms(seed * 100003 + it, (B, 2 * gamma + 1))
    return np.ascontiguousarray(u[:, :gamma]), np.ascontiguousarray(u[:, gamma:])


def oracle_loop(algo: str, target_logits, draft_logits, gamma: int, B: int, iters: int, temperature: float, seed: int):
    target_logits = np.asarray(target_logits, dtype=np.float32)
    draft_logits = np.asarray(draft_logits, dtype=np.float32)
    V = target_logits.shape[0]
    tl = np.ascontiguousarray(np.broadcast_to(target_logits, (B, gamma + 1, V)))
    dl = np.ascontiguousarray(np.broadcast_to(draft_logits, (B, gamma, V)))
    taus, ys, xs, margins = [], [], [], []
    for it in range(iters):
        u_draft, u_verify = iteration_uniforms(seed, it, B, gamma)
        x, m_x = oracle.sample_rows(dl.reshape(B * gamma, V), u_draft.reshape(-1), temperature)
        x = x.reshape(B, gamma)
        out = oracle.verify(ALGO[algo], tl, dl, x, u_verify, temperature)
        taus.append(out["accept_len"]); ys.append(out["next_token"]); xs.append(x)
        margins.append(np.minimum(m_x.reshape(B, gamma).min(axis=1), out["margins"].min(axis=1)))
    return {"tau": np.stack(taus), "y": np.stack(ys), "x": np.stack(xs), "margin": np.stack(margins)}


def ccdf(tau, gamma):
    """P(tau >= k), k = 0 .. gamma."""
    tau = np.asarray(tau).reshape(-1)
    return np.array([(tau >= k).mean() for k in range(gamma + 1)])
