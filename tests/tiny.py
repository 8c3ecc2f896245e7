"""Exact laws on tiny vocabularies, obtained by running the REAL oracle.

A tiny model is a table ``M[prefix] -> probability vector`` over V tokens for every
prefix (tuple of token ids) up to some length.  Given a target table, a draft table
and gamma, `output_law` returns the exact joint law of (X^gamma, tau, Y) produced by
the oracle when X^gamma ~ M_s^gamma and the uniforms are i.i.d. U[0,1): the oracle's
output is piecewise constant in the uniforms, so one evaluation at the midpoint of
every cell of a grid that refines all of its breakpoints, weighted by the cell's
volume, integrates it exactly.  Nothing here re-implements a verification algorithm;
the only formulas are the grid (any grid that is too coarse makes the pins fail, never
pass) and products of table entries.
"""
from __future__ import annotations

import itertools

import numpy as np

import oracle


class TinyModel:
    """Conditionals M(. | prefix) for every prefix of length 0..depth.

    The oracle takes float32 logits, so the model IS the softmax of float32 logits:
    ``logits[prefix]`` is float32(log of the requested probabilities) and
    ``prob[prefix]`` is its softmax in float64 -- the distribution the oracle sees.
    `model[prefix]` returns the latter.
    """

    def __init__(self, V, depth, requested):
        self.V, self.depth = V, depth
        self.logits, self.prob = {}, {}
        for L in range(depth + 1):
            for prefix in itertools.product(range(V), repeat=L):
                with np.errstate(divide="ignore"):          # a probability of zero is a logit of -inf (a masked token)
                    lg = np.log(np.asarray(requested(prefix), dtype=np.float64)).astype(np.float32)
                e = np.exp(lg.astype(np.float64) - float(lg.max()))
                self.logits[prefix] = lg
                self.prob[prefix] = e / e.sum()

    def __getitem__(self, prefix):
        return self.prob[tuple(prefix)]


def random_tables(rng, V, depth, concentration=0.7):
    """Context-dependent random conditionals (Dirichlet, kept away from zero)."""
    return TinyModel(V, depth, lambda prefix: rng.dirichlet(np.full(V, concentration)) * 0.98 + 0.02 / V)


def sparse_tables(rng, V, depth, p_zero=0.35):
    """Context-dependent random conditionals in which tokens are masked out (probability exactly zero,
    logit -inf) at random, as top-k / top-p warping does; every conditional keeps at least one token."""
    def requested(prefix):
        p = rng.dirichlet(np.full(V, 0.7)) * 0.98 + 0.02 / V
        keep = rng.random(V) >= p_zero
        if not keep.any():
            keep[rng.integers(V)] = True
        p = np.where(keep, p, 0.0)
        return p / p.sum()
    return TinyModel(V, depth, requested)


def constant_tables(probs, V, depth):
    return TinyModel(V, depth, lambda prefix: probs)


def joint(table, seq):
    """M^len(seq)(seq) = prod_j M(seq_j | seq^{j-1})."""
    out = 1.0
    for j, x in enumerate(seq):
        out *= table[tuple(seq[:j])][x]
    return out


def _rows(Mb, Ms, xs, gamma, form="logits"):
    src_b, src_s = (Mb.logits, Ms.logits) if form == "logits" else (Mb.prob, Ms.prob)
    tl = np.stack([src_b[tuple(xs[:i])] for i in range(gamma + 1)])
    dl = np.stack([src_s[tuple(xs[:i])] for i in range(gamma)])
    return tl, dl


def _run(form):
    """The oracle entry for a form of the inputs: "logits" (float32 logits, T = 1) or "probs" (the same
    models handed over as float64 probability rows)."""
    if form == "logits":
        return lambda algo, tl, dl, tok, uni: oracle.verify(algo, tl, dl, tok, uni, 1.0)
    return lambda algo, tl, dl, tok, uni: oracle.verify_probs(algo, tl, dl, tok, uni, dtype=oracle.F64)


def _f32_mid(lo, hi):
    """A float32 strictly inside (lo, hi), or None if the cell is too narrow."""
    m = np.float32(0.5 * (lo + hi))
    if lo < float(m) < hi and hi - lo > 4e-7:
        return m
    return None


def output_law(algo, Mb, Ms, V, gamma, form="logits"):
    """dict (xs, tau, Y) -> probability, plus per-draft debug blocks and the skipped volume."""
    run = _run(form)
    law = {}
    dbg_by_draft = {}
    skipped = 0.0
    for xs in itertools.product(range(V), repeat=gamma):
        if joint(Ms, xs) == 0.0:
            continue                                        # a draft the drafter never produces
        tl, dl = _rows(Mb, Ms, xs, gamma, form)
        tok = np.asarray(xs, dtype=np.int32)[None]
        probe = run(algo, tl[None], dl[None], tok, np.zeros((1, gamma + 1), np.float32))
        dbg = probe["dbg"][0]
        dbg_by_draft[xs] = dbg
        h = dbg[:, 2]
        w = dbg[:, 0]
        # breakpoints of u: every residual CDF that could be used (any tau, w_i or 1), and p_gamma
        P = np.stack([Mb[xs[:i]] for i in range(gamma + 1)])
        Q = np.stack([Ms[xs[:i]] for i in range(gamma)])
        cuts = {0.0, 1.0}
        for i in range(gamma):
            for wi in (w[i], 1.0):
                rho = np.maximum(wi * P[i] - Q[i], 0.0)
                if rho.sum() > 0:
                    cuts.update((np.cumsum(rho) / rho.sum()).tolist())
        cuts.update(np.cumsum(P[gamma]).tolist())
        cuts = sorted(c for c in cuts if 0.0 <= c <= 1.0)
        u_cells = [(a, b) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
        eta_cells = []
        for i in range(1, gamma + 1):
            hi = float(min(max(h[i], 0.0), 1.0))
            eta_cells.append([(0.0, hi), (hi, 1.0)])
        pts, vols = [], []
        for combo in itertools.product(*eta_cells):
            vol_eta = float(np.prod([b - a for a, b in combo]))
            if vol_eta == 0.0:
                continue
            mids = [_f32_mid(a, b) for a, b in combo]
            for (ua, ub) in u_cells:
                um = _f32_mid(ua, ub)
                vol = vol_eta * (ub - ua)
                if um is None or any(m is None for m in mids):
                    skipped += vol * joint(Ms, xs)
                    continue
                pts.append(mids + [um])
                vols.append(vol)
        n = len(pts)
        if n == 0:
            continue
        uni = np.asarray(pts, dtype=np.float32)
        out = run(algo, np.repeat(tl[None], n, 0), np.repeat(dl[None], n, 0), np.repeat(tok, n, 0), uni)
        assert out["n_fallback"] == 0
        ms = joint(Ms, xs)
        for k in range(n):
            key = (xs, int(out["accept_len"][k]), int(out["next_token"][k]))
            law[key] = law.get(key, 0.0) + ms * vols[k]
    return law, dbg_by_draft, skipped


def emitted_law(law, Mb, V, gamma, length=None):
    """Law of O = (X^tau, Y, Z...) truncated/extended to `length` tokens, Z ~ M_b."""
    length = gamma + 1 if length is None else length
    out = {}
    for (xs, tau, y), m in law.items():
        prefix = tuple(xs[:tau]) + (y,)
        for z in itertools.product(range(V), repeat=length - len(prefix)):
            seq = prefix + z
            pm = m
            for j in range(len(prefix), length):
                pm *= Mb[tuple(seq[:j])][seq[j]]
            out[seq] = out.get(seq, 0.0) + pm
    return out
