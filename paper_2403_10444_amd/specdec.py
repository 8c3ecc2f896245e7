"""The outer loop of speculative decoding (Alg. 3) on the device, for context-independent toy models.

Sec. 2 illustrates block verification with models that ignore the context: every conditional
distribution of a model is the same vector.  Then the loop's three steps per iteration - draft gamma
tokens from M_s, score them with both models, verify - need no language model: scoring is repeating
two logit vectors.  Drafting and verification run in the library's kernels (`spec_sample_tokens`,
`spec_verify_*`); this module only arranges buffers and feeds the uniforms.  With context-independent
models the iterations are independent draws, so B sequences x `iters` iterations give B * iters
samples of the accepted length tau: enough to reproduce the complementary CDF of tau (the paper's
figure for gamma = 10) and the block efficiency E[tau] + 1 against gamma.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding

_VERIFY = {"block": binding.spec_verify_block, "token": binding.spec_verify_token, "greedy": binding.spec_verify_greedy}


def toy_speculative_decoding(algo: str, target_logits, draft_logits, gamma: int, B: int, iters: int,
                             temperature: float, uniforms, device="cuda"):
    """Runs `iters` iterations of Alg. 3 for B sequences of two context-independent models.

    target_logits, draft_logits: [V] float32.  `uniforms(it)` returns the iteration's two host arrays,
    draft uniforms [B, gamma] and verification uniforms [B, gamma + 1] (float32 in [0, 1)): the random
    numbers are inputs, so that a reference implementation can be fed the same ones.
    Returns numpy arrays tau [iters, B], y [iters, B], x [iters, B, gamma].
    """
    dev = torch.device(device)
    t = torch.as_tensor(np.asarray(target_logits, dtype=np.float32), device=dev)
    d = torch.as_tensor(np.asarray(draft_logits, dtype=np.float32), device=dev)
    V = t.numel()
    tl = t.expand(B, gamma + 1, V).contiguous()           # "parallel scoring": every row is the same vector
    dl = d.expand(B, gamma, V).contiguous()
    ws = binding.alloc_workspace(B, gamma, V, dev)
    x = torch.empty((B, gamma), dtype=torch.int32, device=dev)
    tau = torch.empty(B, dtype=torch.int32, device=dev)
    y = torch.empty(B, dtype=torch.int32, device=dev)
    taus, ys, xs = [], [], []
    for it in range(iters):
        u_draft, u_verify = uniforms(it)
        ud = torch.as_tensor(u_draft, device=dev)
        uv = torch.as_tensor(u_verify, device=dev)
        binding.spec_sample_tokens(dl, ud, temperature, tokens=x)
        _VERIFY[algo](tl, dl, x, uv, temperature, workspace=ws, accept_len=tau, next_token=y)
        taus.append(tau.cpu().numpy().copy()); ys.append(y.cpu().numpy().copy()); xs.append(x.cpu().numpy().copy())
    return {"tau": np.stack(taus), "y": np.stack(ys), "x": np.stack(xs)}


def _main():
    """Prints the block efficiency E[tau] + 1 against gamma and the complementary CDF of tau at gamma = 10 for the
    toy models of Sec. 2 (M_b = (1/3, 2/3), M_s = (2/3, 1/3)), measured on the device."""
    import workloads
    mb, ms = np.log(np.array([1 / 3, 2 / 3])), np.log(np.array([2 / 3, 1 / 3]))
    B, iters = 8192, 32

    def uniforms_for(gamma, seed):
        def f(it):
            u = workloads.philox_uniforms(seed * 100003 + it, (B, 2 * gamma + 1))
            return np.ascontiguousarray(u[:, :gamma]), np.ascontiguousarray(u[:, gamma:])
        return f

    print(f"toy models of Sec. 2, {B * iters} draws per cell")
    print("gamma   token   block   greedy   (block efficiency E[tau] + 1)")
    keep = {}
    for gamma in (4, 6, 8, 10):
        row = []
        for algo in ("token", "block", "greedy"):
            r = toy_speculative_decoding(algo, mb, ms, gamma, B, iters, 1.0, uniforms_for(gamma, 17))
            row.append(1.0 + r["tau"].mean())
            keep[algo, gamma] = r["tau"].reshape(-1)
        print(f"{gamma:5d}  {row[0]:.4f}  {row[1]:.4f}  {row[2]:.4f}")
    print("Pr(tau >= k) at gamma = 10, k = 0 .. 10")
    for algo in ("token", "block"):
        print(f"{algo:6s}", " ".join(f"{(keep[algo, 10] >= k).mean():.4f}" for k in range(11)))


if __name__ == "__main__":
    _main()
