"""Seeded synthetic inputs for draft verification.

This module only *makes inputs*: logits, drafted tokens and uniforms.  It holds none
of the verification arithmetic and is the one module that both the CPU oracle's tests
and the HIP path's tests / benchmark import.  The paper's own workloads are language
model outputs on datasets that are not available here; the five configurations below
are synthetic stand-ins of the same shapes (batch, draft length gamma, vocabulary V,
logit dtype, temperature).

Recipe of one call (B sequences):
  * target logits [B, gamma+1, V] = sigma_t * N(0,1) (+ a Zipf-shaped bias
    -1.1*log(rank+1) over one seeded permutation of the vocabulary, shared by all rows);
  * draft logits  [B, gamma, V]   = the unrounded fp32 target rows 0..gamma-1
    + sigma_d * N(0,1); target and draft are then each rounded to the logit dtype
    (round-to-nearest-even for bf16);
  * draft token X_i is an inverse-CDF sample of softmax(draft row i-1 / T), computed
    in float64 from the rounded draft logits with its own uniform stream;
  * uniforms [B, gamma+1] are float32 multiples of 2^-24 in [0,1) from numpy's Philox
    generator keyed by the seed: eta_1..eta_gamma for the accept tests, then u for Y.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np
import torch


@dataclass(frozen=True)
class Config:
    name: str
    B: int
    gamma: int
    V: int
    dtype: str            # "f32" or "bf16"
    sigma_target: float
    sigma_draft: float
    temperature: float
    zipf: bool
    calls: int            # distinct input sets the configuration asks for

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2

    @property
    def algorithmic_bytes(self) -> int:
        """Every logit read once: B * (2*gamma+1) * V * sizeof(dtype)."""
        return self.B * (2 * self.gamma + 1) * self.V * self.elem_bytes


CONFIGS = {
    1: Config("cfg1_B1_g4_V1000_f32", 1, 4, 1000, "f32", 2.0, 0.5, 1.0, False, 10000),
    2: Config("cfg2_B8_g8_V32000_f32", 8, 8, 32000, "f32", 3.0, 1.0, 1.0, False, 1000),
    3: Config("cfg3_B64_g8_V128256_bf16", 64, 8, 128256, "bf16", 4.0, 1.5, 0.8, True, 8),
    4: Config("cfg4_B256_g16_V152064_bf16", 256, 16, 152064, "bf16", 4.0, 1.5, 1.0, True, 2),
    5: Config("cfg5_B1024_g8_V256000_bf16", 1024, 8, 256000, "bf16", 8.0, 2.0, 0.6, False, 1),
}
CFG4_DRAFT_SIGMAS = (0.5, 1.5, 3.0)


def with_overrides(cfg: Config, **kw) -> Config:
    return replace(cfg, **kw)


def torch_dtype(cfg: Config):
    return torch.float32 if cfg.dtype == "f32" else torch.bfloat16


def philox_uniforms(seed: int, shape) -> np.ndarray:
    """float32 multiples of 2^-24 in [0,1) from numpy's Philox bit generator."""
    rng = np.random.Generator(np.random.Philox(key=int(seed)))
    ints = rng.integers(0, 1 << 24, size=shape, dtype=np.int64)
    return (ints.astype(np.float64) * 2.0 ** -24).astype(np.float32)


def _zipf_bias(cfg: Config, seed: int, device) -> torch.Tensor:
    g = torch.Generator(device="cpu").manual_seed(int(seed) * 7919 + 17)
    perm = torch.randperm(cfg.V, generator=g)            # token id -> rank
    bias = -1.1 * torch.log(perm.to(torch.float64) + 1.0)
    return bias.to(torch.float32).to(device)


def generate(cfg: Config, seed: int, device="cpu", chunk_bytes: int = 1 << 30,
             top_k_target: int = 0, top_k_draft: int = 0) -> dict:
    """One call's inputs as torch tensors on `device`.

    Returns ``target_logits`` [B, gamma+1, V], ``draft_logits`` [B, gamma, V] (cfg dtype),
    ``draft_tokens`` [B, gamma] int32, ``uniforms`` [B, gamma+1] float32.
    The same (cfg, seed, device type) always gives the same tensors.
    `top_k_target` / `top_k_draft` > 0 keep only that many largest logits of every target / draft row and
    set the rest to -inf, the way top-k warping masks a distribution (draft tokens are then drawn from
    the masked draft rows; a drafted token may fall outside the target's support).
    """
    device = torch.device(device)
    B, g, V = cfg.B, cfg.gamma, cfg.V
    dt = torch_dtype(cfg)
    gen = torch.Generator(device=device).manual_seed(int(seed))
    target = torch.empty((B, g + 1, V), dtype=dt, device=device)
    draft = torch.empty((B, g, V), dtype=dt, device=device)
    tokens = torch.empty((B, g), dtype=torch.int32, device=device)
    bias = _zipf_bias(cfg, seed, device) if cfg.zipf else None

    # uniforms that draw the draft tokens: a stream of their own
    tok_u = torch.from_numpy(philox_uniforms(seed * 2 + 1, (B, g)).astype(np.float64)).to(device)

    per_seq = (2 * g + 1) * V * 8 * 3      # float64 temporaries dominate
    nb = max(1, min(B, chunk_bytes // per_seq))
    for b0 in range(0, B, nb):
        b1 = min(B, b0 + nb)
        t32 = torch.randn((b1 - b0, g + 1, V), generator=gen, device=device, dtype=torch.float32)
        t32.mul_(cfg.sigma_target)
        if bias is not None:
            t32.add_(bias)
        d32 = torch.randn((b1 - b0, g, V), generator=gen, device=device, dtype=torch.float32)
        d32.mul_(cfg.sigma_draft).add_(t32[:, :g, :])
        target[b0:b1] = t32.to(dt)
        draft[b0:b1] = d32.to(dt)
        del t32, d32
        for rows, keep in ((target[b0:b1], top_k_target), (draft[b0:b1], top_k_draft)):
            if 0 < keep < V:
                kth = torch.topk(rows.float(), keep, dim=-1).values[..., -1:]
                rows.masked_fill_(rows.float() < kth, float("-inf"))
        # X_i ~ softmax(draft row i-1 / T), inverse CDF in float64 on the rounded logits
        z = draft[b0:b1].to(torch.float64) / cfg.temperature
        z = torch.softmax(z, dim=-1)
        cdf = torch.cumsum(z, dim=-1)
        del z
        t = tok_u[b0:b1].unsqueeze(-1) * cdf[..., -1:]
        idx = torch.searchsorted(cdf, t, right=True).squeeze(-1).clamp_(max=V - 1)
        tokens[b0:b1] = idx.to(torch.int32)
        del cdf, t, idx

    uniforms = torch.from_numpy(philox_uniforms(seed * 2, (B, g + 1))).to(device)
    return {"target_logits": target, "draft_logits": draft,
            "draft_tokens": tokens, "uniforms": uniforms}


def logits_to_numpy(x: torch.Tensor) -> np.ndarray:
    """Host numpy view for the oracle: float32 as is, bf16 as uint16 bit patterns."""
    x = x.detach().cpu().contiguous()
    if x.dtype == torch.bfloat16:
        return x.view(torch.int16).numpy().view(np.uint16)
    return x.numpy()


def to_numpy(inputs: dict) -> dict:
    """All four input tensors as host numpy arrays in the form the oracle takes."""
    return {
        "target_logits": logits_to_numpy(inputs["target_logits"]),
        "draft_logits": logits_to_numpy(inputs["draft_logits"]),
        "draft_tokens": inputs["draft_tokens"].detach().cpu().numpy().astype(np.int32),
        "uniforms": inputs["uniforms"].detach().cpu().numpy().astype(np.float32),
    }
