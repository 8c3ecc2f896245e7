"""The entry point that allocates nothing (spec_verify_ex_noalloc, for callers that cannot allocate device memory):
its results on the library's built-in scratch memory equal those of spec_verify_ex on a workspace."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import paper_2403_10444_amd as sv
import workloads

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _cfg(B, gamma, V, dtype="bf16"):
    return workloads.Config(f"noalloc_B{B}_g{gamma}_V{V}_{dtype}", B, gamma, V, dtype, 2.5, 1.0, 0.9, False, 1)


def _both(algo, cfg, seed, draft_lens=None):
    inp = workloads.generate(cfg, seed=seed, device=DEV)
    shape = (cfg.B, cfg.gamma + 1, 3)
    dbg_a = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    dbg_b = torch.full(shape, float("nan"), dtype=torch.float32, device=DEV)
    tau_a, y_a = sv.spec_verify_ex(algo, inp["target_logits"], inp["draft_logits"], inp["draft_tokens"], inp["uniforms"],
                                   cfg.temperature, draft_lens=draft_lens, debug_out=dbg_a)
    tau_b = torch.full((cfg.B,), -7, dtype=torch.int32, device=DEV)
    y_b = torch.full((cfg.B,), -7, dtype=torch.int32, device=DEV)
    sv.spec_verify_ex_noalloc(algo, inp["target_logits"], inp["draft_logits"], inp["draft_tokens"], inp["uniforms"],
                              cfg.temperature, tau_b, y_b, draft_lens=draft_lens, debug_out=dbg_b)
    # and once more without the debug block (the kernels then leave out what cannot matter)
    tau_c = torch.full((cfg.B,), -7, dtype=torch.int32, device=DEV)
    y_c = torch.full((cfg.B,), -7, dtype=torch.int32, device=DEV)
    sv.spec_verify_ex_noalloc(algo, inp["target_logits"], inp["draft_logits"], inp["draft_tokens"], inp["uniforms"],
                              cfg.temperature, tau_c, y_c, draft_lens=draft_lens)
    torch.cuda.synchronize()
    assert torch.all((tau_a >= 0) & (tau_a <= cfg.gamma)) and torch.all((y_a >= 0) & (y_a < cfg.V))
    assert torch.equal(tau_a, tau_b) and torch.equal(y_a, y_b), (algo, cfg.name)
    assert torch.equal(tau_a, tau_c) and torch.equal(y_a, y_c), (algo, cfg.name)
    a, b = dbg_a.cpu().numpy(), dbg_b.cpu().numpy()
    assert np.array_equal(a, b, equal_nan=True), (algo, cfg.name)


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_two_calls_in_a_row_the_second_one_smaller(algo):
    """The scratch array keeps what the first call left; the second call has another, smaller shape."""
    _both(algo, _cfg(24, 6, 40000), seed=31)
    _both(algo, _cfg(5, 3, 9000), seed=32)
    _both(algo, _cfg(5, 3, 9000), seed=33)          # the same shape again: nothing is prepared anew
    _both(algo, _cfg(24, 6, 40000), seed=34)        # and back to the larger one


def test_draft_lengths_and_float_rows():
    lens = torch.tensor([1 + (b * 3) % 5 for b in range(12)], dtype=torch.int32, device=DEV)
    _both("block", _cfg(12, 5, 8191, "f32"), seed=35, draft_lens=lens)


def test_sizes_beyond_the_built_in_scratch_are_refused():
    B, gamma, V = 1024, 8, 256000
    assert sv.spec_verify_workspace_bytes(B, gamma, V) > sv.binding.SV_STATIC_SCRATCH_BYTES
    lib = sv.load()
    fake = 0x1000          # refused before anything is dereferenced
    rc = lib.spec_verify_ex_noalloc(0, fake, fake, fake, None, 0, 0, fake, B, gamma, V, 1, 1.0, fake, fake, None, None)
    assert rc == sv.binding.SV_ERR_STATIC_SCRATCH_TOO_SMALL
    assert "scratch" in sv.status_string(rc)
