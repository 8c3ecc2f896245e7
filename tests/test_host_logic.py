"""Host-side logic that needs no GPU: the workload table, the bench's refusal of more than one GPU, the binding's
refusal to run without the built library, and the profile summaries' parsers."""
from __future__ import annotations

import os
import subprocess
import sys

import pytest

import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_algorithmic_bytes_per_call_are_every_logit_once():
    """B (2 gamma + 1) V sizeof(dtype): the figure the roofline line divides by."""
    want = {1: 36_000, 2: 17_408_000, 3: 279_085_056, 4: 2_569_273_344, 5: 8_912_896_000}
    for cfg_id, nbytes in want.items():
        cfg = workloads.CONFIGS[cfg_id]
        size = 2 if cfg.dtype == "bf16" else 4
        assert cfg.algorithmic_bytes == nbytes == cfg.B * (2 * cfg.gamma + 1) * cfg.V * size


def test_headline_workload_is_the_quoted_configuration():
    cfg = workloads.CONFIGS[3]
    assert (cfg.B, cfg.gamma, cfg.V, cfg.dtype) == (64, 8, 128256, "bf16") and cfg.temperature == pytest.approx(0.8)


@pytest.mark.parametrize("extra_env", [{}, {"WORLD_SIZE": "2"}])
def test_bench_refuses_more_than_one_gpu(extra_env):
    env = dict(os.environ, **extra_env)
    args = [sys.executable, os.path.join(ROOT, "bench.py"), "--steps", "1", "--warmup", "0"]
    if not extra_env:
        args += ["--gpus", "2"]
    out = subprocess.run(args, env=env, capture_output=True, text=True, timeout=300)
    assert out.returncode != 0
    assert "one GPU" in out.stderr or "--gpus 1" in out.stderr
    assert out.stdout.strip() == ""                       # no JSON line for a run that did not happen


def test_binding_fails_loudly_without_the_built_library(monkeypatch, tmp_path):
    import paper_2403_10444_amd.binding as binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libspecverify.so"))
    with pytest.raises((OSError, RuntimeError)):
        binding.load()
