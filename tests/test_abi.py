"""The C-ABI library loads and exports what include/specverify.h declares; argument
validation is host-side and runs without a GPU (no kernel is launched in this file)."""
from __future__ import annotations

import ctypes
import os
import re

import pytest

import paper_2403_10444_amd as sv
from paper_2403_10444_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "specverify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    # what only a tuning build of the library exports is not part of the product ABI
    text = re.sub(r"#ifdef SPECVERIFY_PROFILE_BUILD.*?#endif", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spec_(?:verify|sample)_\w+)\s*\(", text)))


def test_header_and_library_agree_on_exports():
    lib = sv.load()
    declared = _declared_functions()
    assert declared == sorted(binding.EXPORTED)
    for name in declared:
        assert hasattr(lib, name), name


def test_workspace_query():
    assert sv.spec_verify_workspace_bytes(64, 8, 128256) > 0
    assert sv.spec_verify_workspace_bytes(64, 8, 128256) % 256 == 0
    assert sv.spec_verify_workspace_bytes(0, 8, 128256) == 0
    assert sv.spec_verify_workspace_bytes(1, 0, 10) == 0
    assert sv.spec_verify_workspace_bytes(1, 1, 0) == 0
    assert sv.spec_verify_workspace_bytes(1, 65, 10) == 0          # above SV_MAX_GAMMA
    assert sv.spec_verify_workspace_bytes(1 << 20, 64, 1 << 30) == 0  # grid would overflow


def _raw(name, *, B=2, gamma=3, V=100, dtype=0, T=1.0, ws=0x1000, ws_bytes=1 << 30,
         target=0x1000, draft=0x1000, tokens=0x1000, uniforms=0x1000, tau=0x1000, y=0x1000):
    # fake non-null pointers: validation must reject the call before anything is dereferenced
    lib = sv.load()
    return getattr(lib, name)(target, draft, tokens, uniforms, B, gamma, V, dtype, T, ws, ws_bytes,
                              tau, y, None, None)


@pytest.mark.parametrize("name", ["spec_verify_block", "spec_verify_token", "spec_verify_greedy"])
def test_argument_validation_returns_codes(name):
    assert _raw(name, B=0) == binding.SV_ERR_INVALID_ARG
    assert _raw(name, gamma=0) == binding.SV_ERR_INVALID_ARG
    assert _raw(name, V=0) == binding.SV_ERR_INVALID_ARG
    assert _raw(name, T=0.0) == binding.SV_ERR_INVALID_ARG
    assert _raw(name, T=-1.0) == binding.SV_ERR_INVALID_ARG
    assert _raw(name, T=float("inf")) == binding.SV_ERR_INVALID_ARG
    assert _raw(name, T=float("nan")) == binding.SV_ERR_INVALID_ARG
    assert _raw(name, dtype=7) == binding.SV_ERR_INVALID_ARG
    assert _raw(name, target=None) == binding.SV_ERR_INVALID_ARG
    assert _raw(name, tau=None) == binding.SV_ERR_INVALID_ARG
    assert _raw(name, ws=None) == binding.SV_ERR_INVALID_ARG
    assert _raw(name, ws=0x1010) == binding.SV_ERR_INVALID_ARG       # workspace not 256-byte aligned
    assert _raw(name, gamma=65) == binding.SV_ERR_UNSUPPORTED
    assert _raw(name, ws_bytes=16) == binding.SV_ERR_WORKSPACE_TOO_SMALL


def test_workspace_init_validates_on_the_host():
    lib = sv.load()
    assert lib.spec_verify_workspace_init(None, 1 << 30, 2, 3, 100, None) == binding.SV_ERR_INVALID_ARG
    assert lib.spec_verify_workspace_init(0x1010, 1 << 30, 2, 3, 100, None) == binding.SV_ERR_INVALID_ARG
    assert lib.spec_verify_workspace_init(0x1000, 1 << 30, 0, 3, 100, None) == binding.SV_ERR_INVALID_ARG
    assert lib.spec_verify_workspace_init(0x1000, 1 << 30, 2, 65, 100, None) == binding.SV_ERR_UNSUPPORTED
    assert lib.spec_verify_workspace_init(0x1000, 16, 2, 3, 100, None) == binding.SV_ERR_WORKSPACE_TOO_SMALL
    assert lib.spec_verify_workspace_check(None, 2, 3, 100, None) == binding.SV_ERR_INVALID_ARG


def test_forcing_the_fused_path_refuses_vocabularies_it_cannot_take():
    try:
        sv.spec_verify_debug_config(2, -1)
        assert _raw("spec_verify_block", V=128 * 8192 + 1) == binding.SV_ERR_UNSUPPORTED
        sv.spec_verify_debug_config(0, -1)
        assert _raw("spec_verify_block", V=128 * 8192 + 1, ws_bytes=16) == binding.SV_ERR_WORKSPACE_TOO_SMALL
    finally:
        sv.spec_verify_debug_config(0, -1)


def test_status_strings():
    seen = {sv.status_string(c) for c in range(6)}
    assert len(seen) == 6 and "ok" in seen
    assert sv.status_string(99) == "unknown status"


def test_binding_refuses_cpu_tensors():
    import torch
    t = torch.zeros((1, 2, 8))
    with pytest.raises(ValueError):
        sv.spec_verify_block(t, t[:, :1], torch.zeros((1, 1), dtype=torch.int32), torch.zeros((1, 2)), 1.0)


def test_copy_probe_validates_its_arguments():
    lib = sv.load()
    assert lib.spec_verify_debug_copy(None, 0x1000, 256, None) == binding.SV_ERR_INVALID_ARG
    assert lib.spec_verify_debug_copy(0x1000, None, 256, None) == binding.SV_ERR_INVALID_ARG
    assert lib.spec_verify_debug_copy(0x1000, 0x2000, 0, None) == binding.SV_ERR_INVALID_ARG
    assert lib.spec_verify_debug_copy(0x1000, 0x2000, 24, None) == binding.SV_ERR_INVALID_ARG      # not a multiple of 16
    assert lib.spec_verify_debug_copy(0x1008, 0x2000, 256, None) == binding.SV_ERR_INVALID_ARG    # misaligned


def test_stream_probe_validates_its_arguments():
    lib = sv.load()

    def call(a=0x10000, b=0x20000, nbytes=16384, out=0x30000, short=0, long=0):
        return lib.spec_verify_debug_stream_probe(a, b, nbytes, out, short, long, None)

    assert call(a=None) == binding.SV_ERR_INVALID_ARG
    assert call(b=None) == binding.SV_ERR_INVALID_ARG
    assert call(out=None) == binding.SV_ERR_INVALID_ARG
    assert call(nbytes=0) == binding.SV_ERR_INVALID_ARG
    assert call(nbytes=16384 + 16) == binding.SV_ERR_INVALID_ARG       # whole workgroups only
    assert call(a=0x10008) == binding.SV_ERR_INVALID_ARG               # misaligned
    assert call(short=-1) == binding.SV_ERR_INVALID_ARG
    assert call(long=65) == binding.SV_ERR_INVALID_ARG


def test_sample_tokens_validates_its_arguments():
    lib = sv.load()
    ok = dict(logits=0x1000, rows=4, V=10, dtype=0, T=1.0, uniforms=0x1000, tokens=0x1000)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.spec_sample_tokens(a["logits"], a["rows"], a["V"], a["dtype"], a["T"], a["uniforms"], a["tokens"], None)

    assert call(logits=None) == binding.SV_ERR_INVALID_ARG
    assert call(uniforms=None) == binding.SV_ERR_INVALID_ARG
    assert call(tokens=None) == binding.SV_ERR_INVALID_ARG
    assert call(rows=0) == binding.SV_ERR_INVALID_ARG
    assert call(V=0) == binding.SV_ERR_INVALID_ARG
    assert call(T=0.0) == binding.SV_ERR_INVALID_ARG
    assert call(T=float("nan")) == binding.SV_ERR_INVALID_ARG
    assert call(dtype=5) == binding.SV_ERR_INVALID_ARG
    assert call(rows=1 << 31) == binding.SV_ERR_UNSUPPORTED


def test_extended_entry_validates_its_arguments():
    lib = sv.load()

    def call(algo=0, lens=0x1000, B=2, ts=0, ds=0):
        return lib.spec_verify_ex(algo, 0x1000, 0x1000, 0x1000, lens, ts, ds, 0x1000, B, 3, 100, 0, 1.0, 0x1000,
                                  1 << 30, 0x1000, 0x1000, None, None)

    assert call(algo=3) == binding.SV_ERR_INVALID_ARG
    assert call(B=0) == binding.SV_ERR_INVALID_ARG
    assert call(ts=99) == binding.SV_ERR_INVALID_ARG       # a stride below V
    assert call(ds=-1) == binding.SV_ERR_INVALID_ARG


def test_probs_entry_validates_its_arguments():
    lib = sv.load()

    def call(algo=0, target=0x1000, B=2, ts=0, dtype=0, ws_bytes=1 << 30):
        return lib.spec_verify_probs(algo, target, 0x1000, 0x1000, None, ts, 0, 0x1000, B, 3, 100, dtype, 0x1000,
                                     ws_bytes, 0x1000, 0x1000, None, None)

    assert call(algo=7) == binding.SV_ERR_INVALID_ARG
    assert call(target=None) == binding.SV_ERR_INVALID_ARG
    assert call(B=0) == binding.SV_ERR_INVALID_ARG
    assert call(ts=50) == binding.SV_ERR_INVALID_ARG
    assert call(dtype=9) == binding.SV_ERR_INVALID_ARG
    assert call(ws_bytes=16) == binding.SV_ERR_WORKSPACE_TOO_SMALL
