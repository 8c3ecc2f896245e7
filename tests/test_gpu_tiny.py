"""The one-workgroup-per-sequence kernel (sequences whose 2 gamma + 1 rows fit into LDS together) against the CPU
oracle: forced through the testing hook, and as the library's own choice for such shapes."""
from __future__ import annotations

import numpy as np
import pytest
import torch

import paper_2403_10444_amd as sv
from paper_2403_10444_amd import binding
import oracle
import workloads
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda"
TINY = 5                     # spec_verify_debug_config path
MAX_FLOATS = 14336           # (2 gamma + 1) V that the kernel takes


@pytest.fixture(autouse=True)
def forced():
    sv.spec_verify_debug_config(TINY, -1)
    yield
    sv.spec_verify_debug_config(0, -1)


def _custom(B, gamma, V, dtype="f32", sigma_t=3.0, sigma_d=1.0, T=1.0, zipf=False):
    assert (2 * gamma + 1) * V <= MAX_FLOATS
    return workloads.Config(f"tiny_B{B}_g{gamma}_V{V}_{dtype}", B, gamma, V, dtype, sigma_t, sigma_d, T, zipf, 1)


SHAPES = [
    # B, gamma, V, dtype
    (1, 4, 1000, "f32"),        # configuration 1
    (300, 4, 1000, "f32"),
    (64, 8, 840, "bf16"),
    (33, 1, 4736, "bf16"),      # one position, the widest rows that fit
    (17, 2, 2816, "f32"),
    (40, 64, 111, "bf16"),      # the longest draft the library takes
    (25, 16, 64, "f32"),        # rows of one wave's width
    (9, 3, 3, "f32"),           # a vocabulary of three tokens
    (12, 5, 2, "bf16"),         # the worked example's vocabulary
    (50, 7, 777, "bf16"),       # nothing a multiple of anything
]


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("B,gamma,V,dtype", SHAPES)
def test_shapes(B, gamma, V, dtype, algo):
    cfg = _custom(B, gamma, V, dtype, sigma_t=2.5, sigma_d=0.8, T=0.9)
    for seed in (31, 32):
        inp = workloads.generate(cfg, seed=seed + B + gamma, device=DEV)
        rep = parity.compare(parity.run_gpu(algo, inp, cfg.temperature), parity.run_oracle(algo, inp, cfg.temperature),
                             label=f"{cfg.name}/{algo}/tiny", greedy=algo == "greedy")
        parity.record(rep)


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_the_librarys_own_choice_for_small_sequences_is_this_kernel(algo):
    """Without the hook the library takes this kernel for such shapes: same outputs, bit for bit, debug block included;
    the large kernel forced on the same inputs agrees with both on tau and Y."""
    cfg = _custom(200, 6, 1100, "bf16", sigma_t=3.0, sigma_d=1.0, T=0.8)
    inp = workloads.generate(cfg, seed=77, device=DEV)
    a = parity.run_gpu(algo, inp, cfg.temperature)
    sv.spec_verify_debug_config(0, -1)
    b = parity.run_gpu(algo, inp, cfg.temperature)
    assert sv.spec_verify_debug_last_kernel() == binding.SV_KERNEL_TINY
    sv.spec_verify_debug_config(3, -1)
    c = parity.run_gpu(algo, inp, cfg.temperature)
    assert sv.spec_verify_debug_last_kernel() == binding.SV_KERNEL_FUSED
    for key in ("accept_len", "next_token", "dbg"):
        assert np.array_equal(a[key], b[key], equal_nan=True), key
    ref = parity.run_oracle(algo, inp, cfg.temperature)
    safe = ref["margins"].min(axis=1) >= parity.MARGIN
    assert np.array_equal(a["accept_len"][safe], c["accept_len"][safe]) and np.array_equal(a["next_token"][safe], c["next_token"][safe])


def test_shapes_beyond_its_limit_are_refused_when_forced():
    cfg = workloads.Config("too_wide", 2, 4, 2000, "f32", 2.0, 1.0, 1.0, False, 1)       # 9 x 2000 logits > the limit
    inp = workloads.generate(cfg, seed=1, device=DEV)
    with pytest.raises(sv.SpecVerifyError) as e:
        sv.spec_verify_block(inp["target_logits"], inp["draft_logits"], inp["draft_tokens"], inp["uniforms"], 1.0)
    assert e.value.code == binding.SV_ERR_UNSUPPORTED


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_identical_models_accept_everything(algo):
    cfg = _custom(16, 5, 1200, "bf16", sigma_t=4.0)
    inp = workloads.generate(cfg, seed=5, device=DEV)
    inp["draft_logits"] = inp["target_logits"][:, :cfg.gamma].contiguous()
    gpu = parity.run_gpu(algo, inp, 0.7)
    assert np.all(gpu["accept_len"] == cfg.gamma)
    parity.compare(gpu, parity.run_oracle(algo, inp, 0.7), greedy=algo == "greedy")


@pytest.mark.parametrize("algo", ["block", "token"])
def test_disjoint_supports_reject_everything(algo):
    cfg = _custom(8, 4, 1024, "f32", sigma_t=1.0)
    inp = workloads.generate(cfg, seed=6, device=DEV)
    V = cfg.V
    inp["target_logits"][..., : V // 2] -= 60.0
    inp["draft_logits"][..., V // 2:] -= 60.0
    q = torch.softmax(inp["draft_logits"].double(), -1)
    inp["draft_tokens"] = torch.multinomial(q.view(-1, V), 1).view(cfg.B, cfg.gamma).to(torch.int32)
    gpu = parity.run_gpu(algo, inp, 1.0)
    assert np.all(gpu["accept_len"] == 0)
    assert np.all(gpu["next_token"] >= V // 2)
    parity.compare(gpu, parity.run_oracle(algo, inp, 1.0))


def test_uniform_extremes():
    cfg = _custom(6, 4, 1500, "bf16")
    inp = workloads.generate(cfg, seed=8, device=DEV)
    for value in (0.0, 1.0 - 2.0 ** -24):
        inp2 = dict(inp, uniforms=torch.full_like(inp["uniforms"], value))
        for algo in ("block", "token", "greedy"):
            parity.compare(parity.run_gpu(algo, inp2, 1.0), parity.run_oracle(algo, inp2, 1.0))


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("kt,kd", [(50, 50), (20, 200), (500, 5), (1, 40)])
def test_masked_logits_top_k(algo, kt, kd):
    cfg = _custom(16, 6, 1100, "bf16", sigma_t=3.0, sigma_d=1.0, T=0.9)
    inp = workloads.generate(cfg, seed=300 + kt + kd, device=DEV, top_k_target=kt, top_k_draft=kd)
    assert torch.isinf(inp["target_logits"]).any() and torch.isinf(inp["draft_logits"]).any()
    parity.compare(parity.run_gpu(algo, inp, cfg.temperature), parity.run_oracle(algo, inp, cfg.temperature),
                   greedy=(algo == "greedy"))


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("B,gamma,V,dtype", [(24, 8, 840, "bf16"), (9, 5, 1291, "f32"), (130, 16, 300, "bf16")])
def test_ragged_draft_lengths(algo, B, gamma, V, dtype):
    """Sequence b must come out exactly as a call with gamma = draft_lens[b] on its leading rows does; the rows beyond
    a sequence's length are poisoned with NaN to show that they are never read."""
    cfg = _custom(B, gamma, V, dtype, sigma_t=2.5, sigma_d=1.0, T=0.8)
    inp = workloads.generate(cfg, seed=500 + B + gamma, device=DEV)
    rng = np.random.default_rng(B * gamma)
    lens = rng.integers(1, gamma + 1, size=B).astype(np.int32)
    lens[0], lens[-1] = gamma, 1
    tl, dl = inp["target_logits"].clone(), inp["draft_logits"].clone()
    for b in range(B):
        tl[b, lens[b] + 1:] = float("nan")
        dl[b, lens[b]:] = float("nan")
    tau, y = sv.spec_verify_ex(algo, tl, dl, inp["draft_tokens"], inp["uniforms"], cfg.temperature,
                               draft_lens=torch.as_tensor(lens, device=DEV))
    torch.cuda.synchronize()
    tau, y = tau.cpu().numpy(), y.cpu().numpy()
    host = workloads.to_numpy(inp)
    odt = oracle.BF16 if dtype == "bf16" else oracle.F32
    n_safe = 0
    for g in np.unique(lens):
        sel = np.nonzero(lens == g)[0]
        ref = oracle.verify(parity.ALGOS[algo][0], host["target_logits"][sel, :g + 1], host["draft_logits"][sel, :g],
                            host["draft_tokens"][sel, :g], host["uniforms"][sel, :g + 1], cfg.temperature, dtype=odt)
        safe = ref["margins"].min(axis=1) >= parity.MARGIN
        n_safe += int(safe.sum())
        assert np.array_equal(tau[sel][safe], ref["accept_len"][safe]), (g, algo)
        same_tau = safe & (tau[sel] == ref["accept_len"])
        assert np.array_equal(y[sel][same_tau], ref["next_token"][same_tau]), (g, algo)
        assert np.all(tau[sel] <= g)
    assert n_safe >= 0.8 * B


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("B,gamma,V,dtype,pad_t,pad_d", [(16, 8, 800, "bf16", 96, 32), (7, 4, 1191, "f32", 1, 9),
                                                          (70, 2, 2800, "bf16", 3, 5)])
def test_padded_rows(algo, B, gamma, V, dtype, pad_t, pad_d):
    """Rows inside buffers whose last dimension is padded (stride > V); the padding is poisoned with NaN."""
    cfg = _custom(B, gamma, V, dtype, sigma_t=2.5, sigma_d=1.0, T=0.8)
    inp = workloads.generate(cfg, seed=700 + B + gamma, device=DEV)
    tbuf = torch.full((B, gamma + 1, V + pad_t), float("nan"), dtype=inp["target_logits"].dtype, device=DEV)
    dbuf = torch.full((B, gamma, V + pad_d), float("nan"), dtype=inp["draft_logits"].dtype, device=DEV)
    tbuf[..., :V] = inp["target_logits"]
    dbuf[..., :V] = inp["draft_logits"]
    tau, y = sv.spec_verify_ex(algo, tbuf[..., :V], dbuf[..., :V], inp["draft_tokens"], inp["uniforms"], cfg.temperature)
    torch.cuda.synchronize()
    ref = parity.run_oracle(algo, inp, cfg.temperature)
    safe = ref["margins"].min(axis=1) >= parity.MARGIN
    assert safe.sum() >= 0.8 * B
    assert np.array_equal(tau.cpu().numpy()[safe], ref["accept_len"][safe])
    assert np.array_equal(y.cpu().numpy()[safe], ref["next_token"][safe])


def test_workspace_must_be_initialised_for_the_shape():
    """This kernel needs nothing of the workspace, but the contract is one: a workspace prepared for another shape
    gives -1 outputs."""
    cfg = _custom(4, 3, 500, "f32")
    inp = workloads.generate(cfg, seed=3, device=DEV)
    ws = sv.alloc_workspace(cfg.B, cfg.gamma + 1, cfg.V, DEV)
    tau, y = sv.spec_verify_block(inp["target_logits"], inp["draft_logits"], inp["draft_tokens"], inp["uniforms"], 1.0,
                                  workspace=ws)
    torch.cuda.synchronize()
    assert bool((tau == -1).all()) and bool((y == -1).all())
