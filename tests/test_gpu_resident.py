"""The kernel for calls whose workgroups all run at once (every workgroup of a row forms the row's S_i, the one that
holds the token draws it from its registers) against the CPU oracle: forced through the testing hook, as the library's
own choice for such calls, and in turns with the large kernel on one workspace."""
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
RESIDENT = 7                 # spec_verify_debug_config path
FUSED = 3                    # the large kernel, small units


@pytest.fixture(autouse=True)
def forced():
    sv.spec_verify_debug_config(RESIDENT, -1)
    yield
    sv.spec_verify_debug_config(0, -1)


def _custom(B, gamma, V, dtype="bf16", sigma_t=3.0, sigma_d=1.0, T=1.0, zipf=False):
    return workloads.Config(f"resident_B{B}_g{gamma}_V{V}_{dtype}", B, gamma, V, dtype, sigma_t, sigma_d, T, zipf, 1)


SHAPES = [
    # B, gamma, V, dtype
    (8, 8, 32000, "f32"),       # configuration 2
    (8, 4, 32000, "bf16"),
    (3, 1, 1, "f32"),           # one-token vocabulary
    (3, 2, 7, "bf16"),          # tiny, unaligned rows
    (5, 3, 8191, "f32"),        # one element short of a workgroup's chunk, unaligned
    (5, 3, 8192, "bf16"),       # exactly one chunk
    (4, 2, 8200, "bf16"),       # a chunk and a ragged tail, aligned
    (4, 5, 16389, "bf16"),      # unaligned, three chunks
    (2, 4, 50001, "f32"),       # unaligned, odd
    (2, 64, 2048, "bf16"),      # the longest draft the library takes
    (1, 8, 128256, "bf16"),     # one sequence of the headline shape
    (1, 2, 262144, "f32"),      # the widest rows it takes: 32 workgroups
    (2, 1, 262100, "bf16"),
    (100, 1, 1024, "bf16"),     # many sequences of one workgroup per row
    (12, 6, 30000, "bf16"),
    # more workgroups than run at once: what cannot matter is left out, last target rows are read only where needed
    (40, 8, 32000, "bf16"),
    (12, 8, 128256, "bf16"),
    (90, 3, 20001, "f32"),
]


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("B,gamma,V,dtype", SHAPES)
def test_shapes(B, gamma, V, dtype, algo):
    cfg = _custom(B, gamma, V, dtype, sigma_t=2.5, sigma_d=0.8, T=0.9)
    for seed in (41, 42):
        inp = workloads.generate(cfg, seed=seed + B + gamma, device=DEV)
        rep = parity.compare(parity.run_gpu(algo, inp, cfg.temperature), parity.run_oracle(algo, inp, cfg.temperature),
                             label=f"{cfg.name}/{algo}/resident", greedy=algo == "greedy")
        parity.record(rep)


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_configuration_2_two_seeds(algo):
    cfg = workloads.CONFIGS[2]
    for seed in (2000, 2001):
        inp = workloads.generate(cfg, seed=seed, device=DEV)
        rep = parity.compare(parity.run_gpu(algo, inp, cfg.temperature), parity.run_oracle(algo, inp, cfg.temperature),
                             label=f"cfg2/seed{seed}/{algo}/resident", greedy=algo == "greedy")
        parity.record(rep)


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_the_librarys_own_choice_for_calls_of_one_resident_set_is_this_kernel(algo):
    """Without the hook the library takes this kernel where the call's workgroups all run at once: same outputs, bit for
    bit, debug block included; the large kernel forced on the same inputs agrees with both on tau and Y (its residual
    masses are sums in another order)."""
    cfg = _custom(12, 6, 20000, "bf16", sigma_t=3.0, sigma_d=1.0, T=0.8)
    inp = workloads.generate(cfg, seed=78, device=DEV)
    a = parity.run_gpu(algo, inp, cfg.temperature)
    assert sv.spec_verify_debug_last_kernel() == binding.SV_KERNEL_RESIDENT
    sv.spec_verify_debug_config(0, -1)
    b = parity.run_gpu(algo, inp, cfg.temperature)
    assert sv.spec_verify_debug_last_kernel() == binding.SV_KERNEL_RESIDENT
    sv.spec_verify_debug_config(FUSED, -1)
    c = parity.run_gpu(algo, inp, cfg.temperature)
    assert sv.spec_verify_debug_last_kernel() == binding.SV_KERNEL_FUSED
    for key in ("accept_len", "next_token", "dbg"):
        assert np.array_equal(a[key], b[key], equal_nan=True), key
    assert not np.array_equal(a["dbg"], c["dbg"], equal_nan=True)          # (another summation order: another kernel ran)
    ref = parity.run_oracle(algo, inp, cfg.temperature)
    safe = ref["margins"].min(axis=1) >= parity.MARGIN
    assert np.array_equal(a["accept_len"][safe], c["accept_len"][safe]) and np.array_equal(a["next_token"][safe], c["next_token"][safe])


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_in_turns_with_the_large_kernel_on_one_workspace(algo):
    """The two kernels share the control words and the call count of a workspace: calls of either may follow each
    other, in any order, and every call gives what it gives on a fresh workspace."""
    cfg = _custom(9, 5, 12000, "bf16", sigma_t=2.5, sigma_d=1.0, T=0.8)
    ws = sv.alloc_workspace(cfg.B, cfg.gamma, cfg.V, DEV)
    order = [RESIDENT, FUSED, FUSED, RESIDENT, RESIDENT, FUSED, RESIDENT, 4, RESIDENT, FUSED]          # (4: the large kernel with its large units)
    for n, path in enumerate(order):
        inp = workloads.generate(cfg, seed=900 + n, device=DEV)
        sv.spec_verify_debug_config(path, -1)
        got = parity.run_gpu(algo, inp, cfg.temperature, workspace=ws)
        assert binding.spec_verify_workspace_check(ws, cfg.B, cfg.gamma, cfg.V) == binding.SV_OK
        parity.compare(got, parity.run_oracle(algo, inp, cfg.temperature), label=f"turn{n}/path{path}", greedy=algo == "greedy")


def test_calls_beyond_its_limits_are_refused_when_forced_and_go_to_the_large_kernel_otherwise():
    for B, gamma, V in ((400, 8, 32000), (1, 1, 270000)):       # more workgroups than run at once; rows of 33 workgroups
        cfg = workloads.Config("not_resident", B, gamma, V, "bf16", 2.0, 1.0, 1.0, False, 1)
        inp = workloads.generate(cfg, seed=1, device=DEV)
        with pytest.raises(sv.SpecVerifyError) as e:
            sv.spec_verify_block(inp["target_logits"], inp["draft_logits"], inp["draft_tokens"], inp["uniforms"], 1.0)
        assert e.value.code == binding.SV_ERR_UNSUPPORTED
        sv.spec_verify_debug_config(0, -1)
        parity.compare(parity.run_gpu("block", inp, 1.0), parity.run_oracle("block", inp, 1.0))
        assert sv.spec_verify_debug_last_kernel() == binding.SV_KERNEL_FUSED
        sv.spec_verify_debug_config(RESIDENT, -1)


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("B,gamma", [(6, 5), (6, 64), (60, 8)])           # (60 x 9 x 3 workgroups: more than run at once)
def test_identical_models_accept_everything(algo, B, gamma):
    cfg = _custom(B, gamma, 9000 if B == 6 else 20000, "bf16", sigma_t=4.0)
    inp = workloads.generate(cfg, seed=5, device=DEV)
    inp["draft_logits"] = inp["target_logits"][:, :cfg.gamma].contiguous()
    gpu = parity.run_gpu(algo, inp, 0.7)
    assert np.all(gpu["accept_len"] == cfg.gamma)
    parity.compare(gpu, parity.run_oracle(algo, inp, 0.7), greedy=algo == "greedy")


@pytest.mark.parametrize("algo", ["block", "token"])
def test_disjoint_supports_reject_everything(algo):
    cfg = _custom(8, 4, 4096, "f32", sigma_t=1.0)
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
    cfg = _custom(6, 4, 15000, "bf16")
    inp = workloads.generate(cfg, seed=8, device=DEV)
    for value in (0.0, 1.0 - 2.0 ** -24):
        inp2 = dict(inp, uniforms=torch.full_like(inp["uniforms"], value))
        for algo in ("block", "token", "greedy"):
            parity.compare(parity.run_gpu(algo, inp2, 1.0), parity.run_oracle(algo, inp2, 1.0))


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("kt,kd", [(50, 50), (20, 200), (500, 5), (1, 40)])
def test_masked_logits_top_k(algo, kt, kd):
    cfg = _custom(16, 6, 11000, "bf16", sigma_t=3.0, sigma_d=1.0, T=0.9)
    inp = workloads.generate(cfg, seed=300 + kt + kd, device=DEV, top_k_target=kt, top_k_draft=kd)
    assert torch.isinf(inp["target_logits"]).any() and torch.isinf(inp["draft_logits"]).any()
    parity.compare(parity.run_gpu(algo, inp, cfg.temperature), parity.run_oracle(algo, inp, cfg.temperature),
                   greedy=(algo == "greedy"))


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("B,gamma,V,dtype", [(24, 8, 8400, "bf16"), (9, 5, 12917, "f32"), (40, 16, 3000, "bf16"), (50, 8, 30000, "bf16")])
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
    ws = sv.alloc_workspace(B, gamma, V, DEV)
    host = workloads.to_numpy(inp)
    odt = oracle.BF16 if dtype == "bf16" else oracle.F32
    # twice on one workspace, the second time after a call of the large kernel that used every position
    for turn in range(2):
        tau, y = sv.spec_verify_ex(algo, tl, dl, inp["draft_tokens"], inp["uniforms"], cfg.temperature,
                                   draft_lens=torch.as_tensor(lens, device=DEV), workspace=ws)
        torch.cuda.synchronize()
        tau, y = tau.cpu().numpy(), y.cpu().numpy()
        n_safe = 0
        for g in np.unique(lens):
            sel = np.nonzero(lens == g)[0]
            ref = oracle.verify(parity.ALGOS[algo][0], host["target_logits"][sel, :g + 1], host["draft_logits"][sel, :g],
                                host["draft_tokens"][sel, :g], host["uniforms"][sel, :g + 1], cfg.temperature, dtype=odt)
            safe = ref["margins"].min(axis=1) >= parity.MARGIN
            n_safe += int(safe.sum())
            assert np.array_equal(tau[sel][safe], ref["accept_len"][safe]), (g, algo, turn)
            same_tau = safe & (tau[sel] == ref["accept_len"])
            assert np.array_equal(y[sel][same_tau], ref["next_token"][same_tau]), (g, algo, turn)
            assert np.all(tau[sel] <= g)
        assert n_safe >= 0.8 * B
        sv.spec_verify_debug_config(FUSED, -1)
        sv.spec_verify_ex(algo, inp["target_logits"], inp["draft_logits"], inp["draft_tokens"], inp["uniforms"], cfg.temperature, workspace=ws)
        sv.spec_verify_debug_config(RESIDENT, -1)


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("B,gamma,V,dtype,pad_t,pad_d", [(16, 8, 8000, "bf16", 96, 32), (7, 4, 11912, "f32", 1, 9),
                                                          (20, 2, 28000, "bf16", 3, 5)])
def test_padded_rows(algo, B, gamma, V, dtype, pad_t, pad_d):
    """Rows inside buffers whose last dimension is padded (stride > V); the padding is poisoned
    with NaN."""
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
    cfg = _custom(4, 3, 5000, "f32")
    inp = workloads.generate(cfg, seed=3, device=DEV)
    ws = sv.alloc_workspace(cfg.B, cfg.gamma + 1, cfg.V, DEV)
    tau, y = sv.spec_verify_block(inp["target_logits"], inp["draft_logits"], inp["draft_tokens"], inp["uniforms"], 1.0,
                                  workspace=ws)
    torch.cuda.synchronize()
    assert bool((tau == -1).all()) and bool((y == -1).all())


def test_waits_that_run_out_give_minus_one_and_the_workspace_says_so():
    """A spin limit of zero polls makes every wait that finds its word missing give up at once; the kernel still ends,
    every sequence either has its correct result or -1, and the workspace reports the error where any gave up."""
    cfg = _custom(40, 6, 16000, "bf16", sigma_t=2.5, sigma_d=1.0, T=0.8)
    inp = workloads.generate(cfg, seed=11, device=DEV)
    ws = sv.alloc_workspace(cfg.B, cfg.gamma, cfg.V, DEV)
    sv.spec_verify_debug_config(RESIDENT, 0)
    try:
        tau, y = sv.spec_verify_block(inp["target_logits"], inp["draft_logits"], inp["draft_tokens"], inp["uniforms"],
                                      cfg.temperature, workspace=ws)
        torch.cuda.synchronize()
        status = binding.spec_verify_workspace_check(ws, cfg.B, cfg.gamma, cfg.V)
    finally:
        sv.spec_verify_debug_config(RESIDENT, -1)
    assert status in (0, 5)                      # 5 = SV_ERR_INTERNAL when some wave really had to wait
    tau, y = tau.cpu().numpy(), y.cpu().numpy()
    ref = parity.run_oracle("block", inp, cfg.temperature)
    gave_up = tau == -1
    assert np.array_equal(gave_up, y == -1)
    if status == 0:
        assert not gave_up.any()
    safe = (ref["margins"].min(axis=1) >= parity.MARGIN) & ~gave_up
    assert np.array_equal(tau[safe], ref["accept_len"][safe]) and np.array_equal(y[safe], ref["next_token"][safe])
    sv.spec_verify_workspace_init(ws, cfg.B, cfg.gamma, cfg.V)
    parity.compare(parity.run_gpu("block", inp, cfg.temperature, workspace=ws), ref)
    assert binding.spec_verify_workspace_check(ws, cfg.B, cfg.gamma, cfg.V) == 0
