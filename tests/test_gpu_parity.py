"""Parity of the HIP path (through the C ABI) with the CPU oracle on seeded inputs."""
from __future__ import annotations

import json

import numpy as np
import pytest
import torch

import paper_2403_10444_amd as sv
import oracle
import workloads
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda"


# "default": the library's own choice of kernels by the shape of the call (one workgroup per sequence, the kernel for calls
# of few resident sets, the fused kernel with the unit size it picks); the others force a path through the testing hook
PATHS = {"default": 0, "staged": 1, "fused": 3, "fused-large": 4}


@pytest.fixture(autouse=True, params=list(PATHS))
def path(request):
    """Every test runs on every kernel path: the library's own choice, the single-launch fused kernel with its small
    units, the same with its large units (bf16 rows on the 16-byte path; other calls fall back to the small ones), and
    the staged kernels."""
    sv.spec_verify_debug_config(PATHS[request.param], -1)
    yield request.param
    sv.spec_verify_debug_config(0, -1)


def _say(report):
    print(json.dumps(parity.record(report)), flush=True)


def _custom(B, gamma, V, dtype="f32", sigma_t=3.0, sigma_d=1.0, T=1.0, zipf=False):
    return workloads.Config(f"custom_B{B}_g{gamma}_V{V}_{dtype}", B, gamma, V, dtype, sigma_t, sigma_d, T, zipf, 1)


# ------------------------------------------------------------------ the five configurations
@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_cfg1_ten_thousand_calls_batched(algo, path):
    # the 10,000 calls of configuration 1 as one batch of 10,000 independent sequences
    cfg = workloads.with_overrides(workloads.CONFIGS[1], B=10000)
    inp = workloads.generate(cfg, seed=101, device=DEV)
    rep = parity.compare(parity.run_gpu(algo, inp, cfg.temperature), parity.run_oracle(algo, inp, cfg.temperature),
                         label=f"cfg1/{algo}/{path}")
    _say(rep)


def test_cfg1_single_sequence_calls(path):
    cfg = workloads.CONFIGS[1]
    ws = sv.alloc_workspace(cfg.B, cfg.gamma, cfg.V, DEV)
    for call in range(40):
        inp = workloads.generate(cfg, seed=1000 + call, device=DEV)
        for algo in ("block", "token"):
            parity.record(parity.compare(parity.run_gpu(algo, inp, cfg.temperature, workspace=ws),
                                         parity.run_oracle(algo, inp, cfg.temperature),
                                         label=f"cfg1/call{call}/single-sequence-calls/{algo}/{path}"))


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_cfg2_calls(algo, path):
    cfg = workloads.CONFIGS[2]
    ws = sv.alloc_workspace(cfg.B, cfg.gamma, cfg.V, DEV)
    taus = []
    for call in range(12):
        inp = workloads.generate(cfg, seed=2000 + call, device=DEV)
        gpu = parity.run_gpu(algo, inp, cfg.temperature, workspace=ws)
        rep = parity.record(parity.compare(gpu, parity.run_oracle(algo, inp, cfg.temperature),
                                           label=f"cfg2/call{call}/{algo}/{path}"))
        taus.append(rep["mean_tau"])
    print(json.dumps({"label": f"cfg2/{algo}/{path}", "mean_tau": float(np.mean(taus)), "last": rep}), flush=True)


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_cfg3_full_batch(algo, path):
    cfg = workloads.CONFIGS[3]
    for seed in (3000, 3001):
        inp = workloads.generate(cfg, seed=seed, device=DEV)
        rep = parity.compare(parity.run_gpu(algo, inp, cfg.temperature),
                             parity.run_oracle(algo, inp, cfg.temperature), label=f"cfg3/seed{seed}/{algo}/{path}")
        _say(rep)
    # (the headline shape is the fused kernel's by the library's own choice too)
    assert sv.spec_verify_debug_last_kernel() == (1 if path == "staged" else 2)


# ------------------------------------------------------------------ shapes and edge cases
SHAPES = [
    # B, gamma, V, dtype           what it exercises
    (3, 1, 1, "f32"),            # one-token vocabulary
    (3, 2, 7, "bf16"),           # tiny, unaligned rows
    (5, 3, 8191, "f32"),         # one element short of a chunk, unaligned
    (5, 3, 8192, "bf16"),        # exactly one chunk
    (4, 2, 8200, "bf16"),        # a chunk and a ragged tail, aligned
    (4, 5, 16389, "bf16"),       # unaligned, three chunks
    (2, 4, 50001, "f32"),        # unaligned, odd
    (7, 64, 1000, "f32"),        # the longest draft block the library takes
    (1, 8, 128256, "bf16"),      # one sequence of the headline shape
    (33, 6, 32000, "bf16"),
    (2, 2, 140001, "bf16"),      # rows of more than 64 wave chunks (two row words per lane), unaligned
    (1, 2, 300000, "f32"),       # more than 128 wave chunks (four row words per lane)
    (1, 1, 600008, "bf16"),      # more than 256 wave chunks (eight row words per lane)
]


@pytest.mark.parametrize("B,gamma,V,dtype", SHAPES)
@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_shapes(B, gamma, V, dtype, algo):
    cfg = _custom(B, gamma, V, dtype, sigma_t=2.5, sigma_d=0.8, T=0.9)
    inp = workloads.generate(cfg, seed=B * 1000 + gamma * 10 + V % 7, device=DEV)
    rep = parity.compare(parity.run_gpu(algo, inp, cfg.temperature), parity.run_oracle(algo, inp, cfg.temperature),
                         label=f"{cfg.name}/{algo}")
    print(json.dumps(rep), flush=True)


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
def test_unaligned_base_pointers(algo, path):
    cfg = _custom(4, 3, 4096, "bf16")
    inp = workloads.generate(cfg, seed=77, device=DEV)
    # shift both logit buffers by one element so that the 16-byte path cannot be taken
    def shifted(t):
        buf = torch.empty(t.numel() + 1, dtype=t.dtype, device=t.device)
        buf[1:] = t.reshape(-1)
        return buf[1:].view(t.shape)
    inp2 = dict(inp, target_logits=shifted(inp["target_logits"]), draft_logits=shifted(inp["draft_logits"]))
    assert inp2["target_logits"].data_ptr() % 16 != 0
    a = parity.run_gpu(algo, inp, cfg.temperature)
    b = parity.run_gpu(algo, inp2, cfg.temperature)
    assert np.array_equal(a["accept_len"], b["accept_len"]) and np.array_equal(a["next_token"], b["next_token"])
    if path == "fused-large":
        # the shifted buffers take the small units (the large ones need the 16-byte path): another summation order
        assert np.allclose(a["dbg"], b["dbg"], rtol=1e-5, atol=1e-7)
    else:
        assert np.array_equal(a["dbg"], b["dbg"])
    parity.compare(b, parity.run_oracle(algo, inp, cfg.temperature))


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("gamma", [5, 64])          # (64: the longest draft - every bit of the word of test results is used)
def test_identical_models_accept_everything(algo, gamma, path):
    cfg = _custom(16 if gamma == 5 else 3, gamma, 20000 if gamma == 5 else 9000, "bf16", sigma_t=4.0)
    inp = workloads.generate(cfg, seed=5, device=DEV)
    inp["draft_logits"] = inp["target_logits"][:, :cfg.gamma].contiguous()
    gpu = parity.run_gpu(algo, inp, 0.7)
    assert np.all(gpu["accept_len"] == cfg.gamma)
    parity.compare(gpu, parity.run_oracle(algo, inp, 0.7), greedy=algo == "greedy")


@pytest.mark.parametrize("algo", ["block", "token"])
def test_disjoint_supports_reject_everything(algo):
    # the draft puts its mass where the target has none: ratios underflow, tau = 0, and Y comes from
    # the residual, which is the target itself to rounding
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


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_residual_without_mass_draws_from_the_target_row(dtype, algo, path):
    """The draw of Y where float32 leaves a residual no mass at all (Alg. 2 draws from the residual; the kernels' and the
    oracle's fallback is the target row itself).  Consistent arithmetic cannot reach it - a position whose residual is
    empty cannot become tau - so the case is built from underflow: the two models agree on every token that float32 can
    see and differ only on tokens 200 and 300 logits below the rest, one of which is drafted right behind position i.
    Then tests 1 .. i pass with ratio 1, test i + 1 fails with a ratio of 2^-144, tau = i (as in the oracle), and the
    kernels' S_i is exactly 0: Y must be the inverse-CDF draw from p_i.  (The oracle, in double, still sees the residual
    on the far tokens and draws there: Y is compared with the draw from p_i instead, tau with the oracle.)  One sequence
    per position i = 0 .. gamma - 1: the last one is the finishing wave's own row, the others come in through the
    positions' words."""
    gamma, V, T = 3, 20000, 1.0
    cfg = _custom(gamma, gamma, V, dtype, sigma_t=3.0)
    inp = workloads.generate(cfg, seed=77, device=DEV)
    tgt = inp["target_logits"].float()
    live = V - 64                                            # the last 64 tokens are the far ones
    tgt[..., live:live + 32] = -300.0
    tgt[..., live + 32:] = -200.0
    drf = tgt[:, :gamma].clone()
    drf[..., live:live + 32] = -200.0
    drf[..., live + 32:] = -300.0
    dt = inp["target_logits"].dtype
    inp["target_logits"], inp["draft_logits"] = tgt.to(dt).contiguous(), drf.to(dt).contiguous()
    # drafted tokens: the row's most likely token (ratio exactly 1) up to position b, a far token behind it
    top = inp["draft_logits"].float().argmax(-1).to(torch.int32)          # [B, gamma]
    tokens = top.clone()
    for b in range(gamma):
        tokens[b, b] = live + 3                                           # X_{b+1}: target -300, draft -200
    inp["draft_tokens"] = tokens.contiguous()
    # u in the middle of the cell of row i's most likely token: no rounding of a float32 sum moves the draw out of it
    rows = inp["target_logits"].double()[torch.arange(gamma), torch.arange(gamma)]
    cdf = torch.cumsum(torch.softmax(rows / T, -1), -1).cpu().numpy()
    want = rows.argmax(-1).cpu().numpy()
    mid = np.array([(cdf[b, want[b]] + (cdf[b, want[b] - 1] if want[b] > 0 else 0.0)) / 2 / cdf[b, -1] for b in range(gamma)])
    assert all(cdf[b, want[b]] - (cdf[b, want[b] - 1] if want[b] > 0 else 0.0) > 1e-3 for b in range(gamma))
    inp["uniforms"][:, :gamma] = 0.5
    inp["uniforms"][:, gamma] = torch.as_tensor(mid.astype(np.float32), device=DEV)
    ref = parity.run_oracle(algo, inp, T)
    gpu = parity.run_gpu(algo, inp, T)
    assert np.array_equal(gpu["accept_len"], np.arange(gamma)), gpu["accept_len"]
    assert np.array_equal(gpu["accept_len"], ref["accept_len"])
    assert np.all(gpu["dbg"][np.arange(gamma), np.arange(gamma), 1] == 0.0)      # S_i as the kernels see it
    assert np.array_equal(gpu["next_token"], want), (gpu["next_token"], want)
    assert np.all(gpu["next_token"] < live)


def test_uniform_extremes():
    cfg = _custom(6, 4, 9000, "bf16")
    inp = workloads.generate(cfg, seed=8, device=DEV)
    for value in (0.0, 1.0 - 2.0 ** -24):
        inp2 = dict(inp, uniforms=torch.full_like(inp["uniforms"], value))
        for algo in ("block", "token", "greedy"):
            parity.compare(parity.run_gpu(algo, inp2, 1.0), parity.run_oracle(algo, inp2, 1.0))


def test_results_are_bit_reproducible():
    cfg = workloads.with_overrides(workloads.CONFIGS[3], B=8)
    inp = workloads.generate(cfg, seed=9, device=DEV)
    a = parity.run_gpu("block", inp, cfg.temperature)
    for _ in range(3):
        b = parity.run_gpu("block", inp, cfg.temperature)
        assert np.array_equal(a["accept_len"], b["accept_len"])
        assert np.array_equal(a["next_token"], b["next_token"])
        assert np.array_equal(a["dbg"], b["dbg"])


def test_gamma_one_block_equals_token():
    cfg = _custom(64, 1, 5000, "bf16", sigma_d=1.5)
    inp = workloads.generate(cfg, seed=10, device=DEV)
    a = parity.run_gpu("block", inp, 1.0)
    b = parity.run_gpu("token", inp, 1.0)
    assert np.array_equal(a["accept_len"], b["accept_len"]) and np.array_equal(a["next_token"], b["next_token"])


def test_runs_on_a_side_stream():
    cfg = _custom(4, 3, 30000, "bf16")
    inp = workloads.generate(cfg, seed=11, device=DEV)
    ref = parity.run_gpu("block", inp, 1.0)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        tau, y = sv.spec_verify_block(inp["target_logits"], inp["draft_logits"], inp["draft_tokens"],
                                      inp["uniforms"], 1.0)
    s.synchronize()
    assert np.array_equal(tau.cpu().numpy(), ref["accept_len"]) and np.array_equal(y.cpu().numpy(), ref["next_token"])


def test_two_calls_overlap_on_two_streams_with_their_own_workspaces():
    """Calls are re-entrant given disjoint workspaces: two calls launched on two streams without a
    synchronisation between them (their kernels share the device) give what each gives alone."""
    cfg = _custom(32, 4, 60000, "bf16", sigma_t=2.5, sigma_d=1.0, T=0.9)
    inps = [workloads.generate(cfg, seed=60 + i, device=DEV) for i in range(2)]
    refs = [parity.run_gpu("block", inp, cfg.temperature) for inp in inps]
    wss = [sv.alloc_workspace(cfg.B, cfg.gamma, cfg.V, DEV) for _ in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(3):
        outs = []
        for inp, ws, st in zip(inps, wss, streams):
            with torch.cuda.stream(st):
                outs.append(sv.spec_verify_block(inp["target_logits"], inp["draft_logits"], inp["draft_tokens"],
                                                 inp["uniforms"], cfg.temperature, workspace=ws))
        torch.cuda.synchronize()
        for (tau, y), ref, ws in zip(outs, refs, wss):
            assert np.array_equal(tau.cpu().numpy(), ref["accept_len"]) and np.array_equal(y.cpu().numpy(), ref["next_token"])
            assert sv.spec_verify_workspace_check(ws, cfg.B, cfg.gamma, cfg.V) == 0


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("kt,kd", [(50, 50), (20, 200), (500, 5), (1, 40)])
def test_masked_logits_top_k(algo, kt, kd):
    """Rows warped by top-k: everything but the k largest logits is -inf, independently for target and draft,
    so drafted tokens fall outside the target's support (ratio 0) and units, even whole workgroups, of a
    row hold no finite logit."""
    cfg = _custom(16, 6, 20000, "bf16", sigma_t=3.0, sigma_d=1.0, T=0.9)
    inp = workloads.generate(cfg, seed=300 + kt + kd, device=DEV, top_k_target=kt, top_k_draft=kd)
    assert torch.isinf(inp["target_logits"]).any() and torch.isinf(inp["draft_logits"]).any()
    rep = parity.compare(parity.run_gpu(algo, inp, cfg.temperature), parity.run_oracle(algo, inp, cfg.temperature),
                         label=f"top-k {kt}/{kd}/{algo}", greedy=(algo == "greedy"))
    print(json.dumps(rep), flush=True)


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("B,gamma,V,dtype", [(24, 8, 20000, "bf16"), (9, 5, 8191, "f32"), (130, 16, 3000, "bf16")])
def test_ragged_draft_lengths(algo, B, gamma, V, dtype):
    """Sequences with drafts of different lengths in one call: sequence b must come out exactly as a call with
    gamma = draft_lens[b] on its leading rows does (here: the oracle on those slices).  The rows beyond a
    sequence's length are poisoned with NaN to show that they are never read."""
    cfg = _custom(B, gamma, V, dtype, sigma_t=2.5, sigma_d=1.0, T=0.8)
    inp = workloads.generate(cfg, seed=500 + B + gamma, device=DEV)
    rng = np.random.default_rng(B * gamma)
    lens = rng.integers(1, gamma + 1, size=B).astype(np.int32)
    lens[0], lens[-1] = gamma, 1
    tl, dl = inp["target_logits"].clone(), inp["draft_logits"].clone()
    for b in range(B):
        tl[b, lens[b] + 1:] = float("nan")
        dl[b, lens[b]:] = float("nan")
    dbg = torch.full((B, gamma + 1, 3), float("nan"), dtype=torch.float32, device=DEV)
    tau, y = sv.spec_verify_ex(algo, tl, dl, inp["draft_tokens"], inp["uniforms"], cfg.temperature,
                               draft_lens=torch.as_tensor(lens, device=DEV), debug_out=dbg)
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


@pytest.mark.parametrize("algo", ["block", "token"])
def test_one_workspace_through_calls_with_changing_draft_lengths(algo):
    """The same workspace in a row of calls whose draft lengths change from call to call (long, short, long, one,
    long) and whose inputs change too: words that an earlier call left behind at positions a later call uses again
    (or no longer uses) must never be taken for the later call's.  Every call is compared with the oracle."""
    B, gamma, V = 20, 8, 12000
    cfg = _custom(B, gamma, V, "bf16", sigma_t=2.5, sigma_d=1.0, T=0.8)
    ws = sv.alloc_workspace(B, gamma, V, DEV)
    rng = np.random.default_rng(77)
    patterns = [np.full(B, gamma), np.full(B, 3), rng.integers(1, gamma + 1, size=B), np.full(B, 1),
                np.full(B, gamma), rng.integers(1, gamma + 1, size=B), np.full(B, gamma)]
    for call, lens in enumerate(patterns):
        lens = lens.astype(np.int32)
        inp = workloads.generate(cfg, seed=900 + call, device=DEV)
        tau, y = sv.spec_verify_ex(algo, inp["target_logits"], inp["draft_logits"], inp["draft_tokens"], inp["uniforms"],
                                   cfg.temperature, draft_lens=torch.as_tensor(lens, device=DEV), workspace=ws)
        torch.cuda.synchronize()
        assert sv.spec_verify_workspace_check(ws, B, gamma, V) == 0
        tau, y = tau.cpu().numpy(), y.cpu().numpy()
        host = workloads.to_numpy(inp)
        for g in np.unique(lens):
            sel = np.nonzero(lens == g)[0]
            ref = oracle.verify(parity.ALGOS[algo][0], host["target_logits"][sel, :g + 1], host["draft_logits"][sel, :g],
                                host["draft_tokens"][sel, :g], host["uniforms"][sel, :g + 1], cfg.temperature, dtype=oracle.BF16)
            safe = ref["margins"].min(axis=1) >= parity.MARGIN
            assert np.array_equal(tau[sel][safe], ref["accept_len"][safe]), (call, g)
            same_tau = safe & (tau[sel] == ref["accept_len"])
            assert np.array_equal(y[sel][same_tau], ref["next_token"][same_tau]), (call, g)


def test_ragged_with_full_lengths_equals_the_plain_call():
    cfg = _custom(12, 6, 10000, "bf16")
    inp = workloads.generate(cfg, seed=41, device=DEV)
    a = parity.run_gpu("block", inp, 1.0)
    lens = torch.full((cfg.B,), cfg.gamma, dtype=torch.int32, device=DEV)
    tau, y = sv.spec_verify_ex("block", inp["target_logits"], inp["draft_logits"], inp["draft_tokens"],
                               inp["uniforms"], 1.0, draft_lens=lens)
    torch.cuda.synchronize()
    assert np.array_equal(tau.cpu().numpy(), a["accept_len"]) and np.array_equal(y.cpu().numpy(), a["next_token"])


@pytest.mark.parametrize("algo", ["block", "token", "greedy"])
@pytest.mark.parametrize("B,gamma,V,dtype,pad_t,pad_d", [
    (16, 8, 20000, "bf16", 96, 32),     # strides keep 16-byte alignment: vector loads
    (7, 4, 8191, "f32", 1, 9),          # odd V and odd strides: scalar loads
    (5, 3, 33000, "bf16", 24, 0),       # target padded, draft dense; bf16 stride a multiple of 8 elements
    (70, 2, 3000, "bf16", 3, 5),        # several sequence groups, misaligned strides
])
def test_padded_rows(algo, B, gamma, V, dtype, pad_t, pad_d):
    """Rows of V logits inside buffers whose last dimension is padded (stride > V).  The padding is poisoned
    with NaN to show that it is never read; the result must be the one for dense rows (the oracle's)."""
    cfg = _custom(B, gamma, V, dtype, sigma_t=2.5, sigma_d=1.0, T=0.8)
    inp = workloads.generate(cfg, seed=700 + B + gamma, device=DEV)
    tbuf = torch.full((B, gamma + 1, V + pad_t), float("nan"), dtype=inp["target_logits"].dtype, device=DEV)
    dbuf = torch.full((B, gamma, V + pad_d), float("nan"), dtype=inp["draft_logits"].dtype, device=DEV)
    tbuf[..., :V] = inp["target_logits"]
    dbuf[..., :V] = inp["draft_logits"]
    tau, y = sv.spec_verify_ex(algo, tbuf[..., :V], dbuf[..., :V], inp["draft_tokens"], inp["uniforms"],
                               cfg.temperature)
    torch.cuda.synchronize()
    gpu = {"accept_len": tau.cpu().numpy(), "next_token": y.cpu().numpy()}
    ref = parity.run_oracle(algo, inp, cfg.temperature)
    safe = ref["margins"].min(axis=1) >= parity.MARGIN
    assert safe.sum() >= 0.8 * B
    assert np.array_equal(gpu["accept_len"][safe], ref["accept_len"][safe])
    assert np.array_equal(gpu["next_token"][safe], ref["next_token"][safe])


def test_padded_rows_with_draft_lengths():
    """Both input variants in one call."""
    B, gamma, V = 12, 6, 12000
    cfg = _custom(B, gamma, V, "bf16", sigma_t=2.5, sigma_d=1.0, T=1.0)
    inp = workloads.generate(cfg, seed=77, device=DEV)
    lens = torch.tensor([1 + (b * 5) % gamma for b in range(B)], dtype=torch.int32, device=DEV)
    tbuf = torch.full((B, gamma + 1, V + 40), float("nan"), dtype=torch.bfloat16, device=DEV)
    dbuf = torch.full((B, gamma, V + 8), float("nan"), dtype=torch.bfloat16, device=DEV)
    tbuf[..., :V] = inp["target_logits"]
    dbuf[..., :V] = inp["draft_logits"]
    a = sv.spec_verify_ex("block", inp["target_logits"], inp["draft_logits"], inp["draft_tokens"], inp["uniforms"],
                          1.0, draft_lens=lens)
    b = sv.spec_verify_ex("block", tbuf[..., :V], dbuf[..., :V], inp["draft_tokens"], inp["uniforms"], 1.0,
                          draft_lens=lens)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


def test_captured_in_a_graph_and_replayed():
    """A call is kernel launches only (no allocation, no memset), so it can be captured; every replay, with
    eager calls and synchronisations in between, must give what the eager call gives on the same inputs."""
    cfg = _custom(6, 5, 40000, "bf16")
    sets = [workloads.generate(cfg, seed=200 + i, device=DEV) for i in range(3)]
    static = {k: v.clone() for k, v in sets[0].items() if torch.is_tensor(v)}
    ws = sv.alloc_workspace(cfg.B, cfg.gamma, cfg.V, DEV)
    tau = torch.empty(cfg.B, dtype=torch.int32, device=DEV)
    y = torch.empty(cfg.B, dtype=torch.int32, device=DEV)

    def call():
        sv.spec_verify_block(static["target_logits"], static["draft_logits"], static["draft_tokens"],
                             static["uniforms"], 0.9, workspace=ws, accept_len=tau, next_token=y)

    call()                                   # warm-up outside the capture (one-time occupancy query)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for rep in range(5):
        inp = sets[rep % len(sets)]
        for k in static:
            static[k].copy_(inp[k])
        graph.replay()
        torch.cuda.synchronize()
        got_tau, got_y = tau.cpu().numpy().copy(), y.cpu().numpy().copy()
        ref = parity.run_gpu("block", inp, 0.9)          # eager call (own workspace) between the replays
        assert np.array_equal(got_tau, ref["accept_len"]) and np.array_equal(got_y, ref["next_token"]), rep
    assert sv.spec_verify_workspace_check(ws, cfg.B, cfg.gamma, cfg.V) == 0


def test_workspace_must_be_initialised_for_the_shape(path):
    if path == "staged":
        pytest.skip("only the fused kernel synchronises through the workspace")
    cfg = _custom(4, 3, 9000, "bf16")
    inp = workloads.generate(cfg, seed=12, device=DEV)
    n = sv.spec_verify_workspace_bytes(cfg.B, cfg.gamma, cfg.V)
    ws = torch.zeros(n, dtype=torch.uint8, device=DEV)          # allocated, never initialised
    tau, y = sv.spec_verify_block(inp["target_logits"], inp["draft_logits"], inp["draft_tokens"],
                                  inp["uniforms"], 1.0, workspace=ws)
    torch.cuda.synchronize()
    assert torch.all(tau == -1) and torch.all(y == -1)
    assert sv.spec_verify_workspace_check(ws, cfg.B, cfg.gamma, cfg.V) == 1     # SV_ERR_INVALID_ARG
    sv.spec_verify_workspace_init(ws, cfg.B, cfg.gamma, cfg.V)
    for _ in range(3):                                          # the control words clear themselves
        gpu = parity.run_gpu("block", inp, 1.0, workspace=ws)
        parity.compare(gpu, parity.run_oracle("block", inp, 1.0))
    assert sv.spec_verify_workspace_check(ws, cfg.B, cfg.gamma, cfg.V) == 0
    # initialised for another shape: refused the same way
    other = _custom(2, 3, 9000, "bf16")
    inp2 = workloads.generate(other, seed=13, device=DEV)
    tau, y = sv.spec_verify_block(inp2["target_logits"], inp2["draft_logits"], inp2["draft_tokens"],
                                  inp2["uniforms"], 1.0, workspace=ws)
    torch.cuda.synchronize()
    assert torch.all(tau == -1)


def test_a_wait_that_runs_out_is_reported_not_hung(path):
    if path == "staged":
        pytest.skip("only the fused kernel waits")
    cfg = _custom(16, 8, 40000, "bf16")
    inp = workloads.generate(cfg, seed=14, device=DEV)
    ws = sv.alloc_workspace(cfg.B, cfg.gamma, cfg.V, DEV)
    sv.spec_verify_debug_config(PATHS[path], 0)   # every wait gives up after its first poll
    try:
        tau, y = sv.spec_verify_block(inp["target_logits"], inp["draft_logits"], inp["draft_tokens"],
                                      inp["uniforms"], cfg.temperature, workspace=ws)
        torch.cuda.synchronize()                 # the kernel ends normally whatever it computed
        status = sv.spec_verify_workspace_check(ws, cfg.B, cfg.gamma, cfg.V)
        assert status in (0, 5)                  # 5 = SV_ERR_INTERNAL when some unit really had to wait
        # a sequence any of whose waits ran out reports -1 for both outputs; every other one is complete and right
        tau, y = tau.cpu().numpy(), y.cpu().numpy()
        failed = tau < 0
        assert np.array_equal(failed, y < 0)
        if status == 0:
            assert not failed.any()
        ref = parity.run_oracle("block", inp, cfg.temperature)
        safe = ~failed & (ref["margins"].min(axis=1) >= parity.MARGIN)
        assert np.array_equal(tau[safe], ref["accept_len"][safe]) and np.array_equal(y[safe], ref["next_token"][safe])
    finally:
        sv.spec_verify_debug_config(PATHS[path], -1)
    sv.spec_verify_workspace_init(ws, cfg.B, cfg.gamma, cfg.V)
    parity.compare(parity.run_gpu("block", inp, cfg.temperature, workspace=ws),
                   parity.run_oracle("block", inp, cfg.temperature))
    assert sv.spec_verify_workspace_check(ws, cfg.B, cfg.gamma, cfg.V) == 0


def test_stream_probe_runs_with_and_without_modelled_waits():
    """The measurement hook behind bench.py's floor: it reads its two buffers whole (every wave's float is the sweep's
    result for constant logits) whatever waits are modelled."""
    nbytes = 5 * 16384
    a = torch.full((nbytes,), 0x3c, dtype=torch.uint8, device="cuda")
    b = torch.full((nbytes,), 0x3c, dtype=torch.uint8, device="cuda")
    outs = []
    for waits in ((0, 0), (2, 5)):
        out = torch.full((nbytes // 4096,), float("nan"), dtype=torch.float32, device="cuda")
        sv.spec_verify_debug_stream_probe(a, b, out, waits[0], waits[1])
        torch.cuda.synchronize()
        assert bool(torch.isfinite(out).all())
        outs.append(out.cpu())
    assert bool((outs[0] == outs[1]).all()) and bool((outs[0] == outs[0][0]).all())
