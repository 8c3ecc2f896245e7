"""ctypes binding of libspecverify.so: argument marshalling only.

Every step of the verification path runs in the HIP kernels behind the C ABI declared
in ``include/specverify.h``.  PyTorch is used for device memory and streams, nothing
else.  There is no CPU fallback: if the library has not been built, loading fails.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# the product library; SPECVERIFY_LIBRARY names another build of it in this folder (the tuning build
# libspecverify_profile.so, which adds spec_verify_debug_profile)
LIB_PATH = os.path.join(_HERE, os.environ.get("SPECVERIFY_LIBRARY", "libspecverify.so"))

SV_OK = 0
SV_ERR_INVALID_ARG = 1
SV_ERR_UNSUPPORTED = 2
SV_ERR_WORKSPACE_TOO_SMALL = 3
SV_ERR_HIP = 4
SV_ERR_INTERNAL = 5
SV_ERR_STATIC_SCRATCH_TOO_SMALL = 6
SV_STATIC_SCRATCH_BYTES = 32 << 20
SV_DTYPE_F32 = 0
SV_DTYPE_BF16 = 1

EXPORTED = (
    "spec_verify_workspace_bytes",
    "spec_verify_workspace_init",
    "spec_verify_workspace_check",
    "spec_verify_debug_config",
    "spec_verify_debug_last_kernel",
    "spec_verify_debug_copy",
    "spec_verify_debug_stream_probe",
    "spec_sample_tokens",
    "spec_verify_block",
    "spec_verify_token",
    "spec_verify_greedy",
    "spec_verify_ex",
    "spec_verify_ex_noalloc",
    "spec_verify_probs",
    "spec_verify_status_string",
)

_VERIFY_ARGTYPES = [
    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
    ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, ctypes.c_int, ctypes.c_float,
    ctypes.c_void_p, ctypes.c_size_t,
    ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
]

_lib = None


class SpecVerifyError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"specverify: {text} (status {code})")
        self.code = code


def load() -> ctypes.CDLL:
    """Load the built library; raises if it is missing (build it with build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is not built; run `python -m paper_2403_10444_amd.build` "
                "(there is no fallback implementation)")
        lib = ctypes.CDLL(LIB_PATH)
        lib.spec_verify_workspace_bytes.restype = ctypes.c_size_t
        lib.spec_verify_workspace_bytes.argtypes = [ctypes.c_int32] * 3
        for name in ("spec_verify_block", "spec_verify_token", "spec_verify_greedy"):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = _VERIFY_ARGTYPES
        lib.spec_verify_ex.restype = ctypes.c_int
        lib.spec_verify_ex.argtypes = ([ctypes.c_int] + _VERIFY_ARGTYPES[:3]
                                       + [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64] + _VERIFY_ARGTYPES[3:])
        lib.spec_verify_ex_noalloc.restype = ctypes.c_int
        lib.spec_verify_ex_noalloc.argtypes = [a for j, a in enumerate(lib.spec_verify_ex.argtypes) if j not in (13, 14)]   # no workspace
        lib.spec_verify_probs.restype = ctypes.c_int
        lib.spec_verify_probs.argtypes = [a for j, a in enumerate(lib.spec_verify_ex.argtypes) if j != 12]   # no temperature
        lib.spec_verify_workspace_init.restype = ctypes.c_int
        lib.spec_verify_workspace_init.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32,
                                                   ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        lib.spec_verify_workspace_check.restype = ctypes.c_int
        lib.spec_verify_workspace_check.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                                    ctypes.c_int32, ctypes.c_void_p]
        lib.spec_verify_debug_last_kernel.restype = ctypes.c_int32
        lib.spec_verify_debug_last_kernel.argtypes = []
        lib.spec_verify_debug_config.restype = None
        lib.spec_verify_debug_config.argtypes = [ctypes.c_int32, ctypes.c_int32]
        if hasattr(lib, "spec_verify_debug_profile"):          # tuning builds only
            lib.spec_verify_debug_profile.restype = None
            lib.spec_verify_debug_profile.argtypes = [ctypes.c_void_p]
        lib.spec_verify_debug_copy.restype = ctypes.c_int
        lib.spec_verify_debug_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
        lib.spec_verify_debug_stream_probe.restype = ctypes.c_int
        lib.spec_verify_debug_stream_probe.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p,
                                                       ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p]
        lib.spec_sample_tokens.restype = ctypes.c_int
        lib.spec_sample_tokens.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_int, ctypes.c_float,
                                           ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.spec_verify_status_string.restype = ctypes.c_char_p
        lib.spec_verify_status_string.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def status_string(code: int) -> str:
    return load().spec_verify_status_string(int(code)).decode()


def spec_verify_workspace_bytes(B: int, gamma: int, V: int) -> int:
    return int(load().spec_verify_workspace_bytes(int(B), int(gamma), int(V)))


def spec_verify_workspace_init(workspace: torch.Tensor, B: int, gamma: int, V: int, stream=None) -> None:
    if stream is None:
        stream = torch.cuda.current_stream(workspace.device).cuda_stream
    code = load().spec_verify_workspace_init(workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                             int(B), int(gamma), int(V), stream)
    if code != SV_OK:
        raise SpecVerifyError(code, status_string(code))


def spec_verify_workspace_check(workspace: torch.Tensor, B: int, gamma: int, V: int, stream=None) -> int:
    """Blocks on the stream and returns the workspace's status code (SV_OK when healthy)."""
    if stream is None:
        stream = torch.cuda.current_stream(workspace.device).cuda_stream
    return int(load().spec_verify_workspace_check(workspace.data_ptr(), int(B), int(gamma), int(V), stream))


def spec_verify_debug_config(path: int = 0, spin_limit: int = -1) -> None:
    load().spec_verify_debug_config(int(path), int(spin_limit))


SV_KERNEL_STAGED, SV_KERNEL_FUSED, SV_KERNEL_TINY, SV_KERNEL_RESIDENT, SV_KERNEL_PROBS = 1, 2, 5, 7, 8


def spec_verify_debug_last_kernel() -> int:
    """Which kernels the last verification call of this process launched (SV_KERNEL_*; 0 before the first)."""
    return int(load().spec_verify_debug_last_kernel())


def spec_verify_debug_profile(buffer) -> None:
    """Tuning builds only (see build.py): per-workgroup timestamps of the fused kernel go to `buffer` (a zeroed
    int64 device tensor [B * (gamma + 1) * workgroups per row, 16]) until called again with None."""
    lib = load()
    if not hasattr(lib, "spec_verify_debug_profile"):
        raise RuntimeError("this build of the library has no profiling hook; build with build.py --profile and "
                           "set SPECVERIFY_LIBRARY=libspecverify_profile.so")
    lib.spec_verify_debug_profile(buffer.data_ptr() if buffer is not None else None)


def spec_verify_debug_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    """The library's plain copy kernel (what memory-traffic counters are scaled against)."""
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("dst and src must have the same size in bytes")
    if stream is None:
        stream = torch.cuda.current_stream(src.device).cuda_stream
    code = load().spec_verify_debug_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream)
    if code != SV_OK:
        raise SpecVerifyError(code, status_string(code))


def spec_verify_debug_stream_probe(a: torch.Tensor, b: torch.Tensor, out: torch.Tensor, short_waits: int = 0,
                                   long_waits: int = 0, stream=None) -> None:
    """The library's streaming probe (the floor of the verification kernel's launch shape) over two equally large
    device buffers; `out` takes one float per 4096 bytes of `a`.  `short_waits`, `long_waits` (units of 512 clocks):
    the modelled waits of a verifying kernel, see the header; 0, 0 is the floor."""
    nbytes = a.numel() * a.element_size()
    if b.numel() * b.element_size() != nbytes or out.numel() * 4096 < nbytes or out.dtype != torch.float32:
        raise ValueError("a and b must have the same size in bytes and out one float32 per 4096 bytes of a")
    if stream is None:
        stream = torch.cuda.current_stream(a.device).cuda_stream
    code = load().spec_verify_debug_stream_probe(a.data_ptr(), b.data_ptr(), nbytes, out.data_ptr(),
                                                 int(short_waits), int(long_waits), stream)
    if code != SV_OK:
        raise SpecVerifyError(code, status_string(code))


def spec_sample_tokens(logits: torch.Tensor, uniforms: torch.Tensor, temperature: float, tokens=None, stream=None):
    """One token per row of ``logits`` [..., V] from softmax(logits / T) by the inverse CDF at ``uniforms``
    [...] (the drafting step of Alg. 3).  Returns int32 tokens of the shape of ``uniforms``."""
    V = logits.shape[-1]
    rows = logits.numel() // V
    if logits.device.type != "cuda" or not logits.is_contiguous() or not uniforms.is_contiguous():
        raise ValueError("logits and uniforms must be contiguous cuda tensors")
    if uniforms.numel() != rows or uniforms.dtype != torch.float32:
        raise ValueError("one float32 uniform per row")
    if tokens is None:
        tokens = torch.empty(uniforms.shape, dtype=torch.int32, device=logits.device)
    if stream is None:
        stream = torch.cuda.current_stream(logits.device).cuda_stream
    code = load().spec_sample_tokens(logits.data_ptr(), rows, V, _dtype_code(logits), float(temperature),
                                     uniforms.data_ptr(), tokens.data_ptr(), stream)
    if code != SV_OK:
        raise SpecVerifyError(code, status_string(code))
    return tokens


def alloc_workspace(B: int, gamma: int, V: int, device="cuda") -> torch.Tensor:
    """A device byte buffer of the size the library asks for, initialised for this shape."""
    n = spec_verify_workspace_bytes(B, gamma, V)
    if n == 0:
        raise SpecVerifyError(SV_ERR_UNSUPPORTED, "sizes not supported")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    with torch.cuda.device(ws.device):
        spec_verify_workspace_init(ws, B, gamma, V)
    return ws


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SV_DTYPE_F32
    if t.dtype == torch.bfloat16:
        return SV_DTYPE_BF16
    raise TypeError(f"logits must be float32 or bfloat16, got {t.dtype}")


SV_ALGO = {"block": 0, "token": 1, "greedy": 2}


def _row_stride(t: torch.Tensor, rows_per_seq: int) -> int:
    """Row stride in elements of a [B, rows_per_seq, V] tensor whose rows are dense and evenly spaced
    (a contiguous tensor, or the [..., :V] view of one with a padded last dimension)."""
    B, R, V = t.shape
    sb, sr, sv_ = t.stride()
    if sv_ != 1 or sr < V or (B > 1 and sb != sr * rows_per_seq):
        raise ValueError("logits must have unit stride along the vocabulary and evenly spaced rows")
    return sr


def _call(name, target_logits, draft_logits, draft_tokens, uniforms, temperature,
          workspace=None, accept_len=None, next_token=None, debug_out=None, stream=None, draft_lens=None, algo=None):
    lib = load()
    B, g1, V = target_logits.shape
    gamma = g1 - 1
    dev = target_logits.device
    if dev.type != "cuda":
        raise ValueError("specverify runs on the GPU only; tensors must live on a cuda device")
    if tuple(draft_logits.shape) != (B, gamma, V) or tuple(draft_tokens.shape) != (B, gamma) \
            or tuple(uniforms.shape) != (B, gamma + 1):
        raise ValueError("shape mismatch between the inputs")
    if draft_logits.dtype != target_logits.dtype:
        raise TypeError("target and draft logits must share a dtype")
    for t, want in ((draft_tokens, torch.int32), (uniforms, torch.float32)):
        if t.dtype != want:
            raise TypeError(f"expected {want}, got {t.dtype}")
    extended = name in ("spec_verify_ex", "spec_verify_ex_noalloc", "spec_verify_probs")
    own_workspace = name != "spec_verify_ex_noalloc"
    for t in (target_logits, draft_logits, draft_tokens, uniforms):
        if t.device != dev:
            raise ValueError("inputs must be on one device")
    for t in (draft_tokens, uniforms) + (() if extended else (target_logits, draft_logits)):
        if not t.is_contiguous():
            raise ValueError("inputs must be contiguous")
    if workspace is None and own_workspace:
        workspace = alloc_workspace(B, gamma, V, dev)
    if accept_len is None:
        accept_len = torch.empty(B, dtype=torch.int32, device=dev)
    if next_token is None:
        next_token = torch.empty(B, dtype=torch.int32, device=dev)
    if stream is None:
        stream = torch.cuda.current_stream(dev).cuda_stream
    head = ()
    after_tokens = ()
    if extended:
        if draft_lens is not None and (tuple(draft_lens.shape) != (B,) or draft_lens.dtype != torch.int32
                                       or draft_lens.device != dev or not draft_lens.is_contiguous()):
            raise ValueError("draft_lens must be a contiguous int32 tensor [B] on the inputs' device")
        head = (SV_ALGO[algo],)
        after_tokens = (draft_lens.data_ptr() if draft_lens is not None else None,
                        _row_stride(target_logits, gamma + 1), _row_stride(draft_logits, gamma))
    code = getattr(lib, name)(
        *head, target_logits.data_ptr(), draft_logits.data_ptr(), draft_tokens.data_ptr(), *after_tokens,
        uniforms.data_ptr(),
        B, gamma, V, _dtype_code(target_logits), *(() if name == "spec_verify_probs" else (float(temperature),)),
        *((workspace.data_ptr(), workspace.numel() * workspace.element_size()) if own_workspace else ()),
        accept_len.data_ptr(), next_token.data_ptr(),
        debug_out.data_ptr() if debug_out is not None else None, stream)
    if code != SV_OK:
        raise SpecVerifyError(code, status_string(code))
    return accept_len, next_token


def spec_verify_ex(algo, target_logits, draft_logits, draft_tokens, uniforms, temperature, draft_lens=None, **kw):
    """`algo` ("block", "token" or "greedy") with the input variants of `spec_verify_ex` in the header:
    ``draft_lens`` (int32 device tensor [B], values 1 .. gamma, or None) makes sequence b use only its first
    draft_lens[b] draft positions; the logits may be ``[..., :V]`` views of buffers whose last dimension is
    padded (the row strides are taken from the tensors)."""
    return _call("spec_verify_ex", target_logits, draft_logits, draft_tokens, uniforms, temperature,
                 draft_lens=draft_lens, algo=algo, **kw)


def spec_verify_ex_noalloc(algo, target_logits, draft_logits, draft_tokens, uniforms, temperature, accept_len, next_token,
                           draft_lens=None, debug_out=None, stream=None):
    """`spec_verify_ex` on the library's built-in scratch memory instead of a workspace (see the header): the call
    allocates nothing, so the outputs must be preallocated int32 device tensors [B].  Calls on one GPU must not
    overlap."""
    return _call("spec_verify_ex_noalloc", target_logits, draft_logits, draft_tokens, uniforms, temperature,
                 accept_len=accept_len, next_token=next_token, debug_out=debug_out, stream=stream,
                 draft_lens=draft_lens, algo=algo)


def spec_verify_probs(algo, target_probs, draft_probs, draft_tokens, uniforms, draft_lens=None, **kw):
    """`algo` ("block", "token" or "greedy") on distributions handed over as probabilities (the arrays of the
    paper's App. A), used as given: see `spec_verify_probs` in the header.  ``draft_lens`` and padded rows as for
    `spec_verify_ex`."""
    return _call("spec_verify_probs", target_probs, draft_probs, draft_tokens, uniforms, None,
                 draft_lens=draft_lens, algo=algo, **kw)


def spec_verify_block(target_logits, draft_logits, draft_tokens, uniforms, temperature, **kw):
    """Block verification (Alg. 2): returns (accept_len [B], next_token [B]) int32 device tensors.

    Asynchronous on the current (or given) stream.  Optional keyword arguments: ``workspace``
    (uint8 device tensor from `alloc_workspace`), preallocated ``accept_len`` / ``next_token``,
    ``debug_out`` (float32 [B, gamma+1, 3] device tensor receiving w, S, h) and ``stream``
    (a raw hipStream_t handle)."""
    return _call("spec_verify_block", target_logits, draft_logits, draft_tokens, uniforms, temperature, **kw)


def spec_verify_token(target_logits, draft_logits, draft_tokens, uniforms, temperature, **kw):
    """Token verification (Alg. 1); same arguments and returns as `spec_verify_block`."""
    return _call("spec_verify_token", target_logits, draft_logits, draft_tokens, uniforms, temperature, **kw)


def spec_verify_greedy(target_logits, draft_logits, draft_tokens, uniforms, temperature, **kw):
    """Greedy block verification (Alg. 4); same arguments and returns as `spec_verify_block`."""
    return _call("spec_verify_greedy", target_logits, draft_logits, draft_tokens, uniforms, temperature, **kw)
