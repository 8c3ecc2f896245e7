"""ctypes loader for the CPU oracle (``verify_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports this module, and this module never imports the product package.

The oracle is Alg. 1 (token verification), Alg. 2 (block verification) and
Alg. 4 (greedy block verification) of the paper, in double precision, one
sequence at a time; see the header of ``verify_oracle.c`` for the conventions.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "verify_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_verify.so")

BLOCK, TOKEN, GREEDY = 0, 1, 2
F32, BF16, F64 = 0, 1, 2   # F64: the probability form only, for exact tiny tables in the tests
DBG_STRIDE = 6  # w, S, h, logZ_target, logZ_draft, log r

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_num_threads.argtypes = [ctypes.c_int]
        _lib = lib
    return _lib


def num_threads(requested: int = 0) -> int:
    return int(_load().oracle_num_threads(int(requested)))


def _as_logits(x, dtype_code):
    """A C-contiguous numpy view of the logits: float32, or uint16 holding bf16 bits."""
    if dtype_code == F32:
        arr = np.ascontiguousarray(x, dtype=np.float32)
    elif dtype_code == F64:
        arr = np.ascontiguousarray(x, dtype=np.float64)
    else:
        arr = np.ascontiguousarray(x)
        if arr.dtype != np.uint16:
            raise TypeError("bf16 logits must be passed as their uint16 bit patterns")
    return arr


def _verify(fn_name, with_temperature, algo, target, draft, draft_tokens, uniforms, temperature, dtype, nthreads):
    lib = _load()
    tl = _as_logits(target, dtype)
    dl = _as_logits(draft, dtype)
    tok = np.ascontiguousarray(draft_tokens, dtype=np.int32)
    uni = np.ascontiguousarray(uniforms, dtype=np.float32)
    B, g1, V = tl.shape
    gamma = g1 - 1
    if dl.shape != (B, gamma, V) or tok.shape != (B, gamma) or uni.shape != (B, gamma + 1):
        raise ValueError("shape mismatch between the oracle's inputs")
    tau = np.empty(B, dtype=np.int32)
    y = np.empty(B, dtype=np.int32)
    dbg = np.empty((B, gamma + 1, DBG_STRIDE), dtype=np.float64)
    margins = np.empty((B, 2), dtype=np.float64)
    nfb = ctypes.c_int32(0)
    fn = getattr(lib, fn_name)
    fn.restype = ctypes.c_int
    fn.argtypes = ([ctypes.c_int] + [ctypes.c_void_p] * 4 + [ctypes.c_int] * 4
                   + ([ctypes.c_double] if with_temperature else []) + [ctypes.c_void_p] * 5 + [ctypes.c_int])
    rc = fn(int(algo), tl.ctypes.data, dl.ctypes.data, tok.ctypes.data, uni.ctypes.data,
            B, gamma, V, int(dtype), *((float(temperature),) if with_temperature else ()),
            tau.ctypes.data, y.ctypes.data, dbg.ctypes.data, margins.ctypes.data,
            ctypes.addressof(nfb), int(nthreads))
    if rc != 0:
        raise RuntimeError(f"{fn_name} failed with code {rc}")
    return {"accept_len": tau, "next_token": y, "dbg": dbg, "margins": margins,
            "n_fallback": int(nfb.value)}


def verify(algo: int, target_logits, draft_logits, draft_tokens, uniforms,
           temperature: float, dtype: int = F32, nthreads: int = 0):
    """Run the oracle on a batch.

    target_logits [B, gamma+1, V], draft_logits [B, gamma, V] (float32 arrays, or uint16
    arrays of bf16 bit patterns when ``dtype == BF16``), draft_tokens [B, gamma] int32,
    uniforms [B, gamma+1] float32.  Returns a dict with ``accept_len`` [B], ``next_token``
    [B], ``dbg`` [B, gamma+1, 6] (w, S, h, logZ_target, logZ_draft, log r), ``margins``
    [B, 2] and ``n_fallback``.
    """
    if dtype == F64:
        raise ValueError("logits are float32 or bf16")
    return _verify("oracle_spec_verify", True, algo, target_logits, draft_logits, draft_tokens, uniforms,
                   temperature, dtype, nthreads)


def verify_probs(algo: int, target_probs, draft_probs, draft_tokens, uniforms, dtype: int = F32, nthreads: int = 0):
    """The same with the distributions themselves as inputs (the arrays of App. A): target_probs
    [B, gamma+1, V] = p_i(x), draft_probs [B, gamma, V] = q_i(x), used as given (no temperature, no
    renormalisation).  ``dtype`` may also be F64 (float64 arrays)."""
    return _verify("oracle_spec_verify_probs", False, algo, target_probs, draft_probs, draft_tokens, uniforms,
                   None, dtype, nthreads)


def sample_rows(logits, uniforms, temperature: float, dtype: int = F32):
    """One token per row of ``logits`` [R, V] from softmax(logits / T) by the inverse-CDF walk at
    ``uniforms`` [R] (the drafting step of the outer loop, Alg. 3).  Returns (tokens, margins)."""
    lib = _load()
    lg = _as_logits(logits, dtype)
    uni = np.ascontiguousarray(uniforms, dtype=np.float32)
    R, V = lg.shape
    if uni.shape != (R,):
        raise ValueError("one uniform per row")
    tok = np.empty(R, dtype=np.int32)
    margins = np.empty(R, dtype=np.float64)
    lib.oracle_sample_rows.restype = ctypes.c_int
    lib.oracle_sample_rows.argtypes = [ctypes.c_void_p, ctypes.c_longlong, ctypes.c_int, ctypes.c_int, ctypes.c_double,
                                       ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    rc = lib.oracle_sample_rows(lg.ctypes.data, R, V, int(dtype), float(temperature), uni.ctypes.data,
                                tok.ctypes.data, margins.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_sample_rows failed with code {rc}")
    return tok, margins
