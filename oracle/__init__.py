"""TEST INFRASTRUCTURE -- the CPU oracle for decode attention.

Nothing in the product package imports this.  Only ``tests/``, the smoke
check and the benchmark's ``cpu_baseline`` leg may use it.

Contents
--------
``exact_attention.c``  fp64 two-pass softmax attention (Eq. 1, Section 2.1), the
                       definition the method must reproduce exactly (Section 4.1).
``rescale.py``         partial statistics and the softmax re-scaling operator
                       f(x, y) of Section 4.1, in fp64 numpy (test support: lets
                       the definition be checked by split-and-merge).
``stream_k.py``        the stream-K decomposition of Section 4.3 as interval arithmetic
                       (span edges x tile edges), its pieces folded with f in any
                       order (pins the span bookkeeping of the kernel's walk).

Every function here is pinned by ``tests/test_oracle_pins.py`` against closed
forms, hand-computed cases, invariants and brute-force split/merge; none is
"parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "exact_attention.c")
_LIB = os.path.join(_HERE, "liblean_oracle.so")

F16, BF16, F64 = 0, 1, 2
KV_PADDED, KV_PACKED = 0, 1

_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (host only)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.oracle_decode_attention.restype = ctypes.c_int
        lib.oracle_decode_attention.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
        ]
        lib.oracle_attention.restype = ctypes.c_int
        lib.oracle_attention.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64, ctypes.c_double, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
        ]
        lib.oracle_attention_ragged.restype = ctypes.c_int
        lib.oracle_attention_ragged.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int64, ctypes.c_double, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
        ]
        _lib = lib
    return _lib


def _as_host_array(x, dtype_code):
    """Return a C-contiguous numpy view of the raw elements (uint16 or float64)."""
    if hasattr(x, "detach"):  # torch tensor
        import torch

        x = x.detach().cpu().contiguous()
        if dtype_code == F64:
            return x.to(torch.float64).numpy()
        return x.view(torch.int16).numpy().view(np.uint16)
    x = np.ascontiguousarray(x)
    if dtype_code == F64:
        return x.astype(np.float64, copy=False)
    if x.dtype == np.float16:
        return x.view(np.uint16)
    assert x.dtype == np.uint16, "16-bit inputs must be float16 or raw uint16 bit patterns"
    return x


def dtype_code_of(x) -> int:
    name = str(getattr(x, "dtype", ""))
    if "bfloat16" in name:
        return BF16
    if "float16" in name:
        return F16
    if "float64" in name:
        return F64
    raise TypeError(f"oracle: unsupported element type {name}")


def decode_attention(q, k, v, seqlens, *, Hq, Hkv, D, scale, kv_layout=KV_PADDED, n_stride=0,
                     dtype=None, threads=0, return_threads=False):
    """Exact decode attention in fp64.

    q ``[B,Hq,D]``; k, v PADDED ``[B,Hkv,n_stride,D]`` or PACKED ``[Hkv,sum(seqlens),D]``;
    returns ``(out[B,Hq,D], lse[B,Hq])`` as float64 numpy arrays.
    """
    code = dtype_code_of(q) if dtype is None else dtype
    qa, ka, va = (_as_host_array(t, code) for t in (q, k, v))
    sl = np.ascontiguousarray(np.asarray(seqlens, dtype=np.int32))
    B = sl.shape[0]
    assert qa.size == B * Hq * D, "q must be [B,Hq,D]"
    total = int(sl.sum())
    if kv_layout == KV_PADDED:
        assert ka.size == B * Hkv * n_stride * D and va.size == ka.size, "k/v must be [B,Hkv,n_stride,D]"
    else:
        assert ka.size == Hkv * total * D and va.size == ka.size, "k/v must be [Hkv,sum(seqlens),D]"
    out = np.empty((B, Hq, D), dtype=np.float64)
    lse = np.empty((B, Hq), dtype=np.float64)
    rc = _load().oracle_decode_attention(
        qa.ctypes.data, ka.ctypes.data, va.ctypes.data, sl.ctypes.data, B, Hq, Hkv, D, code,
        kv_layout, int(n_stride), float(scale), out.ctypes.data, lse.ctypes.data, int(threads))
    if rc < 0:
        raise ValueError(f"oracle_decode_attention rejected its arguments (code {rc})")
    return (out, lse, rc) if return_threads else (out, lse)


def attention(q, k, v, seqlens, *, N_q, Hq, Hkv, D, scale, causal, kv_layout=KV_PADDED, n_stride=0,
              dtype=None, threads=0, return_threads=False):
    """Exact attention of N_q query rows per sequence in fp64 (Eq. 1, one row at a time).

    q ``[B,N_q,Hq,D]``; k, v as for :func:`decode_attention`.  The query rows are the last
    N_q cached tokens; with ``causal`` row i attends to the first ``N_b - N_q + i + 1`` rows,
    otherwise to all ``N_b``.  Returns ``(out[B,N_q,Hq,D], lse[B,N_q,Hq])``.
    """
    code = dtype_code_of(q) if dtype is None else dtype
    qa, ka, va = (_as_host_array(t, code) for t in (q, k, v))
    sl = np.ascontiguousarray(np.asarray(seqlens, dtype=np.int32))
    B = sl.shape[0]
    assert qa.size == B * N_q * Hq * D, "q must be [B,N_q,Hq,D]"
    total = int(sl.sum())
    if kv_layout == KV_PADDED:
        assert ka.size == B * Hkv * n_stride * D and va.size == ka.size, "k/v must be [B,Hkv,n_stride,D]"
    else:
        assert ka.size == Hkv * total * D and va.size == ka.size, "k/v must be [Hkv,sum(seqlens),D]"
    out = np.empty((B, N_q, Hq, D), dtype=np.float64)
    lse = np.empty((B, N_q, Hq), dtype=np.float64)
    rc = _load().oracle_attention(
        qa.ctypes.data, ka.ctypes.data, va.ctypes.data, sl.ctypes.data, B, N_q, Hq, Hkv, D, code,
        kv_layout, int(n_stride), float(scale), int(bool(causal)), out.ctypes.data, lse.ctypes.data, int(threads))
    if rc < 0:
        raise ValueError(f"oracle_attention rejected its arguments (code {rc})")
    return (out, lse, rc) if return_threads else (out, lse)


def attention_ragged(q, k, v, seqlens, q_lens, *, Hq, Hkv, D, scale, causal, kv_layout=KV_PADDED, n_stride=0,
                     dtype=None, threads=0):
    """Exact attention with ``q_lens[b]`` query rows for sequence b (its last cached tokens).

    q ``[sum(q_lens),Hq,D]`` (sequence after sequence); k, v as for :func:`decode_attention`.
    With ``causal`` row i of sequence b attends to the first ``N_b - q_lens[b] + i + 1`` rows.
    Returns ``(out[sum(q_lens),Hq,D], lse[sum(q_lens),Hq])``.
    """
    code = dtype_code_of(q) if dtype is None else dtype
    qa, ka, va = (_as_host_array(t, code) for t in (q, k, v))
    sl = np.ascontiguousarray(np.asarray(seqlens, dtype=np.int32))
    ql = np.ascontiguousarray(np.asarray(q_lens, dtype=np.int32))
    B = sl.shape[0]
    assert ql.shape[0] == B, "one query length per sequence"
    n_tok = int(ql.sum())
    assert qa.size == n_tok * Hq * D, "q must be [sum(q_lens),Hq,D]"
    total = int(sl.sum())
    if kv_layout == KV_PADDED:
        assert ka.size == B * Hkv * n_stride * D and va.size == ka.size, "k/v must be [B,Hkv,n_stride,D]"
    else:
        assert ka.size == Hkv * total * D and va.size == ka.size, "k/v must be [Hkv,sum(seqlens),D]"
    out = np.empty((n_tok, Hq, D), dtype=np.float64)
    lse = np.empty((n_tok, Hq), dtype=np.float64)
    rc = _load().oracle_attention_ragged(
        qa.ctypes.data, ka.ctypes.data, va.ctypes.data, sl.ctypes.data, ql.ctypes.data, B, Hq, Hkv, D, code,
        kv_layout, int(n_stride), float(scale), int(bool(causal)), out.ctypes.data, lse.ctypes.data, int(threads))
    if rc < 0:
        raise ValueError(f"oracle_attention_ragged rejected its arguments (code {rc})")
    return out, lse


def attention_row(q, k, v, scale):
    """One query row against ``k[N,D]``, ``v[N,D]`` (float64): ``(out[D], lse)``."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    N, D = k.shape
    out, lse = decode_attention(q.reshape(1, 1, D), k.reshape(1, 1, N, D), v.reshape(1, 1, N, D), [N],
                                Hq=1, Hkv=1, D=D, scale=scale, n_stride=N, dtype=F64, threads=1)
    return out[0, 0], float(lse[0, 0])


def error_metrics(got, want):
    """(max-abs error, relative L2 error) of ``got`` against the fp64 ``want``."""
    g = np.asarray(got, dtype=np.float64).ravel()
    w = np.asarray(want, dtype=np.float64).ravel()
    diff = g - w
    max_abs = float(np.max(np.abs(diff))) if diff.size else 0.0
    denom = float(np.sqrt(np.sum(w * w)))
    rel_l2 = float(np.sqrt(np.sum(diff * diff)) / denom) if denom > 0 else float(np.sqrt(np.sum(diff * diff)))
    return max_abs, rel_l2
