"""Thin ctypes binding over the C ABI of ``include/lean_attn.h``.

Argument marshalling only: every step of the decode path runs in the HIP
library.  There is no fallback: if the library cannot be loaded the import of
a function raises.  Tensors are torch tensors used purely as device memory;
the stream is torch's current HIP stream unless one is given.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

from . import buildlib as _build

F16, BF16 = 0, 1
KV_PADDED, KV_PACKED = 0, 1
OUT_F32, OUT_AS_INPUT = 0, 1
MAX_BATCH, MAX_TILE_ROWS, MAX_QUERY_ROWS, MAX_GRID = 256, 32, 256, 4096

OK = 0
ERR_NULL_POINTER, ERR_BAD_SHAPE, ERR_UNSUPPORTED, ERR_WORKSPACE = -1, -2, -3, -4
ERR_SEQLEN, ERR_BATCH_TOO_LARGE, ERR_HIP, ERR_TUNING, ERR_PEER_TIMEOUT, ERR_STATIC_LIMIT = -5, -6, -7, -8, -9, -10
STATIC_MAX_GRID = 512
NUM_TILE_SHAPES = 9


class Plan(ctypes.Structure):
    _fields_ = [
        ("T_n", ctypes.c_int32), ("T_m", ctypes.c_int32), ("num_output_tiles", ctypes.c_int32),
        ("grid", ctypes.c_int32), ("total_iters", ctypes.c_int64), ("iters_per_cta", ctypes.c_int64),
        ("extra", ctypes.c_int32), ("block_threads", ctypes.c_int32), ("max_resident", ctypes.c_int32),
        ("kernel", ctypes.c_int32), ("fixed_split", ctypes.c_int32), ("C_m", ctypes.c_int32),
        ("tile_shape", ctypes.c_int32), ("tail_grid", ctypes.c_int32), ("tail_iters", ctypes.c_int64),
    ]


class Problem(ctypes.Structure):
    """``lean_attn_problem``: shape and options of one ``lean_attn_attend`` call."""
    _fields_ = [
        ("B", ctypes.c_int32), ("N_q", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
        ("D", ctypes.c_int32), ("dtype", ctypes.c_int32), ("out_dtype", ctypes.c_int32),
        ("kv_layout", ctypes.c_int32), ("causal", ctypes.c_int32), ("scale", ctypes.c_float),
        ("kv_seq_stride", ctypes.c_int64), ("q_lens", ctypes.c_void_p),
    ]

    def set_q_lens(self, q_lens: Optional[Sequence[int]]) -> "Problem":
        """Per-sequence query lengths (host array kept alive by this object); ``None`` clears them."""
        if q_lens is None:
            self._q_lens_host, self._q_lens_list, self.q_lens = None, None, None
            return self
        arr = (ctypes.c_int32 * len(q_lens))(*[int(x) for x in q_lens])
        self._q_lens_host, self._q_lens_list = arr, [int(x) for x in q_lens]
        self.q_lens = ctypes.cast(arr, ctypes.c_void_p).value
        return self

    def query_tokens(self) -> int:
        lens = getattr(self, "_q_lens_list", None)
        return int(sum(lens)) if lens is not None else int(self.B) * int(self.N_q)


class Tuning(ctypes.Structure):
    _fields_ = [
        ("grid", ctypes.c_int32), ("ctas_per_cu", ctypes.c_int32), ("num_cus", ctypes.c_int32),
        ("kernel", ctypes.c_int32), ("tail_grid", ctypes.c_int32), ("spin_limit", ctypes.c_int32),
        ("merge_fanin", ctypes.c_int32), ("tile_shape", ctypes.c_int32), ("grid_multiple", ctypes.c_int32), ("fixed_split", ctypes.c_int32),
        ("debug_delay_store", ctypes.c_int32), ("debug_delay_signal", ctypes.c_int32),
        ("debug_delay_stride", ctypes.c_int32), ("tail_permille", ctypes.c_int32),
        ("cta_clock", ctypes.c_void_p),
    ]


class LeanAttnError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"lean_attn status {status}: {lean_attn_strerror(status)}")


_lib = None


def library_path() -> str:
    """The shared library this binding loads: the in-tree build, or the file named by LEAN_ATTN_LIBRARY
    (for comparing two builds of the library on one machine)."""
    return os.environ.get("LEAN_ATTN_LIBRARY") or _build.LIBRARY


def _load():
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        if path != _build.LIBRARY:
            raise FileNotFoundError(path)
        _build.build()
    lib = ctypes.CDLL(path)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
    lib.lean_attn_workspace_size.restype = sz
    lib.lean_attn_workspace_size.argtypes = [i32] * 5
    lib.lean_attn_workspace_init.restype = i32
    lib.lean_attn_workspace_init.argtypes = [vp, sz, vp]
    lib.lean_attn_workspace_status.restype = i32
    lib.lean_attn_workspace_status.argtypes = [vp, vp]
    lib.lean_attn_schedule.restype = i32
    lib.lean_attn_schedule.argtypes = [vp, i32, i32, i32, i32, i32, i32, ctypes.POINTER(Tuning), ctypes.POINTER(Plan)]
    lib.lean_attn_walk.restype = i32
    lib.lean_attn_walk.argtypes = [ctypes.POINTER(Plan), vp, i32, i32, i32, i32, vp, i32]
    lib.lean_attn_decode.restype = i32
    lib.lean_attn_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, sz, i32, i32, i32, i32, i32, i64,
                                     ctypes.c_float, i32, ctypes.POINTER(Tuning), vp]
    lib.lean_attn_decode_static.restype = i32
    lib.lean_attn_decode_static.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i64,
                                            ctypes.c_float, i32, ctypes.POINTER(Tuning), vp]
    lib.lean_attn_problem_workspace_size.restype = sz
    lib.lean_attn_problem_workspace_size.argtypes = [ctypes.POINTER(Problem)]
    lib.lean_attn_workspace_size_for_grid.restype = sz
    lib.lean_attn_workspace_size_for_grid.argtypes = [ctypes.POINTER(Problem), i32]
    lib.lean_attn_problem_schedule.restype = i32
    lib.lean_attn_problem_schedule.argtypes = [ctypes.POINTER(Problem), vp, ctypes.POINTER(Tuning),
                                               ctypes.POINTER(Plan)]
    lib.lean_attn_attend.restype = i32
    lib.lean_attn_attend.argtypes = [ctypes.POINTER(Problem), vp, vp, vp, vp, vp, vp, vp, sz,
                                     ctypes.POINTER(Tuning), vp]
    lib.lean_attn_launch_block_size.restype = sz
    lib.lean_attn_launch_block_size.argtypes = []
    lib.lean_attn_attend_prepare.restype = i32
    lib.lean_attn_attend_prepare.argtypes = [ctypes.POINTER(Problem), vp, vp, vp, vp, vp, vp, vp, sz,
                                             ctypes.POINTER(Tuning), vp]
    lib.lean_attn_launch.restype = i32
    lib.lean_attn_launch.argtypes = [vp, vp, vp]
    lib.lean_attn_read_probe.restype = i32
    lib.lean_attn_read_probe.argtypes = [vp, sz, vp, i32, i32, vp]
    lib.lean_attn_strerror.restype = ctypes.c_char_p
    lib.lean_attn_strerror.argtypes = [i32]
    _lib = lib
    return lib


_seqlens_cache: dict = {}


def _seqlens_array(seqlens: Sequence[int]):
    """Host int32 array for the C side; repeated calls with the same lengths reuse one array."""
    key = tuple(seqlens)
    arr = _seqlens_cache.get(key)
    if arr is None:
        if len(_seqlens_cache) > 64:
            _seqlens_cache.clear()
        arr = (ctypes.c_int32 * len(key))(*[int(x) for x in key])
        _seqlens_cache[key] = arr
    return arr


def _tuning_ptr(tuning: Optional[Tuning]):
    return ctypes.byref(tuning) if tuning is not None else None


def _stream_handle(stream) -> int:
    if stream is None:
        import torch

        return torch.cuda.current_stream().cuda_stream
    return int(getattr(stream, "cuda_stream", stream))


def _dtype_code(t) -> int:
    name = str(t.dtype)
    if name == "torch.float16":
        return F16
    if name == "torch.bfloat16":
        return BF16
    raise TypeError(f"q/k/v must be float16 or bfloat16, got {name}")


def lean_attn_strerror(status: int) -> str:
    return _load().lean_attn_strerror(int(status)).decode()


def lean_attn_workspace_size(B: int, Hq: int, Hkv: int, D: int, dtype: int) -> int:
    return int(_load().lean_attn_workspace_size(B, Hq, Hkv, D, dtype))


def lean_attn_workspace_init(workspace, stream=None) -> None:
    rc = _load().lean_attn_workspace_init(workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                          _stream_handle(stream))
    if rc != OK:
        raise LeanAttnError(rc)


def lean_attn_workspace_status(workspace, stream=None) -> int:
    return int(_load().lean_attn_workspace_status(workspace.data_ptr(), _stream_handle(stream)))


def lean_attn_schedule(seqlens, Hq, Hkv, D, dtype, kv_layout, tuning: Optional[Tuning] = None) -> Plan:
    plan = Plan()
    arr = _seqlens_array(seqlens)
    rc = _load().lean_attn_schedule(arr, len(seqlens), Hq, Hkv, D, dtype, kv_layout, _tuning_ptr(tuning),
                                    ctypes.byref(plan))
    if rc != OK:
        raise LeanAttnError(rc)
    return plan


def lean_attn_walk(plan: Plan, seqlens, Hkv, kv_layout, g, max_segments: int = 4096):
    """Segments of CTA ``g``: list of dicts (tile_idx, b, h, local_iter, local_iter_end, host, finishing, last_cta)."""
    arr = _seqlens_array(seqlens)
    buf = (ctypes.c_int64 * (8 * max_segments))()
    n = _load().lean_attn_walk(ctypes.byref(plan), arr, len(seqlens), Hkv, kv_layout, g, buf, max_segments)
    if n < 0:
        raise LeanAttnError(n)
    if n > max_segments:
        raise ValueError(f"CTA {g} walks {n} segments; raise max_segments")
    keys = ("tile_idx", "b", "h", "local_iter", "local_iter_end", "host", "finishing", "last_cta")
    return [dict(zip(keys, (int(buf[8 * i + j]) for j in range(8)))) for i in range(n)]


class PreparedCall:
    """One ``lean_attn_decode`` / ``lean_attn_attend`` call with its arguments checked and marshalled
    once: calling the object only crosses the C ABI (for loops that launch on the same buffers
    again and again, where the per-call checks above would cost more host time than the launch).
    It keeps the tensors and host arrays it points to alive; the stream is the one given (or
    current) at preparation."""
    __slots__ = ("_fn", "_args", "_keep")

    def __init__(self, fn, args, keep):
        self._fn, self._args, self._keep = fn, args, keep

    def __call__(self) -> None:
        rc = self._fn(*self._args)
        if rc != OK:
            raise LeanAttnError(rc)


def lean_attn_decode(q, k_cache, v_cache, seqlens, out, workspace, *, Hkv: int, kv_layout: int = KV_PADDED,
                     kv_seq_stride: int = 0, scale: float, lse=None, tuning: Optional[Tuning] = None,
                     stream=None, prepare_only: bool = False):
    """Launch decode attention on the current (or given) HIP stream.  Shapes as in ``lean_attn.h``.

    With ``prepare_only`` nothing is launched and a :class:`PreparedCall` is returned instead.
    ``workspace=None`` calls ``lean_attn_decode_static`` (the library's static scratch)."""
    B, Hq, D = q.shape
    if not (q.is_cuda and k_cache.is_cuda and v_cache.is_cuda and out.is_cuda and
            (workspace is None or workspace.is_cuda)):
        raise ValueError("q, k_cache, v_cache, out and workspace must be device tensors")
    if not (q.is_contiguous() and k_cache.is_contiguous() and v_cache.is_contiguous() and out.is_contiguous()):
        raise ValueError("tensors must be contiguous")
    if str(out.dtype) != "torch.float32" or tuple(out.shape) != (B, Hq, D):
        raise ValueError("out must be float32 [B, Hq, D]")
    if k_cache.dtype != q.dtype or v_cache.dtype != q.dtype or k_cache.shape != v_cache.shape:
        raise ValueError("k_cache and v_cache must match q's dtype and each other's shape")
    if len(seqlens) != B:
        raise ValueError("seqlens must have B entries")
    total = int(sum(int(x) for x in seqlens))
    if kv_layout == KV_PADDED:
        if k_cache.numel() != B * Hkv * kv_seq_stride * D:
            raise ValueError("PADDED k_cache must be [B, Hkv, kv_seq_stride, D]")
    elif k_cache.numel() != Hkv * total * D:
        raise ValueError("PACKED k_cache must be [Hkv, sum(seqlens), D]")
    if lse is not None and (str(lse.dtype) != "torch.float32" or lse.numel() != B * Hq or not lse.is_cuda):
        raise ValueError("lse must be a float32 device tensor [B, Hq]")
    arr = _seqlens_array(seqlens)
    head = (q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), arr, out.data_ptr(),
            lse.data_ptr() if lse is not None else None)
    tail = (B, Hq, Hkv, D, kv_layout, int(kv_seq_stride), float(scale), _dtype_code(q), _tuning_ptr(tuning),
            _stream_handle(stream))
    if workspace is None:
        fn, args = _load().lean_attn_decode_static, head + tail
    else:
        fn = _load().lean_attn_decode
        args = head + (workspace.data_ptr(), workspace.numel() * workspace.element_size()) + tail
    if prepare_only:
        return PreparedCall(fn, args, (q, k_cache, v_cache, out, lse, workspace, arr, tuning))
    rc = fn(*args)
    if rc != OK:
        raise LeanAttnError(rc)


def lean_attn_problem_workspace_size(problem: Problem) -> int:
    return int(_load().lean_attn_problem_workspace_size(ctypes.byref(problem)))


def lean_attn_workspace_size_for_grid(problem: Problem, max_grid: int) -> int:
    return int(_load().lean_attn_workspace_size_for_grid(ctypes.byref(problem), int(max_grid)))


def lean_attn_problem_schedule(problem: Problem, seqlens, tuning: Optional[Tuning] = None) -> Plan:
    plan = Plan()
    if len(seqlens) != problem.B:
        raise ValueError("seqlens must have B entries")
    rc = _load().lean_attn_problem_schedule(ctypes.byref(problem), _seqlens_array(seqlens), _tuning_ptr(tuning),
                                            ctypes.byref(plan))
    if rc != OK:
        raise LeanAttnError(rc)
    return plan


def lean_attn_attend(problem: Problem, q, k_cache, v_cache, seqlens, out, workspace, *, lse=None,
                     tuning: Optional[Tuning] = None, stream=None, prepare_only: bool = False):
    """Launch attention of ``problem.N_q`` query rows per sequence.  Shapes as in ``lean_attn.h``.

    With ``prepare_only`` nothing is launched and a :class:`PreparedCall` is returned instead."""
    p = problem
    if not (q.is_cuda and k_cache.is_cuda and v_cache.is_cuda and out.is_cuda and workspace.is_cuda):
        raise ValueError("q, k_cache, v_cache, out and workspace must be device tensors")
    if not (q.is_contiguous() and k_cache.is_contiguous() and v_cache.is_contiguous() and out.is_contiguous()):
        raise ValueError("tensors must be contiguous")
    n_rows = p.query_tokens() * p.Hq
    if q.numel() != n_rows * p.D or out.numel() != n_rows * p.D:
        raise ValueError("q and out must be [B, N_q, Hq, D] (or [sum(q_lens), Hq, D])")
    if _dtype_code(q) != p.dtype or k_cache.dtype != q.dtype or v_cache.dtype != q.dtype:
        raise ValueError("q, k_cache and v_cache must have the problem's element type")
    want_out = q.dtype if p.out_dtype == OUT_AS_INPUT else "torch.float32"
    if str(out.dtype) != str(want_out):
        raise ValueError(f"out must have dtype {want_out}")
    if k_cache.shape != v_cache.shape:
        raise ValueError("k_cache and v_cache must have the same shape")
    if len(seqlens) != p.B:
        raise ValueError("seqlens must have B entries")
    total = int(sum(int(x) for x in seqlens))
    if p.kv_layout == KV_PADDED:
        if k_cache.numel() != p.B * p.Hkv * p.kv_seq_stride * p.D:
            raise ValueError("PADDED k_cache must be [B, Hkv, kv_seq_stride, D]")
    elif k_cache.numel() != p.Hkv * total * p.D:
        raise ValueError("PACKED k_cache must be [Hkv, sum(seqlens), D]")
    if lse is not None and (str(lse.dtype) != "torch.float32" or lse.numel() != n_rows or not lse.is_cuda):
        raise ValueError("lse must be a float32 device tensor [B, N_q, Hq] (or [sum(q_lens), Hq])")
    arr = _seqlens_array(seqlens)
    args = (ctypes.byref(p), q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), arr,
            out.data_ptr(), lse.data_ptr() if lse is not None else None, workspace.data_ptr(),
            workspace.numel() * workspace.element_size(), _tuning_ptr(tuning), _stream_handle(stream))
    if prepare_only:
        return PreparedCall(_load().lean_attn_attend, args, (p, q, k_cache, v_cache, out, lse, workspace, arr, tuning))
    rc = _load().lean_attn_attend(*args)
    if rc != OK:
        raise LeanAttnError(rc)


def lean_attn_launch_block_size() -> int:
    return int(_load().lean_attn_launch_block_size())


def lean_attn_attend_prepare(problem: Problem, q, k_cache, v_cache, seqlens, out, workspace, block_host, *, lse=None,
                             tuning: Optional[Tuning] = None) -> None:
    """Host-only: write the launch block for :func:`lean_attn_launch` (``block_host``: a pinned uint8 CPU tensor)."""
    if block_host.is_cuda or block_host.numel() * block_host.element_size() < lean_attn_launch_block_size():
        raise ValueError("block_host must be a host tensor of lean_attn_launch_block_size() bytes")
    if len(seqlens) != problem.B:
        raise ValueError("seqlens must have B entries")
    arr = (ctypes.c_int32 * len(seqlens))(*[int(x) for x in seqlens])
    rc = _load().lean_attn_attend_prepare(
        ctypes.byref(problem), q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr(), arr, out.data_ptr(),
        lse.data_ptr() if lse is not None else None, workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _tuning_ptr(tuning), block_host.data_ptr())
    if rc != OK:
        raise LeanAttnError(rc)


def lean_attn_launch(block_host, block_device, stream=None) -> None:
    """Copy the prepared block to ``block_device`` and launch, on the current (or given) stream."""
    if block_host.is_cuda or not block_device.is_cuda:
        raise ValueError("block_host must be a (pinned) host tensor, block_device a device tensor")
    if block_device.numel() * block_device.element_size() < lean_attn_launch_block_size():
        raise ValueError("block_device must hold lean_attn_launch_block_size() bytes")
    rc = _load().lean_attn_launch(block_host.data_ptr(), block_device.data_ptr(), _stream_handle(stream))
    if rc != OK:
        raise LeanAttnError(rc)


def lean_attn_read_probe(buf, sink, grid: int, mode: int = 0, stream=None) -> None:
    rc = _load().lean_attn_read_probe(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), grid, mode,
                                      _stream_handle(stream))
    if rc != OK:
        raise LeanAttnError(rc)
