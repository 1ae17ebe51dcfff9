"""``lean_attn_decode_static``: the decode entry point whose workspace is a static device array.

It must give what ``lean_attn_decode`` gives on a caller-provided workspace (same kernels, same
schedule: bit for bit), and the oracle's result within the parity bar, call after call on the one
shared array: the second call below is a smaller problem that leaves most of the array as the
first call wrote it.
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2405_10480_amd as la
import workloads

pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2 = 2e-3, 1e-3


def _c_abi():
    lib = ctypes.CDLL(la.library_path())
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    lib.lean_attn_decode_static.restype = i32
    lib.lean_attn_decode_static.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i64, ctypes.c_float, i32,
                                            vp, vp]
    lib.lean_attn_decode.restype = i32
    lib.lean_attn_decode.argtypes = [vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, i32, i32, i32, i32, i32, i64,
                                     ctypes.c_float, i32, vp, vp]
    return lib


def _both(lib, w, tuning=None):
    """The same problem through the static entry point and through lean_attn_decode; returns both outputs."""
    inp = workloads.generate(w, device="cuda")
    code = la.F16 if w.dtype == "f16" else la.BF16
    seq = (ctypes.c_int32 * w.B)(*inp.seqlens)
    stream = torch.cuda.current_stream().cuda_stream
    tn = ctypes.byref(tuning) if tuning is not None else None
    outs = []
    for static in (True, False):
        out = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.float32, device="cuda")
        lse = torch.full((w.B, w.Hq), float("nan"), dtype=torch.float32, device="cuda")
        if static:
            rc = lib.lean_attn_decode_static(inp.q.data_ptr(), inp.k.data_ptr(), inp.v.data_ptr(), seq, out.data_ptr(),
                                             lse.data_ptr(), w.B, w.Hq, w.Hkv, w.D, w.kv_layout, w.n_stride, w.scale,
                                             code, tn, stream)
        else:
            ws = torch.empty(la.lean_attn_workspace_size(w.B, w.Hq, w.Hkv, w.D, code), dtype=torch.uint8, device="cuda")
            la.lean_attn_workspace_init(ws)
            rc = lib.lean_attn_decode(inp.q.data_ptr(), inp.k.data_ptr(), inp.v.data_ptr(), seq, out.data_ptr(),
                                      lse.data_ptr(), ws.data_ptr(), ws.numel(), w.B, w.Hq, w.Hkv, w.D, w.kv_layout,
                                      w.n_stride, w.scale, code, tn, stream)
        assert rc == 0, la.lean_attn_strerror(rc)
        torch.cuda.synchronize()
        outs.append((out, lse))
    want, want_lse = oracle.decode_attention(inp.q, inp.k, inp.v, inp.seqlens, Hq=w.Hq, Hkv=w.Hkv, D=w.D, scale=w.scale,
                                             kv_layout=w.kv_layout, n_stride=w.n_stride)
    return outs[0], outs[1], want, want_lse


def _check(w, got, ref, want, want_lse):
    out, lse = got
    assert torch.equal(out, ref[0]) and torch.equal(lse, ref[1]), f"{w.name}: static scratch and workspace differ"
    max_abs, rel_l2 = oracle.error_metrics(out.cpu().numpy(), want)
    assert max_abs <= MAX_ABS and rel_l2 <= REL_L2, f"{w.name}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}"
    fin = np.isfinite(want_lse)
    assert np.max(np.abs(lse.cpu().numpy()[fin] - want_lse[fin]), initial=0.0) <= 1e-4


def test_static_scratch_matches_the_workspace_entry_point_on_consecutive_calls():
    lib = _c_abi()
    # a query group (8-row partial slots, a two-level reduction tree over a full grid), ragged, packed
    big = workloads.Workload("static_gqa", 3, 32, 4, 128, "bf16", (40001, 9000, 300), workloads.KV_PACKED, seed=71,
                             outlier_frac=0.01)
    # then a much smaller single-row problem: fewer workgroups, smaller slots, an empty sequence
    small = workloads.Workload("static_mha", 3, 4, 4, 64, "f16", (1500, 0, 77), workloads.KV_PADDED, seed=72)
    for w in (big, small, big):
        got, ref, want, want_lse = _both(lib, w)
        _check(w, got, ref, want, want_lse)
    # a forced grid of the largest allowed size, a deep tree
    got, ref, want, want_lse = _both(lib, big, la.Tuning(grid=la.binding.STATIC_MAX_GRID, merge_fanin=2))
    _check(big, got, ref, want, want_lse)


def test_static_scratch_rejects_what_does_not_fit_and_launches_nothing():
    lib = _c_abi()
    w = workloads.Workload("static_limit", 1, 16, 2, 128, "bf16", (70000,), workloads.KV_PADDED, seed=73)
    inp = workloads.generate(w, device="cuda")
    seq = (ctypes.c_int32 * 1)(*inp.seqlens)
    out = torch.full((1, 16, 128), 7.0, dtype=torch.float32, device="cuda")
    tn = la.Tuning(grid=la.binding.STATIC_MAX_GRID + 1)
    rc = lib.lean_attn_decode_static(inp.q.data_ptr(), inp.k.data_ptr(), inp.v.data_ptr(), seq, out.data_ptr(), None,
                                     1, 16, 2, 128, w.kv_layout, w.n_stride, w.scale, la.BF16, ctypes.byref(tn),
                                     torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert rc == la.binding.ERR_STATIC_LIMIT and torch.all(out == 7.0)
    assert "static" in la.lean_attn_strerror(rc)
    # the binding reaches the same entry point with workspace=None
    la.lean_attn_decode(inp.q, inp.k, inp.v, inp.seqlens, out, None, Hkv=2, kv_seq_stride=w.n_stride, scale=w.scale)
    torch.cuda.synchronize()
    want, _ = oracle.decode_attention(inp.q, inp.k, inp.v, inp.seqlens, Hq=16, Hkv=2, D=128, scale=w.scale,
                                      kv_layout=w.kv_layout, n_stride=w.n_stride)
    max_abs, rel_l2 = oracle.error_metrics(out.cpu().numpy(), want)
    assert max_abs <= MAX_ABS and rel_l2 <= REL_L2
