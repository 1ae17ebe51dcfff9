"""Do the oracle's pins have teeth?  Each case plants one plausible mistake in a
copy of the C oracle (CPU only, compiled into a temporary directory) and checks
that the pins of test_oracle_pins.py reject the mutant: hand-computed cases,
closed forms and the torch cross-check are re-run against the mutated library.
"""
import ctypes
import json
import math
import os
import subprocess

import numpy as np
import pytest

import oracle

SRC = os.path.join(os.path.dirname(oracle.__file__), "exact_attention.c")
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_cases.json")
QT_GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "query_tile_cases.json")

MUTANTS = {
    "scale_dropped": ("scores[t] = scale * dot;", "scores[t] = dot;"),
    "exp_sign_flipped": ("double w = exp(scores[t] - smax);", "double w = exp(smax - scores[t]);"),
    "max_not_subtracted_in_lse": ("*lse = smax + log(z);", "*lse = log(z);"),
    "not_normalised": ("for (int j = 0; j < D; ++j) out[j] /= z;", ""),
    "value_row_off_by_one": ("widen_row(v_rows, kv_off + t * D, D, dtype, row);\n        for (int j = 0; j < D; ++j) out[j] += w * row[j];",
                             "widen_row(v_rows, kv_off + (t + 1 < n ? t + 1 : t) * D, D, dtype, row);\n        for (int j = 0; j < D; ++j) out[j] += w * row[j];"),
    "kv_head_modulo_instead_of_division": ("h = hq / group;", "h = hq % Hkv;"),
    "last_token_skipped": ("for (int64_t t = 0; t < n; ++t) {\n        widen_row(k_rows,", "for (int64_t t = 0; t < n - (n > 1); ++t) {\n        widen_row(k_rows,"),
    "dot_misses_last_element": ("for (int j = 0; j < D; ++j) dot += qrow[j] * row[j];", "for (int j = 0; j < D - (D > 1); ++j) dot += qrow[j] * row[j];"),
    "bf16_shift_wrong": ("uint32_t u = ((uint32_t)bits) << 16;", "uint32_t u = ((uint32_t)bits) << 15;"),
    "packed_offset_ignores_sequence_start": (": ((int64_t)h * total + cu[b]) * D;", ": ((int64_t)h * total) * D;"),
    "causal_limit_off_by_one": ("n_visible = n_visible - q_lens[b] + i + 1;",
                                "n_visible = n_visible - q_lens[b] + i + (n_visible - q_lens[b] + i > 0 ? 0 : 1);"),
    "causal_mask_ignores_query_row": ("n_visible = n_visible - q_lens[b] + i + 1;", "n_visible = n_visible - q_lens[b] + 1;"),
    "query_row_and_head_transposed": ("int64_t token = r / Hq; /* index into the concatenated query tokens */\n            int hq = (int)(r % Hq);",
                                      "int64_t token = r % q_total;\n            int hq = (int)(r / q_total);"),
    "query_offsets_assume_equal_lengths": ("cu_q[b] = q_total;", "cu_q[b] = (int64_t)b * q_lens[0];"),
    "causal_mask_uses_the_longest_query": ("n_visible = n_visible - q_lens[b] + i + 1;",
                                           "n_visible = n_visible - q_lens[0] + i + 1;"),
    "padded_offset_ignores_head": ("? ((int64_t)(b * (int64_t)Hkv + h) * n_stride) * D", "? ((int64_t)(b * (int64_t)Hkv) * n_stride) * D"),
}


def _compile(tmp_path, name, old, new):
    text = open(SRC).read()
    assert old in text, f"mutation anchor for {name} no longer matches the oracle source"
    path = os.path.join(tmp_path, f"{name}.c")
    lib = os.path.join(tmp_path, f"lib{name}.so")
    with open(path, "w") as fh:
        fh.write(text.replace(old, new, 1))
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-w", "-o", lib, path, "-lm"])
    dll = ctypes.CDLL(lib)
    dll.oracle_decode_attention.restype = ctypes.c_int
    dll.oracle_decode_attention.argtypes = oracle._load().oracle_decode_attention.argtypes
    dll.oracle_attention.restype = ctypes.c_int
    dll.oracle_attention.argtypes = oracle._load().oracle_attention.argtypes
    dll.oracle_attention_ragged.restype = ctypes.c_int
    dll.oracle_attention_ragged.argtypes = oracle._load().oracle_attention_ragged.argtypes
    return dll


def _call(dll, q, k, v, seqlens, Hq, Hkv, D, scale, layout, n_stride, code):
    sl = np.ascontiguousarray(np.asarray(seqlens, dtype=np.int32))
    B = len(seqlens)
    out = np.empty((B, Hq, D))
    lse = np.empty((B, Hq))
    rc = dll.oracle_decode_attention(q.ctypes.data, k.ctypes.data, v.ctypes.data, sl.ctypes.data, B, Hq, Hkv, D, code,
                                     layout, n_stride, scale, out.ctypes.data, lse.ctypes.data, 1)
    assert rc > 0
    return out, lse


def _call_tile(dll, q, k, v, seqlens, N_q, Hq, Hkv, D, scale, causal, n_stride):
    sl = np.ascontiguousarray(np.asarray(seqlens, dtype=np.int32))
    B = len(seqlens)
    out = np.empty((B, N_q, Hq, D))
    lse = np.empty((B, N_q, Hq))
    rc = dll.oracle_attention(q.ctypes.data, k.ctypes.data, v.ctypes.data, sl.ctypes.data, B, N_q, Hq, Hkv, D,
                              oracle.F64, 0, n_stride, scale, int(causal), out.ctypes.data, lse.ctypes.data, 1)
    assert rc > 0
    return out, lse


def _pins_hold(dll) -> bool:
    """A condensed run of the pins; True when every one of them passes."""
    try:
        # hand-computed cases (Eq. 1)
        for case in json.load(open(GOLDEN))["cases"]:
            q = np.array(case["q"], dtype=np.float64)
            klog, kplain = case["k_log_of"], case["k_plain"]
            N, D = len(klog), len(klog[0])
            k = np.array([[math.log(klog[t][j]) if klog[t][j] is not None else kplain[t][j] for j in range(D)]
                          for t in range(N)])
            v = np.array(case["v"], dtype=np.float64)
            out, lse = _call(dll, q, k, v, [N], case["Hq"], case["Hkv"], D, case["scale"], 0, N, oracle.F64)
            if np.max(np.abs(out[0] - np.array(case["out"]))) > 1e-12:
                return False
            if np.max(np.abs(lse[0] - np.log(np.array(case["lse_log_of"])))) > 1e-12:
                return False
        # torch-free cross-check against the textbook definition on random fp64 data, GQA, two layouts
        r = np.random.default_rng(0)
        B, Hq, Hkv, D = 3, 4, 2, 5
        lens = [6, 1, 9]
        nmax = max(lens)
        q = r.normal(size=(B, Hq, D))
        k = r.normal(size=(B, Hkv, nmax, D))
        v = r.normal(size=(B, Hkv, nmax, D))
        kp = np.ascontiguousarray(np.concatenate([k[b, :, :lens[b]] for b in range(B)], axis=1))
        vp = np.ascontiguousarray(np.concatenate([v[b, :, :lens[b]] for b in range(B)], axis=1))
        for layout, kk, vv in ((0, k, v), (1, kp, vp)):
            out, lse = _call(dll, q, kk, vv, lens, Hq, Hkv, D, 0.4, layout, nmax, oracle.F64)
            for b in range(B):
                for h in range(Hq):
                    s = 0.4 * (k[b, h // 2, :lens[b]] @ q[b, h])
                    wgt = np.exp(s - s.max())
                    want = (wgt / wgt.sum()) @ v[b, h // 2, :lens[b]]
                    if np.max(np.abs(out[b, h] - want)) > 1e-12:
                        return False
                    if abs(lse[b, h] - (s.max() + math.log(wgt.sum()))) > 1e-12:
                        return False
        # hand-computed query tiles (N_q = 2), causal and unmasked
        for case in json.load(open(QT_GOLDEN))["cases"]:
            q = np.array(case["q"], dtype=np.float64)
            N_q, Hq = q.shape
            k = np.log(np.array(case["k_log_of"], dtype=np.float64))
            v = np.array(case["v"], dtype=np.float64)
            for causal, tag in ((True, "causal"), (False, "full")):
                out, lse = _call_tile(dll, np.ascontiguousarray(q), k, v, [k.size], N_q, Hq, case["Hkv"], 1, 1.0,
                                      causal, k.size)
                if np.max(np.abs(out[0, :, :, 0] - np.array(case[f"out_{tag}"]))) > 1e-12:
                    return False
                if np.max(np.abs(lse[0] - np.log(np.array(case[f"lse_{tag}_log_of"])))) > 1e-12:
                    return False
        # per-sequence query lengths against the masked score matrix, sequence by sequence
        r = np.random.default_rng(3)
        B, Hq, Hkv, D = 3, 2, 1, 3
        lens, q_lens = [5, 4, 6], [3, 1, 2]
        nmax = max(lens)
        q = r.normal(size=(sum(q_lens), Hq, D))
        k = r.normal(size=(B, Hkv, nmax, D))
        v = r.normal(size=(B, Hkv, nmax, D))
        sl = np.asarray(lens, dtype=np.int32)
        ql = np.asarray(q_lens, dtype=np.int32)
        out = np.empty((sum(q_lens), Hq, D))
        lse = np.empty((sum(q_lens), Hq))
        rc = dll.oracle_attention_ragged(q.ctypes.data, k.ctypes.data, v.ctypes.data, sl.ctypes.data, ql.ctypes.data, B,
                                         Hq, Hkv, D, oracle.F64, 0, nmax, 0.6, 1, out.ctypes.data, lse.ctypes.data, 1)
        if rc <= 0:
            return False
        start = 0
        for b in range(B):
            n, nq = lens[b], q_lens[b]
            for h in range(Hq):
                S = 0.6 * q[start:start + nq, h] @ k[b, 0, :n].T
                S = np.where(np.arange(n)[None, :] <= np.arange(nq)[:, None] + (n - nq), S, -np.inf)
                P = np.exp(S - S.max(axis=1, keepdims=True))
                want = (P / P.sum(axis=1, keepdims=True)) @ v[b, 0, :n]
                if np.max(np.abs(out[start:start + nq, h] - want)) > 1e-12:
                    return False
            start += nq
        # bf16 widening: q = 1.0, one token, v carries the pattern
        bits = np.array([0x3F80, 0x4049, 0xC2F7, 0x0080, 0x3EAA], dtype=np.uint16)
        want = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        n = bits.size
        out, _ = _call(dll, np.full((n, 1, 1), 0x3F80, np.uint16), np.zeros((n, 1, 1, 1), np.uint16),
                       bits.reshape(n, 1, 1, 1).copy(), [1] * n, 1, 1, 1, 1.0, 0, 1, oracle.BF16)
        if not np.array_equal(out.ravel(), want):
            return False
        return True
    except AssertionError:
        return False


def test_unmutated_oracle_passes_the_condensed_pins(tmp_path):
    dll = _compile(str(tmp_path), "identity", "double z = 0.0;", "double z = 0.0;")
    assert _pins_hold(dll)


@pytest.mark.parametrize("name", sorted(MUTANTS))
def test_pins_reject_planted_mistake(tmp_path, name):
    old, new = MUTANTS[name]
    dll = _compile(str(tmp_path), name, old, new)
    assert not _pins_hold(dll), f"the pins did not notice the planted mistake '{name}'"
