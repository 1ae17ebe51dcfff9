"""Pins for the CPU oracle: closed forms, hand-computed cases, invariants,
brute-force split/merge, a library cross-check and the Algorithm 2 emulation.
Each test is chosen so that a plausible slip in the oracle (dropped scale,
wrong sign, transposed operand, wrong head mapping, off-by-one span) fails it.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import rescale, stream_k

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_cases.json")


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- hand cases (Eq. 1)
def _load_cases():
    with open(GOLDEN) as fh:
        return json.load(fh)["cases"]


@pytest.mark.parametrize("case", _load_cases(), ids=lambda c: c["name"])
def test_hand_computed_cases(case):
    q = np.array(case["q"], dtype=np.float64)
    klog = case["k_log_of"]
    kplain = case["k_plain"]
    N, D = len(klog), len(klog[0])
    k = np.zeros((N, D))
    for t in range(N):
        for j in range(D):
            k[t, j] = math.log(klog[t][j]) if klog[t][j] is not None else kplain[t][j]
    v = np.array(case["v"], dtype=np.float64)
    Hq, Hkv = case["Hq"], case["Hkv"]
    out, lse = oracle.decode_attention(q.reshape(1, Hq, D), k.reshape(1, Hkv, N, D), v.reshape(1, Hkv, N, D),
                                       [N], Hq=Hq, Hkv=Hkv, D=D, scale=case["scale"], n_stride=N,
                                       dtype=oracle.F64)
    np.testing.assert_allclose(out[0], np.array(case["out"]), rtol=0, atol=1e-13)
    np.testing.assert_allclose(lse[0], np.log(np.array(case["lse_log_of"])), rtol=0, atol=1e-13)


# ---------------------------------------------------------------- closed forms
def test_equal_scores_give_mean_of_v():
    r = _rng(1)
    N, D = 37, 8
    v = r.normal(size=(N, D))
    # (a) zero query: every score is 0
    out, lse = oracle.attention_row(np.zeros(D), r.normal(size=(N, D)), v, 0.7)
    np.testing.assert_allclose(out, v.mean(axis=0), atol=1e-14)
    assert abs(lse - math.log(N)) < 1e-14
    # (b) identical key rows: every score is the same non-zero s
    q = r.normal(size=D)
    krow = r.normal(size=D)
    s = 0.3 * float(q @ krow)
    out, lse = oracle.attention_row(q, np.tile(krow, (N, 1)), v, 0.3)
    np.testing.assert_allclose(out, v.mean(axis=0), atol=1e-13)
    assert abs(lse - (s + math.log(N))) < 1e-12


def test_single_token_returns_its_value_row():
    r = _rng(2)
    D = 16
    q, k, v = r.normal(size=D), r.normal(size=(1, D)), r.normal(size=(1, D))
    out, lse = oracle.attention_row(q, k, v, 0.25)
    np.testing.assert_array_equal(out, v[0])
    assert abs(lse - 0.25 * float(q @ k[0])) < 1e-14


def test_dominant_score_selects_its_value_row():
    r = _rng(3)
    N, D, tstar, c = 50, 8, 17, 40.0
    q = r.normal(size=D)
    k = np.zeros((N, D))
    k[tstar] = c * q / np.linalg.norm(q) ** 2        # score c at t*, 0 elsewhere (scale 1)
    v = r.normal(size=(N, D))
    out, lse = oracle.attention_row(q, k, v, 1.0)
    bound = (N - 1) * math.exp(-c) * 2 * np.abs(v).max()
    assert np.max(np.abs(out - v[tstar])) <= bound
    assert abs(lse - c) <= (N - 1) * math.exp(-c) * 1.01 + 4 * np.finfo(np.float64).eps * c


def test_two_token_sigmoid_closed_form():
    # N = 2: weights are sigmoid(+-(s0 - s1)); checks the sign inside the exponential
    q = np.array([1.0, 2.0])
    k = np.array([[0.5, -1.0], [2.0, 0.25]])
    v = np.array([[1.0, 0.0], [0.0, 1.0]])
    scale = 0.9
    s0, s1 = scale * (q @ k[0]), scale * (q @ k[1])
    w0 = 1.0 / (1.0 + math.exp(s1 - s0))
    out, lse = oracle.attention_row(q, k, v, scale)
    np.testing.assert_allclose(out, [w0, 1.0 - w0], atol=1e-15)
    assert abs(lse - (max(s0, s1) + math.log1p(math.exp(-abs(s0 - s1))))) < 1e-14


# ---------------------------------------------------------------- invariants
def test_shift_permutation_and_convex_hull():
    r = _rng(4)
    N, D = 64, 8
    q, k, v = r.normal(size=D), r.normal(size=(N, D)), r.normal(size=(N, D))
    out, lse = oracle.attention_row(q, k, v, 0.5)
    # permutation of (k_t, v_t) pairs
    p = r.permutation(N)
    out_p, lse_p = oracle.attention_row(q, k[p], v[p], 0.5)
    np.testing.assert_allclose(out_p, out, atol=1e-14)
    assert abs(lse_p - lse) < 1e-13
    # adding c*q/|q|^2 to every key shifts every score by scale*c
    c = 3.0
    out_s, lse_s = oracle.attention_row(q, k + c * q / (q @ q), v, 0.5)
    np.testing.assert_allclose(out_s, out, atol=1e-13)
    assert abs(lse_s - (lse + 0.5 * c)) < 1e-12
    # a convex combination of the value rows
    assert np.all(out <= v.max(axis=0) + 1e-15) and np.all(out >= v.min(axis=0) - 1e-15)
    # constant value column is reproduced (weights sum to one)
    v1 = v.copy()
    v1[:, 3] = 2.5
    out_c, _ = oracle.attention_row(q, k, v1, 0.5)
    assert abs(out_c[3] - 2.5) < 1e-14


def test_scale_is_applied_to_scores():
    r = _rng(5)
    N, D = 20, 4
    q, k, v = r.normal(size=D), r.normal(size=(N, D)), r.normal(size=(N, D))
    a, la = oracle.attention_row(q, k, v, 0.5)
    b, lb = oracle.attention_row(2.0 * q, k, v, 0.25)      # same scores
    np.testing.assert_allclose(a, b, atol=1e-14)
    c, _ = oracle.attention_row(q, k, v, 1.0)
    assert np.max(np.abs(a - c)) > 1e-3                    # and the scale matters


# ---------------------------------------------------------------- library cross-check
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_against_torch_softmax(seed):
    g = torch.Generator().manual_seed(seed)
    B, Hq, Hkv, N, D = 2, 6, 2, 45, 16
    q = torch.randn(B, Hq, D, generator=g, dtype=torch.float64)
    k = torch.randn(B, Hkv, N, D, generator=g, dtype=torch.float64)
    v = torch.randn(B, Hkv, N, D, generator=g, dtype=torch.float64)
    lens = [N, 31]
    out, lse = oracle.decode_attention(q, k, v, lens, Hq=Hq, Hkv=Hkv, D=D, scale=0.25, n_stride=N,
                                       dtype=oracle.F64)
    for b in range(B):
        for h in range(Hq):
            kk, vv = k[b, h // (Hq // Hkv), :lens[b]], v[b, h // (Hq // Hkv), :lens[b]]
            s = 0.25 * (kk @ q[b, h])
            want = torch.softmax(s, -1) @ vv
            np.testing.assert_allclose(out[b, h], want.numpy(), atol=1e-13)
            assert abs(lse[b, h] - float(torch.logsumexp(s, -1))) < 1e-12


# ---------------------------------------------------------------- 16-bit widening
def test_f16_widening_all_patterns():
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    finite = np.isfinite(want)
    # q = 1, one token, D = 1 => out = v exactly; run the finite patterns through v
    vals = bits[finite]
    n = vals.size
    out, _ = oracle.decode_attention(np.full((n, 1, 1), 0x3C00, np.uint16), np.zeros((n, 1, 1, 1), np.uint16),
                                     vals.reshape(n, 1, 1, 1), [1] * n, Hq=1, Hkv=1, D=1, scale=1.0,
                                     n_stride=1, dtype=oracle.F16)
    np.testing.assert_array_equal(out.ravel(), want[finite])


def test_bf16_widening_all_patterns():
    bits = torch.arange(65536, dtype=torch.int32).to(torch.int16)
    want = bits.view(torch.bfloat16).to(torch.float64).numpy()
    finite = np.isfinite(want)
    vals = bits.numpy().view(np.uint16)[finite]
    n = vals.size
    one = 0x3F80
    out, _ = oracle.decode_attention(np.full((n, 1, 1), one, np.uint16), np.zeros((n, 1, 1, 1), np.uint16),
                                     vals.reshape(n, 1, 1, 1), [1] * n, Hq=1, Hkv=1, D=1, scale=1.0,
                                     n_stride=1, dtype=oracle.BF16)
    np.testing.assert_array_equal(out.ravel(), want[finite])


# ---------------------------------------------------------------- layouts, GQA, edge cases
def test_gqa_equals_mha_on_repeated_kv_heads_and_packed_equals_padded():
    g = torch.Generator().manual_seed(7)
    B, Hq, Hkv, D = 3, 6, 2, 8
    lens = [5, 1, 9]
    nmax = max(lens)
    q = torch.randn(B, Hq, D, generator=g).to(torch.bfloat16)
    k = torch.randn(B, Hkv, nmax, D, generator=g).to(torch.bfloat16)
    v = torch.randn(B, Hkv, nmax, D, generator=g).to(torch.bfloat16)
    out, lse = oracle.decode_attention(q, k, v, lens, Hq=Hq, Hkv=Hkv, D=D, scale=0.3, n_stride=nmax)
    krep = k.repeat_interleave(Hq // Hkv, dim=1)
    vrep = v.repeat_interleave(Hq // Hkv, dim=1)
    out2, lse2 = oracle.decode_attention(q, krep, vrep, lens, Hq=Hq, Hkv=Hq, D=D, scale=0.3, n_stride=nmax)
    np.testing.assert_array_equal(out, out2)
    np.testing.assert_array_equal(lse, lse2)
    kp = torch.cat([k[b, :, :lens[b]] for b in range(B)], dim=1).contiguous()
    vp = torch.cat([v[b, :, :lens[b]] for b in range(B)], dim=1).contiguous()
    out3, lse3 = oracle.decode_attention(q, kp, vp, lens, Hq=Hq, Hkv=Hkv, D=D, scale=0.3,
                                         kv_layout=oracle.KV_PACKED)
    np.testing.assert_array_equal(out, out3)
    np.testing.assert_array_equal(lse, lse3)


def test_empty_context_gives_zero_and_minus_inf():
    q = np.ones((2, 1, 4))
    k = np.ones((2, 1, 3, 4))
    out, lse = oracle.decode_attention(q, k, k, [0, 3], Hq=1, Hkv=1, D=4, scale=1.0, n_stride=3,
                                       dtype=oracle.F64)
    assert np.all(out[0] == 0) and lse[0, 0] == -np.inf
    np.testing.assert_allclose(out[1], 1.0)


def test_bad_arguments_are_rejected():
    q = np.ones((1, 3, 4))
    k = np.ones((1, 2, 3, 4))
    with pytest.raises(ValueError):
        oracle._load()  # make sure the library is there
        oracle.decode_attention(q, k, k, [3], Hq=3, Hkv=2, D=4, scale=1.0, n_stride=3, dtype=oracle.F64)


# ---------------------------------------------------------------- operator f (Section 4.1)
def _compositions(n):
    for cuts in itertools.product([0, 1], repeat=n - 1):
        parts, size = [], 1
        for c in cuts:
            if c:
                parts.append(size)
                size = 1
            else:
                size += 1
        parts.append(size)
        yield parts


def _all_bracketings(items):
    """Every full binary bracketing of a sequence, merged with f."""
    if len(items) == 1:
        yield items[0]
        return
    for cut in range(1, len(items)):
        for left in _all_bracketings(items[:cut]):
            for right in _all_bracketings(items[cut:]):
                yield rescale.f(left, right)


@pytest.mark.parametrize("N", [1, 2, 3, 5, 7])
def test_every_split_and_every_bracketing_equals_unsplit(N):
    r = _rng(100 + N)
    D = 3
    q, k, v = r.normal(size=D), 3.0 * r.normal(size=(N, D)), r.normal(size=(N, D))
    want, want_lse = oracle.attention_row(q, k, v, 0.8)
    count = 0
    for parts in _compositions(N):
        blocks, t = [], 0
        for p in parts:
            blocks.append(rescale.partial(q, k[t:t + p], v[t:t + p], 0.8))
            t += p
        for merged in _all_bracketings(blocks):
            got, got_lse = rescale.finalize(merged)
            assert np.max(np.abs(got - want)) < 1e-12
            assert abs(got_lse - want_lse) < 1e-12
            count += 1
    assert count >= 1


def test_operator_is_associative_and_has_identity():
    r = _rng(9)
    D = 5
    xs = [(r.normal(size=D), float(r.normal() * 10), float(r.uniform(0.1, 50))) for _ in range(3)]
    x, y, z = xs
    a = rescale.f(rescale.f(x, y), z)
    b = rescale.f(x, rescale.f(y, z))
    np.testing.assert_allclose(a[0], b[0], rtol=1e-13)
    assert a[1] == b[1] and abs(a[2] - b[2]) < 1e-12 * abs(a[2])
    # closed form of the three-way merge (last line of the associativity proof)
    m = max(x[1], y[1], z[1])
    want = sum(math.exp(t[1] - m) * t[0] for t in xs)
    np.testing.assert_allclose(a[0], want, rtol=1e-13)
    # identity element of Algorithm 1's initial state, both sides, and with itself
    e = rescale.identity(D)
    for merged in (rescale.f(e, x), rescale.f(x, e)):
        np.testing.assert_array_equal(merged[0], x[0])
        assert merged[1] == x[1] and merged[2] == x[2]
    ee = rescale.f(e, e)
    assert np.all(ee[0] == 0) and ee[1] == -np.inf and ee[2] == 0.0
    assert not np.any(np.isnan(rescale.finalize(ee)[0]))


def test_random_unequal_splits_large_dynamic_range():
    r = _rng(11)
    N, D = 300, 8
    q, v = r.normal(size=D), r.normal(size=(N, D))
    k = r.normal(size=(N, D))
    k[r.random(N) < 0.05] *= 30.0                      # outlier keys: the running max jumps
    want, want_lse = oracle.attention_row(q, k, v, 1.0)
    for _ in range(20):
        cuts = np.sort(r.choice(np.arange(1, N), size=int(r.integers(1, 12)), replace=False))
        edges = [0, *cuts.tolist(), N]
        acc = rescale.identity(D)
        order = r.permutation(len(edges) - 1)          # f is commutative too: merge in any order
        for i in order:
            acc = rescale.f(acc, rescale.partial(q, k[edges[i]:edges[i + 1]], v[edges[i]:edges[i + 1]], 1.0))
        got, got_lse = rescale.finalize(acc)
        assert np.max(np.abs(got - want)) < 1e-11 and abs(got_lse - want_lse) < 1e-11


# ---------------------------------------------------------------- the stream-K decomposition (Section 4.3)
def test_spans_match_the_schedule_of_figure_1():
    # Figure 1 / Section 4.1: 5 SMs, 2 heads, 5 LeanTiles per head: two per CTA;
    # CTA0 and CTA1 take two tiles of head 0, CTA2 one of head 0 and one of head 1.
    assert stream_k.spans(10, 5) == [(0, 2), (2, 4), (4, 6), (6, 8), (8, 10)]
    trace = []
    r = _rng(12)
    T_n, N, D = 4, 20, 4
    q = r.normal(size=(1, 2, D))
    k = r.normal(size=(1, 2, N, D))
    v = r.normal(size=(1, 2, N, D))
    stream_k.attention_by_spans(q, k, v, [N], Hkv=2, T_n=T_n, G=5, scale=0.5, trace=trace)
    seg = {(t["cta"], t["h"]): t for t in trace}
    assert seg[(0, 0)]["host"] and not seg[(0, 0)]["finishing"]
    assert (seg[(2, 0)]["local_iter"], seg[(2, 0)]["local_iter_end"]) == (4, 5)
    assert not seg[(2, 0)]["host"] and seg[(2, 0)]["finishing"]
    assert seg[(2, 1)]["host"] and (seg[(2, 1)]["local_iter"], seg[(2, 1)]["local_iter_end"]) == (0, 1)
    assert (4, 0) not in seg and seg[(4, 1)]["finishing"]


def test_grid_formula_example_from_section_4_3():
    # 108 SMs x 2 CTAs per SM = 216; equal tiles per CTA when the count divides
    G = 108 * 2
    sp = stream_k.spans(G * 7, G)
    assert len(sp) == 216 and all(e - s == 7 for s, e in sp)
    sp = stream_k.spans(G * 7 + 5, G)
    assert [e - s for s, e in sp].count(8) == 5 and sp[-1][1] == G * 7 + 5
    assert len(stream_k.spans(3, 216)) == 3          # never more CTAs than iterations


@pytest.mark.parametrize("G", [1, 2, 3, 5, 7, 16, 33, 1000])
@pytest.mark.parametrize("T_n", [1, 4, 7])
def test_stream_k_pieces_folded_with_f_equal_exact_attention(G, T_n):
    r = _rng(1000 + G * 10 + T_n)
    B, Hq, Hkv, D = 3, 6, 2, 4
    lens = [23, 1, 10]
    nmax = max(lens)
    q = r.normal(size=(B, Hq, D))
    k = 2.0 * r.normal(size=(B, Hkv, nmax, D))
    v = r.normal(size=(B, Hkv, nmax, D))
    want, want_lse = oracle.decode_attention(q, k, v, lens, Hq=Hq, Hkv=Hkv, D=D, scale=0.6, n_stride=nmax,
                                             dtype=oracle.F64)
    trace = []
    got, got_lse = stream_k.attention_by_spans(q, k, v, lens, Hkv=Hkv, T_n=T_n, G=G, scale=0.6, trace=trace)
    np.testing.assert_allclose(got, want, atol=1e-12)
    np.testing.assert_allclose(got_lse, want_lse, atol=1e-12)
    # the pieces of a tile may be folded in any order and bracketing (Section 4.1)
    got, got_lse = stream_k.attention_by_spans(q, k, v, lens, Hkv=Hkv, T_n=T_n, G=G, scale=0.6, rng=r)
    np.testing.assert_allclose(got, want, atol=1e-12)
    np.testing.assert_allclose(got_lse, want_lse, atol=1e-12)
    # every output tile has exactly one host segment; every iteration is covered once
    hosts = {}
    covered = {}
    for t in trace:
        key = (t["b"], t["h"])
        hosts[key] = hosts.get(key, 0) + (1 if t["host"] else 0)
        covered[key] = covered.get(key, 0) + t["local_iter_end"] - t["local_iter"]
    for b in range(B):
        for h in range(Hkv):
            assert hosts[(b, h)] == 1
            assert covered[(b, h)] == math.ceil(lens[b] / T_n)


def test_stream_k_special_cases_of_section_4_3():
    r = _rng(77)
    B, H, D, T_n, N = 2, 3, 4, 4, 32                    # 6 output tiles, 8 iterations each
    q, k, v = r.normal(size=(B, H, D)), r.normal(size=(B, H, N, D)), r.normal(size=(B, H, N, D))
    # grid == number of output tiles: nobody stores a partial (FlashAttention-2 behaviour)
    trace = []
    stream_k.attention_by_spans(q, k, v, [N, N], Hkv=H, T_n=T_n, G=6, scale=0.5, trace=trace)
    assert all(t["host"] and t["finishing"] for t in trace) and len(trace) == 6
    # grid an even multiple: every tile split into the same number of equal parts (fixed split)
    trace = []
    stream_k.attention_by_spans(q, k, v, [N, N], Hkv=H, T_n=T_n, G=12, scale=0.5, trace=trace)
    assert len(trace) == 12 and all(t["local_iter_end"] - t["local_iter"] == 4 for t in trace)
    assert sum(t["host"] for t in trace) == 6


# ---------------------------------------------------------------- query tiles (N_q > 1)
QT_GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "query_tile_cases.json")


def _load_query_tile_cases():
    with open(QT_GOLDEN) as fh:
        return json.load(fh)["cases"]


@pytest.mark.parametrize("case", _load_query_tile_cases(), ids=lambda c: c["name"])
def test_hand_computed_query_tile_cases(case):
    q = np.array(case["q"], dtype=np.float64)                      # [N_q, Hq]
    N_q, Hq = q.shape
    k = np.log(np.array(case["k_log_of"], dtype=np.float64))
    v = np.array(case["v"], dtype=np.float64)
    N = k.size
    for causal, tag in ((True, "causal"), (False, "full")):
        out, lse = oracle.attention(q.reshape(1, N_q, Hq, 1), k.reshape(1, 1, N, 1), v.reshape(1, 1, N, 1), [N],
                                    N_q=N_q, Hq=Hq, Hkv=case["Hkv"], D=1, scale=1.0, causal=causal, n_stride=N,
                                    dtype=oracle.F64)
        np.testing.assert_allclose(out[0, :, :, 0], np.array(case[f"out_{tag}"]), rtol=0, atol=1e-13)
        np.testing.assert_allclose(lse[0], np.log(np.array(case[f"lse_{tag}_log_of"])), rtol=0, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("layout", [oracle.KV_PADDED, oracle.KV_PACKED])
def test_query_tiles_against_masked_score_matrix(causal, layout):
    # textbook form: S = scale * Q K^T with an explicit mask matrix, row softmax, P V
    r = _rng(40 + int(causal))
    B, N_q, Hq, Hkv, D = 4, 3, 6, 2, 5
    lens = [7, 3, 0, 12]                      # one sequence holds exactly the N_q new tokens, one is empty
    nmax, scale = max(lens), 0.37
    q = r.normal(size=(B, N_q, Hq, D))
    k = r.normal(size=(B, Hkv, nmax, D))
    v = r.normal(size=(B, Hkv, nmax, D))
    if layout == oracle.KV_PACKED:
        kk = np.ascontiguousarray(np.concatenate([k[b, :, :lens[b]] for b in range(B)], axis=1))
        vv = np.ascontiguousarray(np.concatenate([v[b, :, :lens[b]] for b in range(B)], axis=1))
    else:
        kk, vv = k, v
    out, lse = oracle.attention(q, kk, vv, lens, N_q=N_q, Hq=Hq, Hkv=Hkv, D=D, scale=scale, causal=causal,
                                kv_layout=layout, n_stride=nmax, dtype=oracle.F64)
    group = Hq // Hkv
    for b in range(B):
        n = lens[b]
        if n == 0:
            assert np.all(out[b] == 0) and np.all(np.isneginf(lse[b]))
            continue
        for hq in range(Hq):
            S = scale * q[b, :, hq] @ k[b, hq // group, :n].T            # [N_q, n]
            if causal:
                rows = np.arange(N_q)[:, None] + (n - N_q)
                S = np.where(np.arange(n)[None, :] <= rows, S, -np.inf)
            P = np.exp(S - S.max(axis=1, keepdims=True))
            want = (P / P.sum(axis=1, keepdims=True)) @ v[b, hq // group, :n]
            np.testing.assert_allclose(out[b, :, hq], want, rtol=0, atol=1e-13)
            np.testing.assert_allclose(lse[b, :, hq], S.max(axis=1) + np.log(P.sum(axis=1)), rtol=0, atol=1e-13)


def test_causal_query_rows_are_decode_steps_on_truncated_contexts():
    # row i of a causal query tile is exactly the decode step taken when the context held
    # N - N_q + i + 1 tokens; the last row and every row of the unmasked form see all N
    r = _rng(42)
    B, N_q, Hq, Hkv, D = 2, 4, 4, 2, 8
    lens = [9, 4]
    nmax = max(lens)
    q = r.normal(size=(B, N_q, Hq, D))
    k = r.normal(size=(B, Hkv, nmax, D))
    v = r.normal(size=(B, Hkv, nmax, D))
    kw = dict(Hq=Hq, Hkv=Hkv, D=D, scale=0.5, n_stride=nmax, dtype=oracle.F64)
    out_c, lse_c = oracle.attention(q, k, v, lens, N_q=N_q, causal=True, **kw)
    out_f, lse_f = oracle.attention(q, k, v, lens, N_q=N_q, causal=False, **kw)
    for i in range(N_q):
        step, step_lse = oracle.decode_attention(np.ascontiguousarray(q[:, i]), k, v, [n - N_q + i + 1 for n in lens], **kw)
        assert np.array_equal(out_c[:, i], step) and np.array_equal(lse_c[:, i], step_lse)
        full, full_lse = oracle.decode_attention(np.ascontiguousarray(q[:, i]), k, v, lens, **kw)
        assert np.array_equal(out_f[:, i], full) and np.array_equal(lse_f[:, i], full_lse)
    assert np.array_equal(out_c[:, -1], out_f[:, -1])


def test_causal_query_tile_longer_than_its_context_is_rejected():
    x = np.zeros((1, 3, 1, 2))
    kv = np.zeros((1, 1, 2, 2))
    with pytest.raises(ValueError):
        oracle.attention(x, kv, kv, [2], N_q=3, Hq=1, Hkv=1, D=2, scale=1.0, causal=True, n_stride=2, dtype=oracle.F64)
    out, _ = oracle.attention(x, kv, kv, [2], N_q=3, Hq=1, Hkv=1, D=2, scale=1.0, causal=False, n_stride=2,
                              dtype=oracle.F64)
    assert out.shape == (1, 3, 1, 2)


# ---------------------------------------------------------------- per-sequence query lengths
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("layout", [oracle.KV_PADDED, oracle.KV_PACKED])
def test_ragged_query_lengths_against_masked_score_matrix(causal, layout):
    # a prefill chunk, decode steps, a sequence without queries and an empty context in one batch
    r = _rng(50 + int(causal))
    B, Hq, Hkv, D = 5, 4, 2, 6
    lens = [9, 5, 7, 0, 3]
    q_lens = [4, 1, 0, 2, 3]
    nmax, scale = max(lens), 0.45
    q = r.normal(size=(sum(q_lens), Hq, D))
    k = r.normal(size=(B, Hkv, nmax, D))
    v = r.normal(size=(B, Hkv, nmax, D))
    if layout == oracle.KV_PACKED:
        kk = np.ascontiguousarray(np.concatenate([k[b, :, :lens[b]] for b in range(B)], axis=1))
        vv = np.ascontiguousarray(np.concatenate([v[b, :, :lens[b]] for b in range(B)], axis=1))
    else:
        kk, vv = k, v
    out, lse = oracle.attention_ragged(q, kk, vv, lens, q_lens, Hq=Hq, Hkv=Hkv, D=D, scale=scale, causal=causal,
                                       kv_layout=layout, n_stride=nmax, dtype=oracle.F64)
    assert out.shape == (sum(q_lens), Hq, D)
    start, group = 0, Hq // Hkv
    for b in range(B):
        n, nq = lens[b], q_lens[b]
        rows = slice(start, start + nq)
        start += nq
        if n == 0:
            assert np.all(out[rows] == 0) and np.all(np.isneginf(lse[rows]))
            continue
        for hq in range(Hq):
            S = scale * q[rows, hq] @ k[b, hq // group, :n].T
            if causal:
                S = np.where(np.arange(n)[None, :] <= np.arange(nq)[:, None] + (n - nq), S, -np.inf)
            P = np.exp(S - S.max(axis=1, keepdims=True))
            np.testing.assert_allclose(out[rows, hq], (P / P.sum(axis=1, keepdims=True)) @ v[b, hq // group, :n],
                                       rtol=0, atol=1e-13)
            np.testing.assert_allclose(lse[rows, hq], S.max(axis=1) + np.log(P.sum(axis=1)), rtol=0, atol=1e-13)


def test_ragged_query_lengths_reduce_to_the_uniform_and_single_sequence_forms():
    r = _rng(52)
    B, Hq, Hkv, D = 3, 2, 2, 4
    lens, nmax = [6, 8, 5], 8
    k = r.normal(size=(B, Hkv, nmax, D))
    v = r.normal(size=(B, Hkv, nmax, D))
    kw = dict(Hq=Hq, Hkv=Hkv, D=D, scale=0.5, causal=True, n_stride=nmax, dtype=oracle.F64)
    # equal lengths: the [B, N_q, ...] form
    q = r.normal(size=(B, 3, Hq, D))
    a, al = oracle.attention_ragged(q.reshape(B * 3, Hq, D), k, v, lens, [3, 3, 3], **kw)
    u, ul = oracle.attention(q, k, v, lens, N_q=3, **kw)
    assert np.array_equal(a.reshape(u.shape), u) and np.array_equal(al.reshape(ul.shape), ul)
    # unequal lengths: every sequence on its own
    q_lens = [2, 5, 1]
    q = r.normal(size=(sum(q_lens), Hq, D))
    a, al = oracle.attention_ragged(q, k, v, lens, q_lens, **kw)
    start = 0
    for b in range(B):
        one, one_l = oracle.attention(q[start:start + q_lens[b]][None], k[b:b + 1], v[b:b + 1], [lens[b]],
                                      N_q=q_lens[b], **kw)
        assert np.array_equal(a[start:start + q_lens[b]], one[0]) and np.array_equal(al[start:start + q_lens[b]], one_l[0])
        start += q_lens[b]
    with pytest.raises(ValueError):   # causal: more query rows than cached tokens
        oracle.attention_ragged(r.normal(size=(13, Hq, D)), k, v, lens, [2, 5, 6], **kw)


def test_error_metrics_on_known_vectors():
    # hand-computed: got - want = (0, 0, 0.5, -2) -> max |.| = 2, ||diff|| = sqrt(4.25), ||want|| = sqrt(1+4+9+16)
    max_abs, rel_l2 = oracle.error_metrics([1.0, 2.0, 3.5, 2.0], [1.0, 2.0, 3.0, 4.0])
    assert max_abs == 2.0 and rel_l2 == pytest.approx(math.sqrt(4.25 / 30.0), rel=1e-15)
    # identical inputs: both zero; a zero reference reports the absolute norm instead of dividing by zero
    assert oracle.error_metrics([[3.0, -4.0]], [[3.0, -4.0]]) == (0.0, 0.0)
    assert oracle.error_metrics([3.0, -4.0], [0.0, 0.0]) == (4.0, 5.0)
    assert oracle.error_metrics([], []) == (0.0, 0.0)
