"""Host logic of the HIP library, run without a GPU: the stream-K scheduler and
span walk (the same code the kernel executes), argument checking, and the
exported symbols of the C ABI.  No compute entry point is called here."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import paper_2405_10480_amd as la
from oracle import stream_k

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _plan(seqlens, Hq, Hkv, D, dtype, layout, **kw):
    return la.lean_attn_schedule(seqlens, Hq, Hkv, D, dtype, layout, la.Tuning(**kw))


def test_library_exports_every_declared_symbol():
    import ctypes

    header = open(os.path.join(ROOT, "include", "lean_attn.h")).read()
    names = set(re.findall(r"\b(lean_attn_[a-z_]+)\s*\(", header))
    assert {"lean_attn_decode", "lean_attn_workspace_size", "lean_attn_schedule", "lean_attn_walk",
            "lean_attn_workspace_init", "lean_attn_workspace_status", "lean_attn_read_probe",
            "lean_attn_strerror", "lean_attn_attend", "lean_attn_problem_schedule",
            "lean_attn_problem_workspace_size"} <= names
    lib = ctypes.CDLL(la.library_path())
    for n in names:
        assert hasattr(lib, n), f"{n} declared in lean_attn.h but not exported"


def test_grid_is_units_times_residency_and_spans_are_equal():
    # the paper's own example: 108 units x 2 CTAs per unit = 216 (Section 4.3)
    p = _plan([65536] * 4, 32, 32, 64, la.F16, la.KV_PADDED, num_cus=108, ctas_per_cu=2)
    assert p.T_n == 128 and p.grid == 216 and p.T_m == 1 and p.kernel == 0
    assert p.total_iters == 4 * 32 * 512
    # the paper's own tile sizes (256 tokens at d = 64, 128 at d = 128) are compiled shapes too
    assert _plan([65536], 32, 32, 64, la.F16, la.KV_PADDED, num_cus=108, tile_shape=1).T_n == 256
    assert _plan([65536], 32, 32, 128, la.F16, la.KV_PADDED, num_cus=108, tile_shape=1).T_n == 128
    assert p.iters_per_cta == p.total_iters // 216 and p.extra == p.total_iters % 216
    # MI355X: 256 units
    p = _plan([65536], 32, 32, 128, la.BF16, la.KV_PADDED, num_cus=256, ctas_per_cu=2)
    assert (p.T_n, p.grid, p.total_iters, p.iters_per_cta, p.extra) == (64, 512, 32768, 64, 0)
    p = _plan([65536], 32, 32, 128, la.BF16, la.KV_PADDED, num_cus=256)
    assert p.grid == 256      # default: one workgroup per compute unit
    # never more CTAs than iterations
    p = _plan([60], 2, 2, 128, la.BF16, la.KV_PADDED, num_cus=256, ctas_per_cu=2)
    assert p.total_iters == 2 and p.grid == 2
    # a forced grid is honoured (it may exceed what is resident), up to the workspace limit
    p = _plan([65536], 32, 32, 128, la.BF16, la.KV_PADDED, num_cus=256, ctas_per_cu=2, grid=7)
    assert p.grid == 7 and p.extra == p.total_iters % 7
    p = _plan([65536], 32, 32, 128, la.BF16, la.KV_PADDED, num_cus=4, ctas_per_cu=2, grid=1000)
    assert p.grid == 1000 and p.max_resident == 8
    p = _plan([65536], 32, 32, 128, la.BF16, la.KV_PADDED, num_cus=4, ctas_per_cu=2, grid=100000)
    assert p.grid == 4096
    p = _plan([65536], 32, 32, 128, la.BF16, la.KV_PADDED, num_cus=256, ctas_per_cu=2, grid_multiple=4)
    assert p.grid == 2048
    # head dim 256: 1 KiB per wave-wide load is two rows, so the default LeanTile is 32 tokens
    # for single query rows; query groups take two 16-token blocks per wave: 128 tokens
    p = _plan([8192], 8, 8, 256, la.BF16, la.KV_PADDED, num_cus=256)
    assert (p.T_n, p.total_iters, p.grid) == (32, 8 * 256, 256)
    p = _plan([8192], 16, 2, 256, la.F16, la.KV_PADDED, num_cus=256)
    assert (p.T_n, p.T_m, p.kernel, p.total_iters) == (128, 8, 1, 2 * 64)
    # query groups use the MFMA kernel, one output tile per KV head
    p = _plan([262144], 64, 8, 128, la.BF16, la.KV_PADDED, num_cus=256, ctas_per_cu=2)
    assert p.kernel == 1 and p.T_m == 8 and p.num_output_tiles == 8
    assert p.total_iters == 8 * math.ceil(262144 / p.T_n)


@pytest.mark.parametrize("layout", [la.KV_PADDED, la.KV_PACKED])
@pytest.mark.parametrize("G", [1, 2, 5, 13, 64, 10_000])
def test_walk_matches_the_interval_arithmetic_of_the_decomposition(G, layout):
    # the span walk the kernel runs (lean_attn_walk is the same code) against the pieces obtained
    # by intersecting the span intervals with the tile intervals
    Hkv, D = 3, 128
    for seqlens in ([700, 1, 0, 257, 3000], [640] * 6, [64], [0, 0, 129]):
        p = _plan(seqlens, Hkv, Hkv, D, la.BF16, layout, num_cus=G, ctas_per_cu=1, grid=G)
        order = "padded" if layout == la.KV_PADDED else "packed"
        work = stream_k.pieces(seqlens, Hkv, p.T_n, G, order)
        stream_k.check_invariants(work, seqlens, Hkv, p.T_n)
        want = {}
        for t in work:
            want.setdefault(t["cta"], []).append(t)
        assert p.grid == len(stream_k.spans(p.total_iters, G))
        for g in range(p.grid):
            got = la.lean_attn_walk(p, seqlens, Hkv, layout, g)
            ref = want.get(g, [])
            assert len(got) == len(ref)
            for a, b in zip(got, ref):
                assert (a["b"], a["h"], a["local_iter"], a["local_iter_end"], bool(a["host"]), bool(a["finishing"]),
                        a["last_cta"]) == \
                       (b["b"], b["h"], b["local_iter"], b["local_iter_end"], b["host"], b["finishing"], b["last_cta"])


def test_walk_on_seeded_random_batches_and_grids():
    # many shapes: the multiply-shift divisions of the walk against plain integer interval arithmetic
    r = np.random.default_rng(2024)
    for trial in range(300):
        B = int(r.integers(1, 9))
        Hkv = int(r.integers(1, 12))
        uniform = trial % 3 == 0
        if uniform:
            seqlens = [int(r.integers(1, 40000))] * B
        else:
            seqlens = [int(x) for x in r.integers(0, 40000, size=B)]
        if sum(seqlens) == 0:
            seqlens[0] = 5
        layout = la.KV_PACKED if trial % 2 else la.KV_PADDED
        G = int(r.choice([1, 2, 3, 7, 8, 63, 64, 255, 256, 257, 512, 1000, 4096]))
        p = _plan(seqlens, Hkv, Hkv, 128, la.BF16, layout, num_cus=G, ctas_per_cu=1, grid=G)
        work = stream_k.pieces(seqlens, Hkv, p.T_n, G, "padded" if layout == la.KV_PADDED else "packed")
        want = {}
        for t in work:
            want.setdefault(t["cta"], []).append(t)
        probe = sorted(set([0, p.grid - 1, p.grid // 2] + [int(x) for x in r.integers(0, p.grid, size=6)]))
        for g in probe:
            got = la.lean_attn_walk(p, seqlens, Hkv, layout, g)
            ref = want.get(g, [])
            assert [(a["b"], a["h"], a["local_iter"], a["local_iter_end"], bool(a["host"]), bool(a["finishing"]),
                     a["last_cta"]) for a in got] == \
                   [(b["b"], b["h"], b["local_iter"], b["local_iter_end"], b["host"], b["finishing"], b["last_cta"])
                    for b in ref], (trial, seqlens, Hkv, layout, G, g)


def _check_invariants(seqlens, Hkv, layout, p):
    """Coverage, one host per tile, at most one published partial per CTA, exact peer ranges."""
    C = [math.ceil(n / p.T_n) for n in seqlens]
    heads = Hkv * max(1, p.C_m)          # output tiles per sequence: KV heads x row blocks
    covered = {}
    hosts = {}
    contributors = {}
    for g in range(p.grid):
        segs = la.lean_attn_walk(p, seqlens, Hkv, layout, g)
        assert segs, "every CTA owns at least one iteration"
        n_iters = sum(s["local_iter_end"] - s["local_iter"] for s in segs)
        assert n_iters == p.iters_per_cta + (1 if g < p.extra else 0)
        for i, s in enumerate(segs):
            key = (s["b"], s["h"])
            assert 0 <= s["local_iter"] < s["local_iter_end"] <= C[s["b"]]
            covered.setdefault(key, []).append((s["local_iter"], s["local_iter_end"]))
            contributors.setdefault(key, []).append(g)
            if s["host"]:
                assert s["local_iter"] == 0
                hosts[key] = (g, s)
            else:
                assert i == 0, "only a CTA's first segment can start mid-tile: one workspace slot per CTA"
            assert bool(s["finishing"]) == (s["local_iter_end"] == C[s["b"]])
            expect_idx = s["b"] * heads + s["h"] if layout == la.KV_PADDED else s["h"] * len(seqlens) + s["b"]
            assert s["tile_idx"] == expect_idx
    for b, n in enumerate(seqlens):
        for h in range(heads):
            if C[b] == 0:
                assert (b, h) not in covered
                continue
            pieces = sorted(covered[(b, h)])
            assert pieces[0][0] == 0 and pieces[-1][1] == C[b]
            assert all(x[1] == y[0] for x, y in zip(pieces, pieces[1:]))
            g, s = hosts[(b, h)]
            peers = sorted(contributors[(b, h)])
            assert peers[0] == g and peers == list(range(g, peers[-1] + 1))
            assert s["last_cta"] == peers[-1]
            assert bool(s["finishing"]) == (len(peers) == 1)


@pytest.mark.parametrize("layout", [la.KV_PADDED, la.KV_PACKED])
@pytest.mark.parametrize("G", [1, 3, 8, 61, 512])
def test_span_invariants_ragged(layout, G):
    seqlens = [1024, 131072, 5000, 0, 77, 128, 129, 40000]
    p = _plan(seqlens, 4, 4, 128, la.BF16, layout, num_cus=G, ctas_per_cu=1, grid=G)
    _check_invariants(seqlens, 4, layout, p)


def _problem(B, N_q, Hq, Hkv, D, dtype=la.BF16, layout=la.KV_PADDED, causal=0, out_dtype=la.OUT_F32, stride=0):
    return la.Problem(B=B, N_q=N_q, Hq=Hq, Hkv=Hkv, D=D, dtype=dtype, out_dtype=out_dtype, kv_layout=layout,
                      causal=causal, scale=1.0, kv_seq_stride=stride)


def test_query_rows_are_cut_into_row_blocks():
    # Algorithm 2: C_m output tiles along the query dimension; the query group is folded into the rows
    tn = la.Tuning(num_cus=256)
    cases = [  # D, N_q, Hq, Hkv -> R, C_m, T_m, kernel      (a tile holds up to 32 rows, 16 at D = 256)
        (128, 1, 8, 8, 1, 1, 1, 0), (128, 1, 64, 8, 8, 1, 8, 1), (128, 1, 64, 2, 32, 1, 32, 1),
        (128, 1, 34, 2, 17, 1, 17, 1), (64, 4, 8, 8, 4, 1, 4, 1), (64, 3, 16, 2, 24, 1, 24, 1),
        (128, 16, 32, 2, 256, 8, 32, 1), (128, 5, 28, 4, 35, 2, 18, 1),
        (256, 1, 64, 2, 32, 2, 16, 1), (256, 1, 34, 2, 17, 2, 9, 1), (256, 5, 28, 4, 35, 3, 12, 1),
        (256, 16, 32, 2, 256, 16, 16, 1),
    ]
    seqlens = [5000, 0, 777]
    for D, N_q, Hq, Hkv, R, C_m, T_m, kernel in cases:
        pr = _problem(3, N_q, Hq, Hkv, D)
        p = la.lean_attn_problem_schedule(pr, seqlens, tn)
        assert (p.C_m, p.T_m, p.kernel) == (C_m, T_m, kernel), (N_q, Hq, Hkv)
        assert p.num_output_tiles == 3 * Hkv * C_m
        assert p.total_iters == Hkv * C_m * sum(math.ceil(n / p.T_n) for n in seqlens)
        assert C_m * T_m >= R > (C_m - 1) * T_m
        ws = la.lean_attn_problem_workspace_size(pr)
        assert ws >= 256 + 4 * 4096 + 4096 * T_m * (D + 2) * 4 and ws % 256 == 0
    # the plain decode entry points are the N_q = 1 problem
    p1 = _plan(seqlens, 64, 2, 128, la.BF16, la.KV_PADDED, num_cus=256)
    p2 = la.lean_attn_problem_schedule(_problem(3, 1, 64, 2, 128), seqlens, tn)
    assert bytes(p1) == bytes(p2)
    assert la.lean_attn_workspace_size(3, 64, 2, 128, la.BF16) == la.lean_attn_problem_workspace_size(_problem(3, 1, 64, 2, 128))


@pytest.mark.parametrize("layout", [la.KV_PADDED, la.KV_PACKED])
@pytest.mark.parametrize("G", [1, 7, 64, 300])
def test_span_invariants_with_row_blocks(layout, G):
    seqlens = [1024, 20000, 0, 77, 129]
    pr = _problem(len(seqlens), 5, 28, 4, 256, layout=layout, causal=1)      # 35 rows per KV head: 3 blocks
    p = la.lean_attn_problem_schedule(pr, seqlens, la.Tuning(num_cus=G, ctas_per_cu=1, grid=G))
    assert p.C_m == 3
    _check_invariants(seqlens, 4, layout, p)


def test_workspace_size_grows_with_the_grid_and_with_the_tile_rows():
    pr = _problem(1, 1, 64, 8, 128)                      # 8 rows per tile
    full = la.lean_attn_problem_workspace_size(pr)
    assert la.lean_attn_workspace_size_for_grid(pr, la.binding.MAX_GRID) == full
    assert la.lean_attn_workspace_size(1, 64, 8, 128, la.BF16) == full
    flags = 256 + 4 * 16 * la.binding.MAX_GRID           # status, then 2 slots x 8 reader words per workgroup
    slot = -(-8 * (128 + 2) * 4 // 256) * 256            # (O~[8,128], m[8], l[8]) in fp32, rounded up to 256 bytes
    for g in (1, 256, 512, 4096):
        assert la.lean_attn_workspace_size_for_grid(pr, g) == flags + 2 * g * slot
    assert la.lean_attn_workspace_size_for_grid(pr, 0) == 0
    assert la.lean_attn_workspace_size_for_grid(pr, la.binding.MAX_GRID + 1) == 0
    # 33 rows per KV head make two blocks of 17; beyond one launch with per-sequence query lengths a
    # chunk may run one block of 32, so that case is sized for the largest tile
    p33 = _problem(2, 3, 11, 1, 64)
    p32 = _problem(2, 2, 16, 1, 64)
    assert la.lean_attn_problem_workspace_size(p33) < la.lean_attn_problem_workspace_size(p32)
    big = _problem(300, 3, 11, 1, 64).set_q_lens([3] * 300)
    assert la.lean_attn_problem_workspace_size(big) == la.lean_attn_problem_workspace_size(p32)


def test_problem_argument_errors():
    tn = la.Tuning(num_cus=4)
    def status(pr, seqlens):
        with pytest.raises(la.LeanAttnError) as e:
            la.lean_attn_problem_schedule(pr, seqlens, tn)
        return e.value.status
    assert status(_problem(1, 0, 2, 2, 128), [10]) == -2
    assert status(_problem(1, 17, 32, 2, 128), [100]) == -2            # 272 query rows per KV head
    assert status(_problem(1, 4, 2, 2, 128, causal=1), [3]) == -5      # fewer cached tokens than query rows
    assert status(_problem(1, 4, 2, 2, 128, causal=2), [30]) == -2
    assert status(_problem(1, 4, 2, 2, 128, out_dtype=7), [30]) == -3
    la.lean_attn_problem_schedule(_problem(2, 4, 2, 2, 128, causal=1), [4, 0], tn)   # exactly N_q tokens, and empty
    la.lean_attn_problem_schedule(_problem(1, 4, 2, 2, 128, causal=0), [3], tn)      # no mask: any length
    with pytest.raises(la.LeanAttnError) as e:                                       # VALU kernel: one row per KV head
        la.lean_attn_problem_schedule(_problem(1, 2, 2, 2, 128), [30], la.Tuning(num_cus=4, kernel=1))
    assert e.value.status == -8
    assert la.lean_attn_problem_workspace_size(_problem(1, 1, 2, 2, 96)) == 0


def test_span_invariants_on_benchmark_shapes():
    import workloads

    for idx in (4, 5):
        w = workloads.named(idx)
        dt = la.BF16
        p = _plan(list(w.seqlens), w.Hq, w.Hkv, w.D, dt, w.kv_layout, num_cus=256, ctas_per_cu=2)
        assert p.grid == 512
        assert p.total_iters == w.Hkv * sum(math.ceil(n / p.T_n) for n in w.seqlens)
        _check_invariants(list(w.seqlens), w.Hkv, w.kv_layout, p)


def test_special_cases_of_section_4_3():
    T_n = _plan([1], 3, 3, 128, la.BF16, la.KV_PADDED, num_cus=1).T_n
    # grid == number of output tiles: every CTA is host and finishing (FlashAttention-2 schedule)
    seqlens = [10 * T_n, 10 * T_n]
    p = _plan(seqlens, 3, 3, 128, la.BF16, la.KV_PADDED, num_cus=6, ctas_per_cu=1)
    assert p.grid == 6 and p.total_iters == 60
    for g in range(6):
        (s,) = la.lean_attn_walk(p, seqlens, 3, la.KV_PADDED, g)
        assert s["host"] and s["finishing"]
    # grid an even multiple of the tile count: equal fixed splits (FlashDecoding schedule)
    p = _plan(seqlens, 3, 3, 128, la.BF16, la.KV_PADDED, num_cus=12, ctas_per_cu=1)
    for g in range(12):
        (s,) = la.lean_attn_walk(p, seqlens, 3, la.KV_PADDED, g)
        assert s["local_iter_end"] - s["local_iter"] == 5 and bool(s["host"]) == (g % 2 == 0)


@pytest.mark.parametrize("layout", [la.KV_PADDED, la.KV_PACKED])
@pytest.mark.parametrize("split", [1, 2, 3, 16])
def test_fixed_split_baseline_schedule(layout, split):
    # Sections 3.3 / 4.3: every output tile cut into `split` near-equal parts (1 = no split)
    seqlens = [1000, 5, 0, 70000, 129]
    Hkv = 3
    p = _plan(seqlens, Hkv, Hkv, 128, la.BF16, layout, num_cus=4, ctas_per_cu=2, fixed_split=split)
    assert p.fixed_split == split and p.grid == len(seqlens) * Hkv * split
    C = [math.ceil(n / p.T_n) for n in seqlens]
    for tile in range(len(seqlens) * Hkv):
        b, h = (tile // Hkv, tile % Hkv) if layout == la.KV_PADDED else (tile % len(seqlens), tile // len(seqlens))
        pieces = []
        for part in range(split):
            segs = la.lean_attn_walk(p, seqlens, Hkv, layout, tile * split + part)
            assert len(segs) <= 1
            if part >= min(split, C[b]):
                assert segs == []
                continue
            (s,) = segs
            assert (s["b"], s["h"], s["tile_idx"]) == (b, h, tile)
            assert s["last_cta"] == tile * split + min(split, C[b]) - 1
            assert bool(s["host"]) == (part == 0) and bool(s["finishing"]) == (part == min(split, C[b]) - 1)
            pieces.append((s["local_iter"], s["local_iter_end"]))
        if C[b]:
            assert pieces[0][0] == 0 and pieces[-1][1] == C[b]
            assert all(x[1] == y[0] for x, y in zip(pieces, pieces[1:]))
            sizes = [y - x for x, y in pieces]
            assert max(sizes) - min(sizes) <= 1
    # the default factor fills one wave of workgroups and stops splitting beyond it
    assert _plan([65536], 32, 32, 128, la.BF16, layout, num_cus=256, ctas_per_cu=2, fixed_split=-1).fixed_split == 16
    assert _plan([4096] * 32, 32, 32, 128, la.BF16, layout, num_cus=256, ctas_per_cu=2, fixed_split=-1).fixed_split == 1


def test_argument_errors():
    with pytest.raises(la.LeanAttnError) as e:
        _plan([10], 3, 2, 128, la.BF16, la.KV_PADDED, num_cus=4)
    assert e.value.status == -2
    with pytest.raises(la.LeanAttnError) as e:
        _plan([10], 2, 2, 96, la.BF16, la.KV_PADDED, num_cus=4)
    assert e.value.status == -3
    with pytest.raises(la.LeanAttnError) as e:
        _plan([10, -1], 2, 2, 128, la.BF16, la.KV_PADDED, num_cus=4)
    assert e.value.status == -5
    with pytest.raises(la.LeanAttnError) as e:
        _plan([1] * 257, 2, 2, 128, la.BF16, la.KV_PADDED, num_cus=4)
    assert e.value.status == -6
    with pytest.raises(la.LeanAttnError) as e:
        _plan([10], 514, 2, 128, la.BF16, la.KV_PADDED, num_cus=4)      # 257 query rows per KV head
    assert e.value.status == -2
    with pytest.raises(la.LeanAttnError) as e:
        _plan([10], 4, 2, 128, la.BF16, la.KV_PADDED, num_cus=4, kernel=1)  # VALU kernel needs Hq == Hkv
    assert e.value.status == -8
    assert la.lean_attn_workspace_size(1, 2, 2, 96, la.BF16) == 0
    sz = la.lean_attn_workspace_size(1, 64, 8, 128, la.BF16)
    assert sz >= 256 + 4 * 4096 + 4096 * 8 * 130 * 4 and sz % 256 == 0
    for code in range(-9, 1):
        assert la.lean_attn_strerror(code) not in ("", "unknown status")


@pytest.mark.parametrize("layout", [la.KV_PADDED, la.KV_PACKED])
def test_span_invariants_beyond_two_to_the_31_iterations(layout):
    # the span walk divides in 32 bits below 2^31 iterations and in 64 bits above: cover the latter
    seqlens = [8388607 - 64 * i for i in range(200)]
    p = _plan(seqlens, 128, 128, 128, la.BF16, layout, num_cus=16, ctas_per_cu=1, grid=16)
    assert p.total_iters > 2 ** 31
    _check_invariants(seqlens, 128, layout, p)


@pytest.mark.parametrize("layout", [la.KV_PADDED, la.KV_PACKED])
@pytest.mark.parametrize("uniform", [False, True])
def test_span_invariants_just_below_two_to_the_31_iterations(layout, uniform):
    # the largest iteration spaces the multiply-shift divisions of the walk serve
    seqlens = [8388607 - (0 if uniform else 64 * (i % 3)) for i in range(256)]
    for G in (16, 13):
        p = _plan(seqlens, 63, 63, 128, la.BF16, layout, num_cus=G, ctas_per_cu=1, grid=G)
        assert 2 ** 31 - 2 ** 26 < p.total_iters < 2 ** 31 - 1
        _check_invariants(seqlens, 63, layout, p)


def test_per_sequence_query_lengths_are_validated():
    tn = la.Tuning(num_cus=4)
    def status(pr, seqlens):
        with pytest.raises(la.LeanAttnError) as e:
            la.lean_attn_problem_schedule(pr, seqlens, tn)
        return e.value.status
    ok = _problem(3, 4, 8, 2, 128, causal=1).set_q_lens([4, 1, 0])
    p = la.lean_attn_problem_schedule(ok, [100, 1, 50], tn)
    # the schedule is that of the longest query for every sequence; a single query row still takes the MFMA kernel
    assert (p.T_m, p.C_m, p.kernel) == (16, 1, 1)
    assert bytes(p) == bytes(la.lean_attn_problem_schedule(_problem(3, 4, 8, 2, 128, causal=1), [100, 4, 50], tn))
    assert la.lean_attn_problem_schedule(_problem(2, 1, 2, 2, 128).set_q_lens([1, 0]), [10, 10], tn).kernel == 1
    assert status(_problem(3, 4, 8, 2, 128).set_q_lens([3, 1, 0]), [100, 1, 50]) == -2      # N_q is not the longest
    assert status(_problem(3, 4, 8, 2, 128).set_q_lens([4, 5, 0]), [100, 9, 50]) == -2      # longer than N_q
    assert status(_problem(3, 4, 8, 2, 128).set_q_lens([4, -1, 0]), [100, 9, 50]) == -2
    assert status(_problem(3, 4, 8, 2, 128, causal=1).set_q_lens([4, 2, 0]), [100, 1, 50]) == -5   # 1 cached token, 2 queries
    la.lean_attn_problem_schedule(_problem(3, 4, 8, 2, 128, causal=0).set_q_lens([4, 2, 0]), [100, 1, 50], tn)
    assert ok.query_tokens() == 5 and _problem(3, 4, 8, 2, 128).query_tokens() == 12


def test_many_short_contexts_put_two_workgroups_on_a_unit():
    # large batches of short contexts: every span crosses several tile boundaries
    assert _plan([1000] * 256, 32, 8, 128, la.BF16, la.KV_PADDED, num_cus=256).grid == 512
    assert _plan([1500] * 64 + [0] * 8, 32, 8, 128, la.BF16, la.KV_PACKED, num_cus=256).grid == 512
    # long contexts, or too few tiles to cross boundaries: one workgroup per unit
    assert _plan([4000] * 256, 32, 8, 128, la.BF16, la.KV_PADDED, num_cus=256).grid == 256
    assert _plan([1000] * 32, 32, 8, 128, la.BF16, la.KV_PADDED, num_cus=256).grid == 256
    # an explicit request wins
    assert _plan([1000] * 256, 32, 8, 128, la.BF16, la.KV_PADDED, num_cus=256, ctas_per_cu=1).grid == 256


def test_header_compiles_as_plain_c_and_matches_the_binding_structs(tmp_path):
    # the boundary is a C ABI: the header must be valid C99, and the ctypes mirrors must have its layout
    import ctypes
    import subprocess

    src = tmp_path / "abi.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "lean_attn.h"\n'
        "int main(void) {\n"
        '  printf("%zu %zu %zu ", sizeof(lean_attn_plan), sizeof(lean_attn_tuning), sizeof(lean_attn_problem));\n'
        '  printf("%zu %zu %zu %zu\\n", offsetof(lean_attn_plan, total_iters), offsetof(lean_attn_tuning, cta_clock),\n'
        "         offsetof(lean_attn_problem, kv_seq_stride), offsetof(lean_attn_problem, q_lens));\n"
        "  return 0;\n}\n")
    exe = tmp_path / "abi"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                           "-o", str(exe), str(src)])
    got = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    want = [ctypes.sizeof(la.Plan), ctypes.sizeof(la.Tuning), ctypes.sizeof(la.Problem), la.Plan.total_iters.offset,
            la.Tuning.cta_clock.offset, la.Problem.kv_seq_stride.offset, la.Problem.q_lens.offset]
    assert got == want


def test_prepare_writes_a_launch_block_whose_grid_does_not_depend_on_the_lengths():
    # host-only: no pointer is dereferenced, so made-up (aligned, non-null) addresses do
    import struct

    import torch

    lib = ctypes.CDLL(la.library_path())
    lib.lean_attn_launch_block_size.restype = ctypes.c_size_t
    size = lib.lean_attn_launch_block_size()
    assert size == la.lean_attn_launch_block_size() and size % 16 == 0 and size < 4096
    pr = _problem(3, 1, 16, 2, 128, stride=200000)
    ws_bytes = la.lean_attn_problem_workspace_size(pr)

    class Fake:  # stands in for a device tensor: only data_ptr/numel/element_size are used
        def __init__(self, addr, n=0):
            self.addr, self.n = addr, n
        def data_ptr(self):
            return self.addr
        def numel(self):
            return self.n
        def element_size(self):
            return 1

    q, k, v, out, ws = Fake(0x10000), Fake(0x20000), Fake(0x30000), Fake(0x40000), Fake(0x100000, ws_bytes)
    block = torch.zeros(size, dtype=torch.uint8)
    tn = la.Tuning(num_cus=256)
    grids = []
    for seqlens in ([5000, 0, 777], [1, 1, 1], [0, 0, 0], [200000, 3, 64]):
        la.lean_attn_attend_prepare(pr, q, k, v, seqlens, out, ws, block, tuning=tn)
        magic, fn, grid, threads = struct.unpack_from("<QQII", block.numpy().tobytes(), 0)
        assert magic == int.from_bytes(b"LEANBLK1", "little") and fn != 0 and threads == 256
        grids.append(grid)
    assert grids == [256] * 4          # one workgroup per unit, even with 3 iterations or none at all
    before = block.clone()
    for bad_kwargs, seqlens, status in ((dict(tile_shape=1), [10, 10, 10], -8), (dict(fixed_split=2), [10, 10, 10], -8),
                                        (dict(), [10, -1, 10], -5)):
        with pytest.raises(la.LeanAttnError) as e:
            la.lean_attn_attend_prepare(pr, q, k, v, seqlens, out, ws, block, tuning=la.Tuning(num_cus=256, **bad_kwargs))
        assert e.value.status == status
        assert torch.equal(block, before), "a refused call must leave the block as it was"
    with pytest.raises(la.LeanAttnError) as e:
        la.lean_attn_attend_prepare(_problem(300, 1, 16, 2, 128, stride=8), q, k, v, [5] * 300, out, ws, block, tuning=tn)
    assert e.value.status == -6


def test_default_tile_shapes_are_the_ones_the_committed_sweep_supports():
    # The (head dim, dtype, rows per tile) -> shape table of the library against the committed summary of
    # `bench.py --tile-sweep`: the table's pick is the sweep's default column, and it is within 3 % of the
    # fastest variant of its case (any shape, one or two workgroups per unit).
    path = os.path.join(ROOT, "profiles", "tile_sweep_1GiB_per_call.md")
    rows = [[c.strip() for c in line.strip().strip("|").split("|")] for line in open(path)
            if re.match(r"^\|\s*\d+\s*\|", line)]
    assert len(rows) == 22        # 3 head dims x 2 dtypes x {1, 8, 16, 32} rows, no 32-row tiles at D = 256
    classes = set()
    for D, dtype, n_rows, shape, default_us, _best, best_us, _ratio in rows:
        D, n_rows, shape = int(D), int(n_rows), int(shape)
        code = la.F16 if dtype == "f16" else la.BF16
        ctx = (1 << 30) // (8 * D * 2 * 2)
        p = _plan([ctx], 8 * n_rows, 8, D, code, la.KV_PADDED, num_cus=256)
        assert p.tile_shape == shape, f"D={D} {dtype} rows={n_rows}: library picks {p.tile_shape}, sweep file says {shape}"
        assert p.T_m == n_rows and p.kernel == (0 if n_rows == 1 else 1)
        assert float(default_us) <= 1.03 * float(best_us), f"D={D} {dtype} rows={n_rows}: default is not near the best"
        classes.add((D, dtype, 0 if n_rows == 1 else 1 if n_rows <= 8 else 2 if n_rows <= 16 else 3))
    assert len(classes) == 22     # every cell of the table is covered once
    # the class boundaries: 2..8, 9..16 and 17..32 rows share a default each
    for D, lo, hi in ((64, 9, 16), (128, 17, 32), (64, 2, 8)):
        picks = {_plan([4096], 4 * r, 4, D, la.BF16, la.KV_PADDED, num_cus=256).tile_shape for r in range(lo, hi + 1)}
        assert len(picks) == 1


def test_binding_constants_match_the_header():
    header = open(os.path.join(ROOT, "include", "lean_attn.h")).read()

    def define(name):
        return int(re.search(rf"#define {name}\s+(-?\d+)", header).group(1))

    assert define("LEAN_ATTN_NUM_TILE_SHAPES") == la.NUM_TILE_SHAPES
    assert define("LEAN_ATTN_STATIC_MAX_GRID") == la.binding.STATIC_MAX_GRID
    # a shape number past the last one is a tuning error, a shape that is not built for the core is "unsupported"
    with pytest.raises(la.LeanAttnError) as e:
        _plan([4096], 8, 8, 128, la.BF16, la.KV_PADDED, num_cus=256, tile_shape=la.NUM_TILE_SHAPES + 1)
    assert e.value.status == la.binding.ERR_TUNING
    with pytest.raises(la.LeanAttnError) as e:
        _plan([4096], 8, 8, 128, la.BF16, la.KV_PADDED, num_cus=256, tile_shape=7)   # single-row core: shapes 1..6
    assert e.value.status == la.binding.ERR_UNSUPPORTED
    assert _plan([4096], 64, 8, 128, la.BF16, la.KV_PADDED, num_cus=256, tile_shape=7).T_n == 128
    assert _plan([4096], 64, 8, 256, la.BF16, la.KV_PADDED, num_cus=256, tile_shape=8).T_n == 32


def test_tail_spans_walk_matches_the_interval_arithmetic():
    # short spans at the end of the line for a second class of workgroups: the plan's arithmetic and the walk
    # against the oracle's cut points, on seeded batches, grids, tail sizes and shares
    r = np.random.default_rng(77)
    seen_tail = 0
    for trial in range(200):
        B = int(r.integers(1, 7))
        Hkv = int(r.integers(1, 9))
        seqlens = [int(r.integers(1, 30000))] * B if trial % 3 == 0 else [int(x) for x in r.integers(0, 30000, size=B)]
        if sum(seqlens) == 0:
            seqlens[0] = 777
        layout = la.KV_PACKED if trial % 2 else la.KV_PADDED
        G = int(r.choice([1, 2, 7, 64, 255, 256, 512]))
        P = int(r.choice([1, 3, 16, 64, 256, 1000]))
        permille = int(r.choice([0, 1, 30, 60, 250, 500]))
        p = _plan(seqlens, Hkv, Hkv, 128, la.BF16, layout, num_cus=G, ctas_per_cu=1, grid=G, tail_grid=P,
                  tail_permille=permille)
        head_grid = p.grid - p.tail_grid
        if p.tail_grid == 0:                      # too small a problem: plain stream-K spans
            assert p.tail_iters == 0 and p.grid == min(G, p.total_iters)
            assert p.total_iters - max(P, p.total_iters * (permille or 60) // 1000) < min(G, p.total_iters)
            continue
        seen_tail += 1
        assert p.tail_grid == P and head_grid == min(G, p.total_iters)
        assert p.tail_iters == max(P, p.total_iters * (permille or 60) // 1000)
        head_iters = p.total_iters - p.tail_iters
        assert (p.iters_per_cta, p.extra) == (head_iters // head_grid, head_iters % head_grid) and p.iters_per_cta >= 1
        tail = (p.tail_grid, p.tail_iters)
        edges = stream_k.span_edges(p.total_iters, head_grid, tail)
        assert len(edges) == p.grid + 1 and edges[-1] == p.total_iters and np.all(np.diff(edges) >= 1)
        work = stream_k.pieces(seqlens, Hkv, p.T_n, head_grid, "padded" if layout == la.KV_PADDED else "packed", tail)
        stream_k.check_invariants(work, seqlens, Hkv, p.T_n)
        want = {}
        for t in work:
            want.setdefault(t["cta"], []).append(t)
        probe = sorted(set([0, head_grid - 1, head_grid, p.grid - 1] + [int(x) for x in r.integers(0, p.grid, size=8)]))
        for g in probe:
            got = la.lean_attn_walk(p, seqlens, Hkv, layout, g)
            ref = want.get(g, [])
            assert len(got) == len(ref), (trial, g)
            for a, b in zip(got, ref):
                assert (a["b"], a["h"], a["local_iter"], a["local_iter_end"], bool(a["host"]), bool(a["finishing"]),
                        a["last_cta"]) == \
                       (b["b"], b["h"], b["local_iter"], b["local_iter_end"], b["host"], b["finishing"], b["last_cta"]), \
                    (trial, g)
    assert seen_tail > 100
    # limits: a tail with the baseline schedules is ignored, too many workgroups or too large a share are errors
    assert _plan([5000] * 4, 8, 8, 128, la.BF16, la.KV_PADDED, num_cus=8, fixed_split=2, tail_grid=16).tail_grid == 0
    for bad in (dict(grid=4000, tail_grid=200), dict(tail_grid=-1), dict(tail_grid=8, tail_permille=501)):
        with pytest.raises(la.LeanAttnError) as e:
            _plan([50000] * 4, 8, 8, 128, la.BF16, la.KV_PADDED, num_cus=256, **bad)
        assert e.value.status == la.binding.ERR_TUNING
