"""Parity of the HIP decode path against the fp64 CPU oracle, through the C ABI.

Bar (stated by the task for 16-bit inputs with fp32 accumulation): max-abs
error <= 2e-3 and relative L2 error <= 1e-3 over the whole output tensor.
The path accumulates in fp32 and splits P into two 16-bit parts, so the
observed error is orders of magnitude below the bar; a second, tighter
check (1e-4 / 1e-4) guards against a silently dropped low-order term.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import paper_2405_10480_amd as la
import workloads

pytestmark = pytest.mark.gpu

MAX_ABS, REL_L2 = 2e-3, 1e-3
TIGHT_ABS, TIGHT_REL = 1e-4, 1e-4


def _workspace(B, Hq, Hkv, D, dtype_code):
    nbytes = la.lean_attn_workspace_size(B, Hq, Hkv, D, dtype_code)
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    la.lean_attn_workspace_init(ws)
    return ws


def _run(inp, tuning=None, ws=None, want_lse=True):
    w = inp.w
    code = la.F16 if w.dtype == "f16" else la.BF16
    if ws is None:
        ws = _workspace(w.B, w.Hq, w.Hkv, w.D, code)
    out = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((w.B, w.Hq), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    la.lean_attn_decode(inp.q, inp.k, inp.v, inp.seqlens, out, ws, Hkv=w.Hkv, kv_layout=w.kv_layout,
                        kv_seq_stride=w.n_stride, scale=w.scale, lse=lse, tuning=tuning)
    torch.cuda.synchronize()
    assert la.lean_attn_workspace_status(ws) == 0
    return out.cpu().numpy(), (lse.cpu().numpy() if want_lse else None), ws


def _oracle(inp):
    w = inp.w
    return oracle.decode_attention(inp.q, inp.k, inp.v, inp.seqlens, Hq=w.Hq, Hkv=w.Hkv, D=w.D, scale=w.scale,
                                   kv_layout=w.kv_layout, n_stride=w.n_stride)


def _check(got, got_lse, want, want_lse, label=""):
    assert np.all(np.isfinite(got)), f"{label}: non-finite output"
    max_abs, rel_l2 = oracle.error_metrics(got, want)
    assert max_abs <= MAX_ABS and rel_l2 <= REL_L2, f"{label}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}"
    assert max_abs <= TIGHT_ABS and rel_l2 <= TIGHT_REL, f"{label}: (tight) max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}"
    # the worst single output row, against the same bars (an error confined to one head must not hide)
    g2, w2 = np.asarray(got, dtype=np.float64).reshape(-1, got.shape[-1]), want.reshape(-1, want.shape[-1])
    row_err = np.sqrt(((g2 - w2) ** 2).sum(axis=1))
    row_norm = np.sqrt((w2 ** 2).sum(axis=1))
    live = row_norm > 0
    worst = float(np.max(row_err[live] / row_norm[live], initial=0.0))
    assert worst <= 10 * TIGHT_REL, f"{label}: worst row rel_l2={worst:.3e}"
    assert np.all(row_err[~live] == 0), f"{label}: a row that must be zero is not"
    if got_lse is not None:
        fin = np.isfinite(want_lse)
        assert np.array_equal(np.isneginf(got_lse), np.isneginf(want_lse)), f"{label}: lse -inf pattern"
        assert np.max(np.abs(got_lse[fin] - want_lse[fin]), initial=0.0) <= 1e-4, f"{label}: lse"
    return max_abs, rel_l2


N_SHAPES = 9


def _built(rows, D, shape):
    """Which tile shapes exist: 1..6 everywhere but the double-buffered MFMA shapes at D = 256;
    7..9 (K/V staged in LDS) for the MFMA cores at D = 128, 7 and 8 at D = 256."""
    if shape <= 6:
        return not (rows > 1 and D == 256 and shape in (1, 3))
    return rows > 1 and (D == 128 or (D == 256 and shape in (7, 8)))


def _mk(B, Hq, Hkv, D, dtype, seqlens, layout, seed, outlier=0.0):
    w = workloads.Workload(f"t_b{B}_h{Hq}_{Hkv}_d{D}_{dtype}", B, Hq, Hkv, D, dtype, tuple(seqlens), layout,
                           seed=seed, outlier_frac=outlier)
    return workloads.generate(w, device="cuda")


def test_longest_context_a_slab_can_hold():
    # One K/V slab is addressed through a buffer descriptor with 32-bit byte offsets: N_b * D * 2
    # bytes must stay below 2^31.  The longest context at D = 64, one KV head (2 GiB of K, 2 GiB
    # of V), through the single-row kernel and, with four query heads, the MFMA kernel.
    D = 64
    n_max = (2**31 - 1) // (D * 2)
    for Hq in (1, 4):
        inp = _mk(1, Hq, 1, D, "f16", [n_max], workloads.KV_PADDED, seed=90 + Hq, outlier=0.001)
        want, want_lse = _oracle(inp)
        got, got_lse, _ = _run(inp)
        _check(got, got_lse, want, want_lse, f"N={n_max} Hq={Hq}")
        del inp
        torch.cuda.empty_cache()
    with pytest.raises(la.LeanAttnError) as e:
        la.lean_attn_schedule([n_max + 1], 1, 1, D, la.F16, la.KV_PADDED)
    assert e.value.status == la.binding.ERR_SEQLEN


# ------------------------------------------------------------------ small shapes, all variants
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("D", [64, 128, 256])
@pytest.mark.parametrize("group", [1, 2, 7, 8, 16])
def test_small_shapes_every_kernel_variant(dtype, D, group):
    Hkv = 3
    # several LeanTiles, a ragged tail, a single token, an empty sequence, exact tile multiples
    seqlens = [1000, 1, 0, 256, 257, 777]
    for layout in (workloads.KV_PADDED, workloads.KV_PACKED):
        inp = _mk(len(seqlens), Hkv * group, Hkv, D, dtype, seqlens, layout, seed=11 + group)
        want, want_lse = _oracle(inp)
        got, got_lse, _ = _run(inp)
        _check(got, got_lse, want, want_lse, f"{dtype} D{D} g{group} layout{layout}")
        assert np.all(got[2] == 0.0) and np.all(np.isneginf(got_lse[2]))


@pytest.mark.parametrize("group", [1, 8])
@pytest.mark.parametrize("G", [1, 2, 3, 7, 31, 64, 0])
def test_result_does_not_depend_on_the_split(group, G):
    # Section 4.1: any split of the context gives the same attention output
    Hkv, D = 2, 128
    seqlens = [3000, 129, 4097]
    inp = _mk(3, Hkv * group, Hkv, D, "bf16", seqlens, workloads.KV_PADDED, seed=5, outlier=0.02)
    want, want_lse = _oracle(inp)
    plan = la.lean_attn_schedule(seqlens, Hkv * group, Hkv, D, la.BF16, la.KV_PADDED)
    grids = [G] if G else [int(plan.total_iters), int(plan.total_iters) - 1]
    for grid in grids:
        got, got_lse, _ = _run(inp, la.Tuning(grid=grid))
        _check(got, got_lse, want, want_lse, f"G={grid}")


def test_mfma_kernel_on_single_row_groups_matches_valu_kernel_and_oracle():
    inp = _mk(2, 4, 4, 128, "bf16", [2000, 513], workloads.KV_PACKED, seed=8)
    want, want_lse = _oracle(inp)
    for kernel in (1, 2):
        got, got_lse, _ = _run(inp, la.Tuning(kernel=kernel))
        _check(got, got_lse, want, want_lse, f"kernel={kernel}")


def test_bitwise_reproducible_and_workspace_reusable():
    inp = _mk(2, 16, 2, 128, "bf16", [5000, 1234], workloads.KV_PADDED, seed=9)
    first, _, ws = _run(inp)
    # poison the partial slots: a read before the peer's signal would surface as NaN
    ws[256 + 4 * la.binding.MAX_GRID:].view(torch.float32).fill_(float("nan"))
    for _ in range(5):
        again, _, _ = _run(inp, ws=ws)
        assert np.array_equal(first, again)


def test_dominant_key_and_equal_scores_closed_forms():
    # one dominant score selects its V row; all-equal scores give the mean of V
    B, H, D, N = 1, 2, 128, 1500
    w = workloads.Workload("closed", B, H, H, D, "bf16", (N,), workloads.KV_PADDED, seed=3)
    inp = workloads.generate(w, device="cuda")
    inp.k.zero_()
    got, got_lse, _ = _run(inp)
    mean_v = inp.v[0, :, :N].float().mean(dim=1).cpu().numpy()
    assert np.max(np.abs(got[0] - mean_v)) < 1e-5
    assert np.max(np.abs(got_lse[0] - math.log(N))) < 1e-5
    tstar = 1033
    inp.k[0, :, tstar] = (inp.q[0].float() * 8.0).to(inp.k.dtype)
    got, _, _ = _run(inp)
    sel = inp.v[0, :, tstar].float().cpu().numpy()
    qn = (inp.q[0].float() ** 2).sum(-1).cpu().numpy() * 8.0 * w.scale      # the dominant score
    assert np.all(qn > 40)
    assert np.max(np.abs(got[0] - sel)) < 1e-5


def test_error_paths_launch_nothing():
    inp = _mk(1, 2, 2, 128, "bf16", [100], workloads.KV_PADDED, seed=1)
    ws = _workspace(1, 2, 2, 128, la.BF16)
    out = torch.zeros(1, 2, 128, device="cuda")
    with pytest.raises(la.LeanAttnError) as e:
        la.lean_attn_decode(inp.q, inp.k, inp.v, [100], out, ws[:1024], Hkv=2, kv_seq_stride=100, scale=1.0)
    assert e.value.status == la.binding.ERR_WORKSPACE
    with pytest.raises(la.LeanAttnError) as e:
        la.lean_attn_decode(inp.q, inp.k, inp.v, [-3], out, ws, Hkv=2, kv_seq_stride=100, scale=1.0)
    assert e.value.status == la.binding.ERR_SEQLEN
    with pytest.raises(la.LeanAttnError) as e:   # padded stride shorter than the sequence
        la.lean_attn_decode(inp.q, inp.k[:, :, :50].contiguous(), inp.v[:, :, :50].contiguous(), [100], out, ws,
                            Hkv=2, kv_seq_stride=50, scale=1.0)
    assert e.value.status == la.binding.ERR_SEQLEN
    torch.cuda.synchronize()
    assert torch.all(out == 0)


def test_workspace_sized_for_the_launch_grid_and_checked_per_launch():
    # the flags plus two partial slots per workgroup of the launch are all a call needs; one workgroup less is
    # an error and nothing is launched
    inp = _mk(1, 16, 2, 128, "bf16", [40000], workloads.KV_PADDED, seed=5)
    w = inp.w
    want, want_lse = _oracle(inp)
    pr = la.Problem(B=1, N_q=1, Hq=16, Hkv=2, D=128, dtype=la.BF16, out_dtype=la.OUT_F32, kv_layout=la.KV_PADDED,
                    causal=0, scale=w.scale, kv_seq_stride=w.n_stride)
    for tn in (None, la.Tuning(grid=700)):
        grid = la.lean_attn_problem_schedule(pr, inp.seqlens, tn).grid
        assert grid > 8
        ws = torch.empty(la.lean_attn_workspace_size_for_grid(pr, grid), dtype=torch.uint8, device="cuda")
        la.lean_attn_workspace_init(ws)
        got, got_lse, _ = _run(inp, tuning=tn, ws=ws)
        _check(got, got_lse, want, want_lse, f"workspace for grid {grid}")
        small = torch.empty(la.lean_attn_workspace_size_for_grid(pr, grid - 1), dtype=torch.uint8, device="cuda")
        la.lean_attn_workspace_init(small)
        out = torch.full((1, 16, 128), 7.0, dtype=torch.float32, device="cuda")
        with pytest.raises(la.LeanAttnError) as e:
            la.lean_attn_decode(inp.q, inp.k, inp.v, inp.seqlens, out, small, Hkv=2, kv_seq_stride=w.n_stride,
                                scale=w.scale, tuning=tn)
        torch.cuda.synchronize()
        assert e.value.status == la.binding.ERR_WORKSPACE and torch.all(out == 7.0)


def test_chunked_batch_with_query_lengths_and_a_forced_grid_stays_inside_the_workspace():
    # 300 sequences run as two launches.  The whole problem has 33 rows per KV head (two blocks of 17),
    # the second chunk only 32 (one block of 32 rows: larger partial slots); with a forced grid of 4096
    # the partial slab of that chunk must still fit the workspace the size query gave.
    r = np.random.default_rng(11)
    B, Hkv, group, D = 300, 1, 11, 64
    q_lens = [int(x) for x in r.integers(0, 3, size=B)]
    q_lens[3] = 3                                   # 33 rows in the first chunk
    q_lens[256:] = [int(x) for x in r.integers(0, 3, size=B - 256)]
    q_lens[299] = 2
    assert max(q_lens[256:]) == 2 and max(q_lens) == 3
    seqlens = [max(int(x), q) for x, q in zip(r.integers(0, 40, size=B), q_lens)]
    seqlens[7], seqlens[280] = 30000, 30000         # enough LeanTile iterations for a grid of 4096
    w = workloads.Workload("chunked_forced_grid", B, Hkv * group, Hkv, D, "bf16", tuple(seqlens), workloads.KV_PACKED,
                           seed=36, N_q=3, causal=True, q_lens=tuple(q_lens))
    inp = workloads.generate(w, device="cuda")
    pr = _problem_of(w).set_q_lens(q_lens)
    nbytes = la.lean_attn_problem_workspace_size(pr)
    # guard bytes after the workspace: a store past its end would land there
    buf = torch.zeros(nbytes + (1 << 20), dtype=torch.uint8, device="cuda")
    ws = buf[:nbytes]
    la.lean_attn_workspace_init(ws)
    n_tok = int(sum(q_lens))
    out = torch.full((n_tok, w.Hq, D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((n_tok, w.Hq), float("nan"), dtype=torch.float32, device="cuda")
    la.lean_attn_attend(pr, inp.q, inp.k, inp.v, inp.seqlens, out, ws, lse=lse, tuning=la.Tuning(grid=4096))
    torch.cuda.synchronize()
    assert la.lean_attn_workspace_status(ws) == 0
    assert torch.all(buf[nbytes:] == 0), "a partial was stored past the end of the workspace"
    want, want_lse = _oracle_ragged(inp)
    _check(out.cpu().numpy(), lse.cpu().numpy(), want, want_lse, "chunked, forced grid")


def test_all_sequences_empty():
    inp = _mk(2, 4, 2, 64, "f16", [0, 0], workloads.KV_PADDED, seed=1)
    # a padded cache needs at least one row of storage to have a valid pointer
    inp.k = torch.zeros(2, 2, 1, 64, dtype=torch.float16, device="cuda")
    inp.v = torch.zeros_like(inp.k)
    ws = _workspace(2, 4, 2, 64, la.F16)
    out = torch.full((2, 4, 64), float("nan"), device="cuda")
    lse = torch.zeros(2, 4, device="cuda")
    la.lean_attn_decode(inp.q, inp.k, inp.v, [0, 0], out, ws, Hkv=2, kv_seq_stride=1, scale=1.0, lse=lse)
    torch.cuda.synchronize()
    assert torch.all(out == 0) and torch.all(torch.isneginf(lse))


def test_waiting_host_gives_up_instead_of_hanging():
    # a spin limit of one poll forces the bounded wait to expire (or not, if the peer was
    # quicker); either way every kernel exits, the status call reports and repairs.
    inp = _mk(1, 2, 2, 128, "bf16", [60000], workloads.KV_PADDED, seed=2)
    want, want_lse = _oracle(inp)
    ws = _workspace(1, 2, 2, 128, la.BF16)
    out = torch.zeros(1, 2, 128, device="cuda")
    la.lean_attn_decode(inp.q, inp.k, inp.v, [60000], out, ws, Hkv=2, kv_seq_stride=60000, scale=inp.w.scale,
                        tuning=la.Tuning(spin_limit=1))
    torch.cuda.synchronize()
    status = la.lean_attn_workspace_status(ws)
    assert status in (0, la.binding.ERR_PEER_TIMEOUT)
    if status == 0:
        _check(out.cpu().numpy(), None, want, want_lse, "no timeout")
    got, got_lse, _ = _run(inp, ws=ws)      # the workspace is usable again
    _check(got, got_lse, want, want_lse, "after status")


@pytest.mark.parametrize("group", [1, 8])
def test_delayed_publishers_and_poisoned_partials_never_change_a_bit(group):
    # The window between StorePartials and Signal (Algorithm 2), and the one before the stores, held open
    # by sleeping publishers; every partial slot holds NaN before every launch, so a partial read before
    # its flag, or a flag seen before its partial, shows.  50 launches per (grid, fan-in), all bit-equal.
    Hkv, D = 2, 128
    seqlens = [50001, 300]
    inp = _mk(2, Hkv * group, Hkv, D, "bf16", seqlens, workloads.KV_PADDED, seed=61, outlier=0.01)
    w = inp.w
    want, want_lse = _oracle(inp)
    ws = _workspace(w.B, w.Hq, w.Hkv, w.D, la.BF16)
    partials = ws[256 + 64 * la.binding.MAX_GRID:].view(torch.float32)     # past the status word and the flags
    delays = ((0, 0, 0), (3, 0, 0), (0, 3, 0), (2, 2, 3), (0, 6, 5))    # (before stores, before flag, every n-th CTA)
    for grid in (64, 256, 1000, 4096):
        for fanin in (2, 8, 32, 4096):
            ref = ref_lse = None
            for (d_store, d_signal, stride) in delays:
                tn = la.Tuning(grid=grid, merge_fanin=fanin, debug_delay_store=d_store, debug_delay_signal=d_signal,
                               debug_delay_stride=stride)
                for _ in range(10):
                    partials.fill_(float("nan"))
                    out = torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.float32, device="cuda")
                    lse = torch.full((w.B, w.Hq), float("nan"), dtype=torch.float32, device="cuda")
                    la.lean_attn_decode(inp.q, inp.k, inp.v, inp.seqlens, out, ws, Hkv=w.Hkv, kv_layout=w.kv_layout,
                                        kv_seq_stride=w.n_stride, scale=w.scale, lse=lse, tuning=tn)
                    if ref is None:
                        torch.cuda.synchronize()
                        assert la.lean_attn_workspace_status(ws) == 0
                        ref, ref_lse = out, lse
                        _check(out.cpu().numpy(), lse.cpu().numpy(), want, want_lse, f"grid={grid} fanin={fanin}")
                    else:
                        assert torch.equal(out, ref) and torch.equal(lse, ref_lse), \
                            f"grid={grid} fanin={fanin} delays={(d_store, d_signal, stride)}: result changed"
            assert la.lean_attn_workspace_status(ws) == 0


@pytest.mark.parametrize("group", [1, 4])
def test_every_tile_shape_and_merge_fanin(group):
    # two output tiles shared by hundreds of CTAs: deep reduction trees, every compiled LeanTile size
    Hkv, D = 2, 128
    seqlens = [70001]
    inp = _mk(1, Hkv * group, Hkv, D, "bf16", seqlens, workloads.KV_PADDED, seed=31, outlier=0.01)
    want, want_lse = _oracle(inp)
    for shape in range(N_SHAPES + 1):          # 0: the default of the table, then every compiled shape
        if not _built(group, D, shape):
            with pytest.raises(la.LeanAttnError) as e:
                _run(inp, la.Tuning(tile_shape=shape))
            assert e.value.status == la.binding.ERR_UNSUPPORTED
            continue
        got, got_lse, _ = _run(inp, la.Tuning(tile_shape=shape))
        _check(got, got_lse, want, want_lse, f"shape={shape}")
    for fanin in (2, 3, 5, 8, 16, 4096):
        for ctas in (1, 2):
            got, got_lse, _ = _run(inp, la.Tuning(merge_fanin=fanin, ctas_per_cu=ctas))
            _check(got, got_lse, want, want_lse, f"fanin={fanin} ctas={ctas}")


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("group", [1, 5, 16])
def test_head_dim_256_every_tile_shape(dtype, group):
    # head dim 256: rows of 512 bytes, two 16-byte pieces per lane and row in the MFMA core
    Hkv, D = 2, 256
    seqlens = [20011, 515]
    inp = _mk(2, Hkv * group, Hkv, D, dtype, seqlens, workloads.KV_PACKED, seed=41 + group, outlier=0.01)
    want, want_lse = _oracle(inp)
    for shape in range(N_SHAPES + 1):
        if not _built(group, D, shape):
            with pytest.raises(la.LeanAttnError) as e:
                _run(inp, la.Tuning(tile_shape=shape))
            assert e.value.status == la.binding.ERR_UNSUPPORTED
            continue
        got, got_lse, _ = _run(inp, la.Tuning(tile_shape=shape))
        _check(got, got_lse, want, want_lse, f"D256 {dtype} g{group} shape={shape}")
    got, got_lse, _ = _run(inp, la.Tuning(grid=1000, merge_fanin=3))
    _check(got, got_lse, want, want_lse, f"D256 {dtype} g{group} grid=1000")


@pytest.mark.parametrize("group", [1, 7])
def test_grid_larger_than_resident(group):
    # more workgroups than fit on the device at once: later ones start as earlier ones retire;
    # blocks only wait for lower CTA ids, so this must neither hang nor change the result
    Hkv, D = 4, 128
    seqlens = [50000, 3, 120000, 9000]
    inp = _mk(4, Hkv * group, Hkv, D, "bf16", seqlens, workloads.KV_PACKED, seed=32)
    want, want_lse = _oracle(inp)
    for tn in (dict(grid_multiple=4), dict(grid=4096), dict(grid=3001, merge_fanin=2), dict(grid=4096, merge_fanin=4096)):
        got, got_lse, _ = _run(inp, la.Tuning(**tn))
        _check(got, got_lse, want, want_lse, f"{tn}")


@pytest.mark.parametrize("group", [1, 8])
def test_fixed_split_baseline_schedules_give_the_same_result(group):
    Hkv, D = 3, 128
    seqlens = [9000, 70, 0, 33000]
    inp = _mk(4, Hkv * group, Hkv, D, "bf16", seqlens, workloads.KV_PACKED, seed=34)
    want, want_lse = _oracle(inp)
    for split in (1, 2, 7, 64, -1):
        got, got_lse, _ = _run(inp, la.Tuning(fixed_split=split))
        _check(got, got_lse, want, want_lse, f"fixed_split={split}")


def test_graph_replay_matches_eager():
    # The decode call allocates nothing, takes its schedule by value and leaves the workspace
    # flags clean, so it can be captured once and replayed.  Replays are interleaved with eager
    # work and synchronisations; every replay must reproduce the eager result bit for bit.
    inp = _mk(2, 16, 2, 128, "bf16", [30000, 4097], workloads.KV_PACKED, seed=35)
    w = inp.w
    want, want_lse = _oracle(inp)
    eager, _, ws = _run(inp)
    out = torch.zeros(w.B, w.Hq, w.D, dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        la.lean_attn_decode(inp.q, inp.k, inp.v, inp.seqlens, out, ws, Hkv=w.Hkv, kv_layout=w.kv_layout,
                            kv_seq_stride=w.n_stride, scale=w.scale)     # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        la.lean_attn_decode(inp.q, inp.k, inp.v, inp.seqlens, out, ws, Hkv=w.Hkv, kv_layout=w.kv_layout,
                            kv_seq_stride=w.n_stride, scale=w.scale)
    for i in range(4):
        out.fill_(float("nan"))
        scratch = torch.randn(1 << 20, device="cuda").sum()          # unrelated eager work in between
        graph.replay()
        torch.cuda.synchronize()
        assert la.lean_attn_workspace_status(ws) == 0
        got = out.cpu().numpy()
        assert np.array_equal(got, eager), f"replay {i} differs from the eager launch"
        del scratch
    _check(got, None, want, want_lse, "graph replay")


def test_maximum_batch_ragged():
    # the largest batch the schedule table holds, lengths from 0 to a few tiles, both layouts
    r = np.random.default_rng(256)
    seqlens = [int(x) for x in r.integers(0, 700, size=la.binding.MAX_BATCH)]
    seqlens[0], seqlens[-1], seqlens[100] = 0, 0, 1
    for group, layout in ((1, workloads.KV_PACKED), (4, workloads.KV_PADDED)):
        inp = _mk(len(seqlens), 2 * group, 2, 64, "f16", seqlens, layout, seed=33)
        want, want_lse = _oracle(inp)
        got, got_lse, _ = _run(inp)
        _check(got, got_lse, want, want_lse, f"B=256 group={group}")
    with pytest.raises(la.LeanAttnError) as e:
        la.lean_attn_schedule(seqlens + [5], 2, 2, 64, la.F16, la.KV_PACKED)
    assert e.value.status == la.binding.ERR_BATCH_TOO_LARGE


def test_batches_beyond_one_launch_are_split():
    # 700 sequences: three consecutive launches share the workspace; decode, both layouts
    r = np.random.default_rng(700)
    seqlens = [int(x) for x in r.integers(0, 300, size=700)]
    seqlens[255], seqlens[256], seqlens[511], seqlens[512] = 299, 0, 1, 257
    for group, layout in ((1, workloads.KV_PACKED), (4, workloads.KV_PADDED)):
        inp = _mk(len(seqlens), 2 * group, 2, 64, "bf16", seqlens, layout, seed=34)
        want, want_lse = _oracle(inp)
        got, got_lse, _ = _run(inp)
        _check(got, got_lse, want, want_lse, f"B=700 group={group}")
    # per-sequence query lengths across the launch boundaries, one chunk without any query token
    q_lens = [int(x) for x in r.integers(0, 4, size=700)]
    q_lens[256:512] = [0] * 256
    q_lens[0], q_lens[699] = 3, 2
    seq2 = [max(n, q) for n, q in zip(seqlens, q_lens)]
    w = workloads.Workload("b700_mixed", 700, 8, 2, 128, "f16", tuple(seq2), workloads.KV_PACKED, seed=35,
                           N_q=max(q_lens), causal=True, q_lens=tuple(q_lens))
    inp = workloads.generate(w, device="cuda")
    want, want_lse = _oracle_ragged(inp)
    got, got_lse = _run_ragged(inp)
    _check(got.cpu().numpy(), got_lse, want, want_lse, "B=700 mixed")
    # an invalid length in the last chunk: nothing may have been launched
    bad = list(seqlens)
    bad[650] = -1
    out = torch.full((700, 2, 64), 7.0, dtype=torch.float32, device="cuda")
    inp = _mk(700, 2, 2, 64, "bf16", seqlens, workloads.KV_PADDED, seed=34)
    ws = _workspace(700, 2, 2, 64, la.BF16)
    with pytest.raises(la.LeanAttnError) as e:
        la.lean_attn_decode(inp.q, inp.k, inp.v, bad, out, ws, Hkv=2, kv_layout=la.KV_PADDED,
                            kv_seq_stride=inp.w.n_stride, scale=0.125)
    torch.cuda.synchronize()
    assert e.value.status == la.binding.ERR_SEQLEN and torch.all(out == 7.0)


# ------------------------------------------------------------------ the five workloads, scaled down
@pytest.mark.parametrize("idx,factor", [(1, 1), (2, 8), (3, 16), (4, 16), (5, 16)])
def test_named_workloads_scaled(idx, factor):
    w = workloads.named(idx)
    if factor > 1:
        w = workloads.scaled_down(w, factor)
    inp = workloads.generate(w, device="cuda")
    want, want_lse = _oracle(inp)
    got, got_lse, _ = _run(inp)
    max_abs, rel_l2 = _check(got, got_lse, want, want_lse, w.name)
    print(f"{w.name}: max_abs={max_abs:.2e} rel_l2={rel_l2:.2e}")


# ------------------------------------------------------------------ full sizes, as bench.py launches them
@pytest.mark.parametrize("idx", [2, 3, 5])
def test_named_workloads_full_size(idx):
    w = workloads.named(idx)
    inp = workloads.generate(w, device="cuda")
    got, got_lse, _ = _run(inp)
    want, want_lse = _oracle(inp)
    max_abs, rel_l2 = _check(got, got_lse, want, want_lse, w.name)
    print(f"{w.name}: max_abs={max_abs:.2e} rel_l2={rel_l2:.2e}")


@pytest.mark.parametrize("idx", [6, 7, 8])
def test_widened_named_workloads_full_size(idx):
    # head dim 256; a causal query tile of 4 tokens x 4 heads per KV head; 32 query heads per KV head
    w = workloads.named(idx)
    inp = workloads.generate(w, device="cuda")
    got, got_lse = _run_attend(inp)
    want, want_lse = _oracle_attend(inp)
    max_abs, rel_l2 = _check(got.cpu().numpy().reshape(want.shape), got_lse, want, want_lse, w.name)
    print(f"{w.name}: max_abs={max_abs:.2e} rel_l2={rel_l2:.2e}")


def test_ragged_batch_full_size_sampled_heads():
    # 21 GB of cache: the oracle checks every sequence for a seeded sample of 8 of the 32 KV heads
    w = workloads.named(4)
    inp = workloads.generate(w, device="cuda")
    got, got_lse, _ = _run(inp)
    assert np.all(np.isfinite(got))
    heads = sorted(np.random.default_rng(4).choice(w.Hkv, size=8, replace=False).tolist())
    for h in heads:
        sub = workloads.Workload("sub", w.B, 1, 1, w.D, w.dtype, w.seqlens, workloads.KV_PACKED)
        want, want_lse = oracle.decode_attention(inp.q[:, h:h + 1].contiguous(), inp.k[h:h + 1], inp.v[h:h + 1],
                                                 inp.seqlens, Hq=1, Hkv=1, D=w.D, scale=w.scale,
                                                 kv_layout=oracle.KV_PACKED)
        _check(got[:, h:h + 1], got_lse[:, h:h + 1], want, want_lse, f"{w.name} head {h}")
        del sub


# ------------------------------------------------------------------ query tiles (N_q > 1), row blocks, 16-bit out
def _mk_tile(B, N_q, Hq, Hkv, D, dtype, seqlens, layout, seed, causal, outlier=0.0):
    w = workloads.Workload(f"t_b{B}_q{N_q}_h{Hq}_{Hkv}_d{D}_{dtype}", B, Hq, Hkv, D, dtype, tuple(seqlens), layout,
                           seed=seed, outlier_frac=outlier, N_q=N_q, causal=causal)
    return workloads.generate(w, device="cuda")


def _problem_of(w, out_dtype=la.OUT_F32):
    return la.Problem(B=w.B, N_q=w.N_q, Hq=w.Hq, Hkv=w.Hkv, D=w.D, dtype=la.F16 if w.dtype == "f16" else la.BF16,
                      out_dtype=out_dtype, kv_layout=w.kv_layout, causal=int(w.causal), scale=w.scale,
                      kv_seq_stride=w.n_stride)


def _run_attend(inp, tuning=None, out_dtype=la.OUT_F32, want_lse=True):
    w = inp.w
    pr = _problem_of(w, out_dtype)
    ws = torch.empty(la.lean_attn_problem_workspace_size(pr), dtype=torch.uint8, device="cuda")
    la.lean_attn_workspace_init(ws)
    odt = torch.float32 if out_dtype == la.OUT_F32 else w.torch_dtype
    out = torch.full((w.B, w.N_q, w.Hq, w.D), float("nan"), dtype=odt, device="cuda")
    lse = torch.full((w.B, w.N_q, w.Hq), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    la.lean_attn_attend(pr, inp.q, inp.k, inp.v, inp.seqlens, out, ws, lse=lse, tuning=tuning)
    torch.cuda.synchronize()
    assert la.lean_attn_workspace_status(ws) == 0
    return out, (lse.cpu().numpy() if want_lse else None)


def _oracle_attend(inp):
    w = inp.w
    return oracle.attention(inp.q, inp.k, inp.v, inp.seqlens, N_q=w.N_q, Hq=w.Hq, Hkv=w.Hkv, D=w.D, scale=w.scale,
                            causal=w.causal, kv_layout=w.kv_layout, n_stride=w.n_stride)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("D", [64, 128, 256])
@pytest.mark.parametrize("N_q,group", [(2, 1), (4, 4), (16, 1), (3, 8), (5, 7), (1, 17), (1, 32), (16, 16)])
def test_query_tiles_and_row_blocks_small_shapes(causal, D, N_q, group):
    # rows per KV head from 2 to 256: one block, several blocks, a ragged last block
    Hkv = 2
    seqlens = [1000, N_q, 0, 257, 64 + N_q]      # one sequence holds only its query tokens, one is empty
    dtype = "bf16" if (N_q + group) % 2 else "f16"
    for layout in (workloads.KV_PADDED, workloads.KV_PACKED):
        inp = _mk_tile(len(seqlens), N_q, Hkv * group, Hkv, D, dtype, seqlens, layout, seed=50 + N_q + group,
                       causal=causal)
        want, want_lse = _oracle_attend(inp)
        got, got_lse = _run_attend(inp)
        _check(got.cpu().numpy(), got_lse, want, want_lse, f"N_q={N_q} g={group} D={D} causal={causal} l={layout}")
        assert np.all(got[2].cpu().numpy() == 0.0) and np.all(np.isneginf(got_lse[2]))


@pytest.mark.parametrize("N_q,group", [(4, 4), (6, 8)])
def test_query_tiles_deep_trees_any_split_and_tile_shape(N_q, group):
    Hkv, D = 2, 128
    seqlens = [50001, 4099]
    inp = _mk_tile(2, N_q, Hkv * group, Hkv, D, "bf16", seqlens, workloads.KV_PADDED, seed=61, causal=True,
                   outlier=0.01)
    want, want_lse = _oracle_attend(inp)
    for tn in (la.Tuning(), la.Tuning(grid=3), la.Tuning(grid=1000, merge_fanin=3), la.Tuning(fixed_split=5),
               la.Tuning(tile_shape=1), la.Tuning(tile_shape=4), la.Tuning(tile_shape=5, ctas_per_cu=2),
               la.Tuning(tile_shape=7), la.Tuning(tile_shape=8, grid=700), la.Tuning(tile_shape=9, fixed_split=3)):
        got, got_lse = _run_attend(inp, tn)
        _check(got.cpu().numpy(), got_lse, want, want_lse, f"N_q={N_q} g={group} grid={tn.grid} shape={tn.tile_shape}")


def test_causal_last_row_equals_plain_decode():
    # the last query row sees the whole context: same rows as a decode call on the same cache
    Hkv, group, D, N_q = 2, 4, 128, 4
    inp = _mk_tile(1, N_q, Hkv * group, Hkv, D, "bf16", [9000], workloads.KV_PADDED, seed=63, causal=True)
    got, _ = _run_attend(inp)
    w = inp.w
    out = torch.empty(1, w.Hq, D, dtype=torch.float32, device="cuda")
    ws = _workspace(1, w.Hq, Hkv, D, la.BF16)
    la.lean_attn_decode(inp.q[:, -1].contiguous(), inp.k, inp.v, inp.seqlens, out, ws, Hkv=Hkv,
                        kv_seq_stride=w.n_stride, scale=w.scale)
    torch.cuda.synchronize()
    assert torch.max(torch.abs(out - got[:, -1])).item() < 2e-6


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("N_q,group", [(1, 1), (1, 8), (3, 8)])
def test_sixteen_bit_output_is_the_rounded_fp32_output(dtype, N_q, group):
    Hkv, D = 3, 128
    seqlens = [3000, 0, 129 + N_q]
    inp = _mk_tile(3, N_q, Hkv * group, Hkv, D, dtype, seqlens, workloads.KV_PACKED, seed=70 + group, causal=N_q > 1)
    want, want_lse = _oracle_attend(inp)
    out32, lse32 = _run_attend(inp)
    out16, lse16 = _run_attend(inp, out_dtype=la.OUT_AS_INPUT)
    assert out16.dtype == inp.w.torch_dtype
    # same kernel, same arithmetic: the 16-bit result is the fp32 result rounded to nearest even
    assert torch.equal(out16, out32.to(out16.dtype))
    assert np.array_equal(lse16, lse32, equal_nan=True)
    # against the oracle: half an ulp of the output type on top of the fp32 bar
    half_ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -11      # relative, 8 and 11 significand bits
    err = np.abs(out16.float().cpu().numpy() - want)
    assert np.all(err <= TIGHT_ABS + half_ulp * np.abs(want) * 1.01 + 1e-7)
    assert np.all(out16[1].float().cpu().numpy() == 0.0)


def test_all_sequences_empty_with_query_tiles_and_sixteen_bit_output():
    inp = _mk_tile(2, 3, 4, 2, 64, "f16", [0, 0], workloads.KV_PADDED, seed=80, causal=True)
    # a PADDED cache whose rows are never read (a stride of 0 would leave no memory to point at)
    pr = _problem_of(inp.w, la.OUT_AS_INPUT)
    pr.kv_seq_stride = 4
    kv = torch.zeros(2, 2, 4, 64, dtype=torch.float16, device="cuda")
    ws = torch.empty(la.lean_attn_problem_workspace_size(pr), dtype=torch.uint8, device="cuda")
    la.lean_attn_workspace_init(ws)
    out = torch.full((2, 3, 4, 64), float("nan"), dtype=torch.float16, device="cuda")
    lse = torch.full((2, 3, 4), float("nan"), dtype=torch.float32, device="cuda")
    la.lean_attn_attend(pr, inp.q, kv, kv, [0, 0], out, ws, lse=lse)
    torch.cuda.synchronize()
    assert torch.all(out == 0) and torch.all(torch.isneginf(lse))


def test_attend_error_paths():
    inp = _mk_tile(1, 4, 4, 2, 128, "bf16", [100], workloads.KV_PADDED, seed=81, causal=True)
    pr = _problem_of(inp.w)
    ws = torch.empty(la.lean_attn_problem_workspace_size(pr), dtype=torch.uint8, device="cuda")
    la.lean_attn_workspace_init(ws)
    out = torch.zeros(1, 4, 4, 128, device="cuda")
    with pytest.raises(la.LeanAttnError) as e:       # causal with fewer cached tokens than query rows
        la.lean_attn_attend(pr, inp.q, inp.k, inp.v, [3], out, ws)
    assert e.value.status == la.binding.ERR_SEQLEN
    with pytest.raises(la.LeanAttnError) as e:       # workspace sized for a smaller tile on the same grid
        grid = la.lean_attn_problem_schedule(pr, [100]).grid
        one_row = la.Problem(B=1, N_q=1, Hq=2, Hkv=2, D=128, dtype=la.BF16, out_dtype=la.OUT_F32,
                             kv_layout=la.KV_PADDED, causal=0, scale=1.0, kv_seq_stride=100)
        small = torch.empty(la.lean_attn_workspace_size_for_grid(one_row, grid), dtype=torch.uint8, device="cuda")
        la.lean_attn_attend(pr, inp.q, inp.k, inp.v, [100], out, small)
    assert e.value.status == la.binding.ERR_WORKSPACE
    with pytest.raises(ValueError):                  # out dtype must match the problem
        la.lean_attn_attend(pr, inp.q, inp.k, inp.v, [100], out.to(torch.bfloat16), ws)
    la.lean_attn_attend(pr, inp.q, inp.k, inp.v, [100], out, ws)
    torch.cuda.synchronize()
    want, _ = _oracle_attend(inp)
    _check(out.cpu().numpy(), None, want, None, "after errors")


def test_two_streams_with_their_own_workspaces_run_concurrently():
    # calls in flight at the same time need separate workspaces, nothing else; each launch's
    # workgroups only wait for lower ids of their own launch, so co-resident launches cannot block each other
    inp_a = _mk(2, 16, 2, 128, "bf16", [40000, 999], workloads.KV_PADDED, seed=90)
    inp_b = _mk(3, 8, 8, 64, "f16", [30000, 1, 5000], workloads.KV_PACKED, seed=91)
    want_a, _ = _oracle(inp_a)
    want_b, _ = _oracle(inp_b)
    outs, wss, streams = [], [], [torch.cuda.Stream(), torch.cuda.Stream()]
    for inp in (inp_a, inp_b):
        w = inp.w
        wss.append(_workspace(w.B, w.Hq, w.Hkv, w.D, la.F16 if w.dtype == "f16" else la.BF16))
        outs.append(torch.full((w.B, w.Hq, w.D), float("nan"), dtype=torch.float32, device="cuda"))
    torch.cuda.synchronize()
    for rep in range(20):
        for i, inp in enumerate((inp_a, inp_b)):
            w = inp.w
            la.lean_attn_decode(inp.q, inp.k, inp.v, inp.seqlens, outs[i], wss[i], Hkv=w.Hkv, kv_layout=w.kv_layout,
                                kv_seq_stride=w.n_stride, scale=w.scale, stream=streams[i])
    torch.cuda.synchronize()
    assert la.lean_attn_workspace_status(wss[0]) == 0 and la.lean_attn_workspace_status(wss[1]) == 0
    _check(outs[0].cpu().numpy(), None, want_a, None, "stream 0")
    _check(outs[1].cpu().numpy(), None, want_b, None, "stream 1")


# ------------------------------------------------------------------ per-sequence query lengths (mixed batches)
def _run_ragged(inp, tuning=None, out_dtype=la.OUT_F32):
    w = inp.w
    pr = _problem_of(w, out_dtype).set_q_lens(list(w.q_lens))
    ws = torch.empty(la.lean_attn_problem_workspace_size(pr), dtype=torch.uint8, device="cuda")
    la.lean_attn_workspace_init(ws)
    n_tok = int(sum(w.q_lens))
    odt = torch.float32 if out_dtype == la.OUT_F32 else w.torch_dtype
    out = torch.full((n_tok, w.Hq, w.D), float("nan"), dtype=odt, device="cuda")
    lse = torch.full((n_tok, w.Hq), float("nan"), dtype=torch.float32, device="cuda")
    la.lean_attn_attend(pr, inp.q, inp.k, inp.v, inp.seqlens, out, ws, lse=lse, tuning=tuning)
    torch.cuda.synchronize()
    assert la.lean_attn_workspace_status(ws) == 0
    return out, lse.cpu().numpy()


def _oracle_ragged(inp):
    w = inp.w
    return oracle.attention_ragged(inp.q, inp.k, inp.v, inp.seqlens, list(w.q_lens), Hq=w.Hq, Hkv=w.Hkv, D=w.D,
                                   scale=w.scale, causal=w.causal, kv_layout=w.kv_layout, n_stride=w.n_stride)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("D", [64, 128, 256])
@pytest.mark.parametrize("group", [1, 4, 8])
def test_mixed_prefill_and_decode_batch(causal, D, group):
    # a prefill chunk, decode steps, a sequence without queries, an empty context, a chunk that is the whole context
    Hkv = 2
    q_lens = [7, 1, 0, 3, 1, 12]
    seqlens = [900, 3000, 500, 0, 1, 12]
    for layout in (workloads.KV_PADDED, workloads.KV_PACKED):
        w = workloads.Workload(f"mixed_g{group}_d{D}", len(seqlens), Hkv * group, Hkv, D, "bf16", tuple(seqlens), layout,
                               seed=95 + group, N_q=max(q_lens), causal=causal, q_lens=tuple(q_lens))
        inp = workloads.generate(w, device="cuda")
        want, want_lse = _oracle_ragged(inp)
        for tn in (None, la.Tuning(grid=37, merge_fanin=3)):
            got, got_lse = _run_ragged(inp, tn)
            _check(got.cpu().numpy(), got_lse, want, want_lse, f"mixed g={group} D={D} causal={causal} layout={layout}")
        # rows of the sequence with an empty context
        first = sum(q_lens[:3])
        assert torch.all(got[first:first + 3] == 0) and np.all(np.isneginf(got_lse[first:first + 3]))


def test_mixed_batch_long_contexts_and_sixteen_bit_output():
    # 64 rows per KV head at the longest (two output tiles), decode sequences reach only the first
    Hkv, group, D = 2, 8, 128
    q_lens = [8, 1, 1, 3]
    seqlens = [30000, 52001, 777, 4100]
    w = workloads.Workload("mixed_long", 4, Hkv * group, Hkv, D, "bf16", tuple(seqlens), workloads.KV_PACKED, seed=99,
                           N_q=8, causal=True, q_lens=tuple(q_lens), outlier_frac=0.01)
    inp = workloads.generate(w, device="cuda")
    want, want_lse = _oracle_ragged(inp)
    got, got_lse = _run_ragged(inp)
    _check(got.cpu().numpy(), got_lse, want, want_lse, "mixed long")
    got16, _ = _run_ragged(inp, out_dtype=la.OUT_AS_INPUT)
    assert torch.equal(got16, got.to(torch.bfloat16))
    # uniform lengths through the per-sequence path give the [B, N_q, ...] result bit for bit
    wu = workloads.Workload("uniform", 2, 8, 2, 128, "bf16", (5000, 300), workloads.KV_PADDED, seed=98, N_q=3, causal=True)
    inp_u = workloads.generate(wu, device="cuda")
    a, a_lse = _run_attend(inp_u)
    wr = workloads.Workload("uniform_r", 2, 8, 2, 128, "bf16", (5000, 300), workloads.KV_PADDED, seed=98, N_q=3, causal=True,
                            q_lens=(3, 3))
    inp_r = workloads.Inputs(wr, inp_u.q.reshape(6, 8, 128), inp_u.k, inp_u.v, list(wr.seqlens))
    b, b_lse = _run_ragged(inp_r)
    assert torch.equal(a.reshape(6, 8, 128), b) and np.array_equal(a_lse.reshape(6, 8), b_lse)


def test_read_probe_modes_and_argument_checks():
    # the measurement helper: every access pattern runs on ragged sizes, bad arguments are refused
    sink = torch.zeros(16, dtype=torch.int32, device="cuda")
    for nbytes in (16, 4096 + 16, (3 << 20) + 48):
        buf = torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device="cuda")
        for mode in range(7):
            for grid in (1, 7, 512):
                la.lean_attn_read_probe(buf, sink, grid, mode)
    torch.cuda.synchronize()
    assert int(sink[0].item()) in (0, 0x9e3779b9 - (1 << 32))     # only written if the folded word hits one magic value
    buf = torch.zeros(64, dtype=torch.uint8, device="cuda")
    for kwargs in (dict(grid=0, mode=0), dict(grid=70000, mode=0), dict(grid=4, mode=7), dict(grid=4, mode=-1)):
        with pytest.raises(la.LeanAttnError) as e:
            la.lean_attn_read_probe(buf, sink, **kwargs)
        assert e.value.status == la.binding.ERR_BAD_SHAPE
    with pytest.raises(la.LeanAttnError):
        la.lean_attn_read_probe(buf[:40], sink, 4, 0)            # not a multiple of 16 bytes


def test_prepared_call_replays_the_checked_call():
    inp = _mk(2, 8, 2, 128, "bf16", [7000, 333], workloads.KV_PADDED, seed=97)
    w = inp.w
    ws = _workspace(w.B, w.Hq, w.Hkv, w.D, la.BF16)
    direct = torch.empty(w.B, w.Hq, w.D, dtype=torch.float32, device="cuda")
    la.lean_attn_decode(inp.q, inp.k, inp.v, inp.seqlens, direct, ws, Hkv=w.Hkv, kv_seq_stride=w.n_stride, scale=w.scale)
    out = torch.full_like(direct, float("nan"))
    call = la.lean_attn_decode(inp.q, inp.k, inp.v, inp.seqlens, out, ws, Hkv=w.Hkv, kv_seq_stride=w.n_stride,
                               scale=w.scale, prepare_only=True)
    torch.cuda.synchronize()
    assert isinstance(call, la.PreparedCall) and torch.all(torch.isnan(out))      # nothing launched yet
    for _ in range(3):
        out.fill_(float("nan"))
        call()
        torch.cuda.synchronize()
        assert torch.equal(out, direct)
    # the general entry point, and a prepared call that the library refuses when it is made
    inp2 = _mk_tile(2, 3, 8, 2, 128, "bf16", [500, 40], workloads.KV_PADDED, seed=96, causal=True)
    a, _ = _run_attend(inp2)
    pr = _problem_of(inp2.w)
    ws2 = torch.empty(la.lean_attn_problem_workspace_size(pr), dtype=torch.uint8, device="cuda")
    la.lean_attn_workspace_init(ws2)
    b = torch.empty_like(a)
    la.lean_attn_attend(pr, inp2.q, inp2.k, inp2.v, inp2.seqlens, b, ws2, prepare_only=True)()
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    bad = la.lean_attn_attend(pr, inp2.q, inp2.k, inp2.v, [500, 2], b, ws2, prepare_only=True)   # 2 < N_q, causal
    with pytest.raises(la.LeanAttnError):
        bad()


def test_seeded_random_problems_against_the_oracle():
    # 60 seeded problems over every option at once: shapes, layouts, masks, per-sequence query
    # lengths, output type, schedule overrides
    r = np.random.default_rng(20240517)
    for case in range(60):
        D = int(r.choice([64, 128, 256]))
        Hkv = int(r.integers(1, 4))
        group = int(r.choice([1, 2, 3, 4, 7, 8, 16, 20]))
        N_q = int(r.choice([1, 1, 2, 3, 5, 8]))
        if N_q * group > 256:
            N_q = 1
        B = int(r.integers(1, 6))
        causal = bool(r.integers(0, 2)) and N_q > 1
        ragged_q = bool(r.integers(0, 2)) and N_q > 1
        q_lens = [int(x) for x in r.integers(0, N_q + 1, size=B)] if ragged_q else [N_q] * B
        if ragged_q:
            q_lens[int(r.integers(0, B))] = N_q
        seqlens = []
        for b in range(B):
            kind = int(r.integers(0, 6))
            n = [0, q_lens[b], int(r.integers(1, 70)), int(r.integers(70, 700)), int(r.integers(700, 5000)),
                 64 * int(r.integers(1, 20))][kind]
            if causal and n != 0:
                n = max(n, q_lens[b])
            seqlens.append(n)
        layout = int(r.integers(0, 2))
        dtype = "bf16" if r.integers(0, 2) else "f16"
        out_dtype = la.OUT_AS_INPUT if r.integers(0, 3) == 0 else la.OUT_F32
        tn = la.Tuning(grid=int(r.choice([0, 0, 1, 5, 64, 700])), merge_fanin=int(r.choice([0, 0, 2, 5, 4096])),
                       tile_shape=int(r.integers(0, N_SHAPES + 1)), ctas_per_cu=int(r.choice([0, 1, 2])),
                       fixed_split=int(r.choice([0, 0, 0, 1, 3])))
        if not _built(N_q * group, D, tn.tile_shape):
            tn.tile_shape = 2
        label = (f"case {case}: D={D} Hkv={Hkv} g={group} N_q={N_q} q_lens={q_lens if ragged_q else None} B={B} "
                 f"seqlens={seqlens} causal={causal} layout={layout} {dtype} out16={out_dtype} grid={tn.grid} "
                 f"fanin={tn.merge_fanin} shape={tn.tile_shape} per_cu={tn.ctas_per_cu} split={tn.fixed_split}")
        w = workloads.Workload(f"rnd{case}", B, Hkv * group, Hkv, D, dtype, tuple(seqlens), layout, seed=3000 + case,
                               outlier_frac=0.02 if case % 3 == 0 else 0.0, N_q=N_q, causal=causal,
                               q_lens=tuple(q_lens) if ragged_q else None)
        if layout == workloads.KV_PADDED and max(seqlens) == 0:
            continue                                  # a padded cache of stride 0 has no memory to point at
        inp = workloads.generate(w, device="cuda")
        if ragged_q:
            if sum(q_lens) == 0:
                continue
            want, want_lse = _oracle_ragged(inp)
            got, got_lse = _run_ragged(inp, tn, out_dtype)
        else:
            want, want_lse = _oracle_attend(inp)
            got, got_lse = _run_attend(inp, tn, out_dtype)
        got = got.float().cpu().numpy().reshape(want.shape)
        got_lse = got_lse.reshape(want_lse.shape)
        if out_dtype == la.OUT_F32:
            _check(got, got_lse, want, want_lse, label)
        else:
            half_ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -11
            assert np.all(np.abs(got - want) <= TIGHT_ABS + half_ulp * np.abs(want) * 1.01 + 1e-7), label


@pytest.mark.parametrize("group,N_q", [(1, 1), (4, 1), (8, 3)])
def test_one_captured_graph_serves_changing_lengths(group, N_q):
    # a decode loop: the launch is captured once; before each replay the host rewrites the argument
    # block for the new lengths (the grid never depends on them)
    Hkv, D, B, stride = 2, 128, 4, 6000
    causal = N_q > 1
    w0 = workloads.Workload("graph_loop", B, Hkv * group, Hkv, D, "bf16", (stride,) * B, workloads.KV_PADDED, seed=120 + group,
                            N_q=N_q, causal=causal)
    inp = workloads.generate(w0, device="cuda")          # a cache of `stride` rows per sequence, filled
    pr = _problem_of(w0)
    ws = torch.empty(la.lean_attn_problem_workspace_size(pr), dtype=torch.uint8, device="cuda")
    la.lean_attn_workspace_init(ws)
    out = torch.full((B, N_q, w0.Hq, D), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((B, N_q, w0.Hq), float("nan"), dtype=torch.float32, device="cuda")
    nbytes = la.lean_attn_launch_block_size()
    block_host = torch.zeros(nbytes, dtype=torch.uint8).pin_memory()
    block_dev = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    q4 = inp.q.view(B, N_q, w0.Hq, D)

    steps = [[3000, 17, 5999, 64], [3001, 18, 6000, 65], [0, N_q, 1500, 1], [0, 0, 0, 0], [6000, 6000, 6000, 6000],
             [N_q, 1000, 0, 4097]]
    steps = [[n if (n == 0 or n >= N_q) else N_q for n in s] for s in steps]
    # eager first (also the first call on this device: runtime queries happen outside the capture)
    la.lean_attn_attend_prepare(pr, q4, inp.k, inp.v, steps[0], out, ws, block_host, lse=lse)
    la.lean_attn_launch(block_host, block_dev)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        la.lean_attn_launch(block_host, block_dev)
    for seqlens in steps:
        la.lean_attn_attend_prepare(pr, q4, inp.k, inp.v, seqlens, out, ws, block_host, lse=lse)
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert la.lean_attn_workspace_status(ws) == 0
        want, want_lse = oracle.attention(q4, inp.k, inp.v, seqlens, N_q=N_q, Hq=w0.Hq, Hkv=Hkv, D=D, scale=w0.scale,
                                          causal=causal, n_stride=stride)
        _check(out.cpu().numpy(), lse.cpu().numpy(), want, want_lse, f"graph loop g={group} N_q={N_q} {seqlens}")
        # the same lengths through the one-call entry point: bit-identical when it picks the same grid
        ref = torch.empty_like(out)
        la.lean_attn_attend(pr, q4, inp.k, inp.v, seqlens, ref, ws, tuning=la.Tuning(ctas_per_cu=1))
        torch.cuda.synchronize()
        plan = la.lean_attn_problem_schedule(pr, seqlens, la.Tuning(ctas_per_cu=1))
        if plan.grid == 256 and plan.total_iters > 0:
            assert torch.equal(out, ref)
    # a refused update leaves the block launchable as it was
    with pytest.raises(la.LeanAttnError):
        la.lean_attn_attend_prepare(pr, q4, inp.k, inp.v, [1, 2, 3, stride + 1], out, ws, block_host)
    graph.replay()
    torch.cuda.synchronize()
    want, _ = oracle.attention(q4, inp.k, inp.v, steps[-1], N_q=N_q, Hq=w0.Hq, Hkv=Hkv, D=D, scale=w0.scale,
                               causal=causal, n_stride=stride)
    _check(out.cpu().numpy(), None, want, None, "after a refused update")


@pytest.mark.parametrize("group", [1, 4, 20])
def test_tail_spans_against_the_oracle(group):
    # tuning.tail_grid: the end of the iteration line in short spans for further workgroups, which start
    # as the first ones retire -- another decomposition of the same sum (Section 4.1), both cores
    Hkv, D = 2, 128
    seqlens = [30011, 517, 0, 9000]
    inp = _mk(4, Hkv * group, Hkv, D, "bf16", seqlens, workloads.KV_PACKED, seed=71 + group, outlier=0.01)
    want, want_lse = _oracle(inp)
    code = la.BF16
    with_tail = 0
    for tn in (la.Tuning(tail_grid=64), la.Tuning(tail_grid=256, tail_permille=200), la.Tuning(grid=7, tail_grid=3, tail_permille=500),
               la.Tuning(grid=64, tail_grid=1000, tail_permille=1), la.Tuning(tail_grid=16, merge_fanin=3), la.Tuning(grid=700, tail_grid=300)):
        plan = la.lean_attn_schedule(seqlens, Hkv * group, Hkv, D, code, la.KV_PACKED, tn)
        assert plan.tail_grid in (0, tn.tail_grid) and plan.grid > plan.tail_grid     # 0: too few iterations for this tail
        with_tail += plan.tail_grid > 0
        got, got_lse, _ = _run(inp, tn)
        _check(got, got_lse, want, want_lse, f"g{group} grid={plan.grid} tail={plan.tail_grid}/{plan.tail_iters}")
        again, again_lse, _ = _run(inp, tn)
        assert np.array_equal(got, again) and np.array_equal(got_lse, again_lse)      # a static decomposition
    assert with_tail >= 4
