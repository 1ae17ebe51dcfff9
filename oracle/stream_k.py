"""TEST INFRASTRUCTURE -- the stream-K decomposition of Section 4.3 as interval arithmetic, in
fp64 numpy.

This is not the oracle of the result (that is ``exact_attention.c``); it pins the *bookkeeping*
the decode kernel must reproduce: which workgroup computes which LeanTile iterations of which
output tile, who holds a tile's first and last iteration, how many partials a workgroup can have
to hand over.  It is built from the definition of the decomposition, not from the control flow of
the paper's listings:

  * the LeanTile iterations of all output tiles lie on one line; the tile edges are the prefix
    sums of the per-tile iteration counts ``C_n = ceil(N_b / T_n)`` (tiles of empty sequences have
    zero length) and the span edges cut the same line into ``G`` near-equal parts;
  * every piece of work is an interval between two consecutive cut points of the union of both
    edge sets: it lies in exactly one span (its workgroup) and one tile;
  * each piece yields a partial ``(O~, m, l)`` by the first display of Section 4.1, the pieces of a
    tile are folded with the operator ``f`` of its second display in ANY order and bracketing
    (associativity, Section 4.1), and the tile's rows are ``O~ / l``.

Readings taken where the paper is silent or garbled:
  * scores are scaled by ``scale`` before max/exp (Eq. 1 has 1/sqrt(d), Section 4 drops it);
  * the line holds the iterations of every (sequence, KV head) tile, as the TilesPerCTA equation of
    Section 4.3 counts them;
  * when the total is not a multiple of ``G`` the first ``I mod G`` workgroups take one iteration
    more, and there are never more workgroups than iterations;
  * tokens past ``N_b`` in a tile's last iteration do not exist (they take no part in max or sum);
  * a query group sharing one KV head forms the rows of one output tile (the paper has no GQA).
"""
from __future__ import annotations

import math

import numpy as np

from . import rescale


def span_edges(total_iters: int, G: int, tail=None) -> np.ndarray:
    """Cut points of the spans: workgroup g owns iterations [edges[g], edges[g+1]).

    ``tail = (P, tail_iters)``: the last ``tail_iters`` iterations are cut into ``P`` near-equal spans of
    their own (workgroups G .. G+P-1) and the first ``G`` workgroups share the rest: the decomposition
    is still a set of consecutive intervals, which is all Section 4.3 needs."""
    if total_iters <= 0:
        return np.zeros(1, dtype=np.int64)
    G = max(1, min(int(G), int(total_iters)))
    if tail is not None and tail[0] > 0:
        P, tail_iters = int(tail[0]), int(tail[1])
        assert P <= tail_iters <= total_iters - G
        head = span_edges(total_iters - tail_iters, G)
        return np.concatenate([head, head[-1] + span_edges(tail_iters, P)[1:]])
    g = np.arange(G + 1, dtype=np.int64)
    return g * (total_iters // G) + np.minimum(g, total_iters % G)


def spans(total_iters: int, G: int):
    e = span_edges(total_iters, G)
    return [(int(e[i]), int(e[i + 1])) for i in range(len(e) - 1)]


def tile_edges(seqlens, Hkv: int, T_n: int, order: str = "padded"):
    """Output tiles in linearisation order and the cut points between them.

    ``order``: "padded" = sequence -> head -> context, "packed" = head -> sequence -> context.
    Returns (tiles, edges): tiles[i] = (b, h) owns iterations [edges[i], edges[i+1])."""
    B = len(seqlens)
    if order == "padded":
        tiles = [(b, h) for b in range(B) for h in range(Hkv)]
    else:
        tiles = [(b, h) for h in range(Hkv) for b in range(B)]
    counts = [math.ceil(seqlens[b] / T_n) for (b, _h) in tiles]
    return tiles, np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)


def pieces(seqlens, Hkv: int, T_n: int, G: int, order: str = "padded", tail=None):
    """Every (workgroup, output tile) overlap, in iteration order.

    One dict per piece: cta, tile, b, h, local_iter, local_iter_end (iterations within the tile),
    host (the piece holds the tile's first iteration), finishing (it holds the last),
    first_cta / last_cta (the workgroups of the tile's first and last piece)."""
    tiles, t_edges = tile_edges(seqlens, Hkv, T_n, order)
    s_edges = span_edges(int(t_edges[-1]), G, tail)
    cuts = np.union1d(t_edges, s_edges)
    out = []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        cta = int(np.searchsorted(s_edges, lo, side="right")) - 1
        tile = int(np.searchsorted(t_edges, lo, side="right")) - 1     # skips tiles of zero length
        t_lo, t_hi = int(t_edges[tile]), int(t_edges[tile + 1])
        assert s_edges[cta] <= lo and hi <= s_edges[cta + 1] and t_lo <= lo and hi <= t_hi
        b, h = tiles[tile]
        out.append(dict(cta=cta, tile=tile, b=b, h=h, local_iter=int(lo) - t_lo, local_iter_end=int(hi) - t_lo,
                        host=int(lo) == t_lo, finishing=int(hi) == t_hi,
                        first_cta=int(np.searchsorted(s_edges, t_lo, side="right")) - 1,
                        last_cta=int(np.searchsorted(s_edges, t_hi - 1, side="right")) - 1))
    return out


def check_invariants(work, seqlens, Hkv: int, T_n: int):
    """What makes one partial slot per workgroup and one reducer per tile sufficient."""
    per_tile, per_cta = {}, {}
    for p in work:
        per_tile.setdefault((p["b"], p["h"]), []).append(p)
        per_cta.setdefault(p["cta"], []).append(p)
    for (b, h), ps in per_tile.items():
        c_n = math.ceil(seqlens[b] / T_n)
        # the pieces tile the tile's iterations without gap or overlap, in workgroup order
        assert ps[0]["local_iter"] == 0 and ps[-1]["local_iter_end"] == c_n
        assert all(a["local_iter_end"] == c["local_iter"] and a["cta"] + 1 == c["cta"] for a, c in zip(ps, ps[1:]))
        assert sum(p["host"] for p in ps) == 1 and sum(p["finishing"] for p in ps) == 1
        assert ps[0]["host"] and ps[-1]["finishing"]
        assert all(p["first_cta"] == ps[0]["cta"] and p["last_cta"] == ps[-1]["cta"] for p in ps)
    tiles_with_work = {(b, h) for b in range(len(seqlens)) for h in range(Hkv) if seqlens[b] > 0}
    assert set(per_tile) == tiles_with_work
    for cta, ps in per_cta.items():
        # only a workgroup's first piece can begin inside a tile: at most one partial to hand over
        assert sum(not p["host"] for p in ps) <= 1 and all(p["host"] for p in ps[1:])
        # and only its last piece can end inside one
        assert all(p["finishing"] for p in ps[:-1])


def attention_by_spans(q, k, v, seqlens, *, Hkv: int, T_n: int, G: int, scale: float, rng=None, trace=None):
    """Decode attention over a padded cache, computed piece by piece and folded with ``f``.

    q [B,Hq,D]; k, v [B,Hkv,Nmax,D]; returns (out[B,Hq,D], lse[B,Hq]).  With ``rng`` the pieces of a
    tile are folded in a random order and bracketing instead of left to right.
    ``trace`` (a list) receives the pieces."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, Hq, D = q.shape
    group = Hq // Hkv
    work = pieces(seqlens, Hkv, T_n, G, "padded")
    check_invariants(work, seqlens, Hkv, T_n)
    if trace is not None:
        trace.extend(work)
    out = np.zeros((B, Hq, D), dtype=np.float64)
    lse = np.full((B, Hq), -np.inf, dtype=np.float64)
    by_tile = {}
    for p in work:
        by_tile.setdefault((p["b"], p["h"]), []).append(p)
    for (b, h), ps in by_tile.items():
        for row in range(h * group, (h + 1) * group):
            parts = []
            for p in ps:
                lo, hi = p["local_iter"] * T_n, min(p["local_iter_end"] * T_n, seqlens[b])
                parts.append(rescale.partial(q[b, row], k[b, h, lo:hi], v[b, h, lo:hi], scale))
            while len(parts) > 1:     # fold two neighbours (any bracketing) or, with rng, any two
                if rng is None:
                    i, j = 0, 1
                else:
                    i, j = sorted(rng.choice(len(parts), size=2, replace=False))
                merged = rescale.f(parts[i], parts[j])
                parts = [x for n, x in enumerate(parts) if n not in (i, j)] + [merged]
            out[b, row], lse[b, row] = rescale.finalize(parts[0])
    return out, lse
