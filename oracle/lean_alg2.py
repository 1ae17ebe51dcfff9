"""TEST INFRASTRUCTURE -- Algorithms 1 and 2 of the paper, step by step, in
fp64 numpy, with the CTAs of the grid emulated one after another.

This is not the oracle of the result (that is ``exact_attention.c``); it pins
the *bookkeeping* of the stream-K walk: spans, host / finishing predicates,
one workspace slot per CTA, the range of peers a host waits for.  Its output
must equal the exact definition for every grid size and tile size.

Readings taken where the printed algorithms are silent or garbled:
  * the score is scaled by ``scale`` before max/exp (Eq. 1 has 1/sqrt(d), the
    algorithms drop it);
  * iteration ranges are half open;
  * the total iteration count sums C_n over every output tile (batch x KV head),
    as the TilesPerCTA equation of Section 4.3 does, not just C_m * C_n;
  * when I is not a multiple of G the first I mod G CTAs take one extra
    iteration, and G is clipped to I;
  * ``last_cta`` is the CTA whose span holds the tile's last iteration;
  * with ragged lengths ``tile_idx`` comes from a prefix table of per-tile C_n;
  * tokens past N_b in the tail tile score -inf;
  * a query group sharing one KV head forms the T_m rows of Q_f (the paper has
    no GQA; with Hq == Hkv, T_m = 1).
CTAs are run from the highest id down so that the partials a host waits for
already exist; ``Wait`` then only asserts the flag.
"""
from __future__ import annotations

import math

import numpy as np


def lean_tile(q_rows, k_ctx, v_ctx, n_ctx, iter_begin, iter_end, T_n, scale):
    """Algorithm 1: online softmax over LeanTile iterations [iter_begin, iter_end).

    q_rows [T_m, D]; k_ctx, v_ctx [>=n_ctx, D].  Returns (O_acc[T_m,D], m[T_m], l[T_m]).
    """
    T_m, D = q_rows.shape
    O_acc = np.zeros((T_m, D), dtype=np.float64)
    m = np.full(T_m, -np.inf, dtype=np.float64)
    l = np.zeros(T_m, dtype=np.float64)
    for it in range(iter_begin, iter_end):
        kk = it * T_n
        hi = min(kk + T_n, n_ctx)
        K_f = k_ctx[kk:hi]
        V_f = v_ctx[kk:hi]
        S_f = scale * (q_rows @ K_f.T)                       # [T_m, tokens]
        m_new = np.maximum(m, S_f.max(axis=1))
        P_f = np.exp(S_f - m_new[:, None])
        alpha = np.where(np.isneginf(m), 0.0, np.exp(m - m_new))
        l = alpha * l + P_f.sum(axis=1)
        O_acc = P_f @ V_f + alpha[:, None] * O_acc
        m = m_new
    return O_acc, m, l


def spans(total_iters: int, G: int):
    """Equal contiguous spans: [(cta_start, cta_end)] for g in range(G')."""
    G = max(1, min(G, total_iters)) if total_iters > 0 else 0
    out = []
    if G == 0:
        return out
    base, extra = divmod(total_iters, G)
    start = 0
    for g in range(G):
        n = base + (1 if g < extra else 0)
        out.append((start, start + n))
        start += n
    assert start == total_iters
    return out


def lean_attention(q, k, v, seqlens, *, Hkv, T_n, G, scale, trace=None):
    """Algorithm 2 over a padded cache.

    q [B,Hq,D]; k, v [B,Hkv,Nmax,D]; returns (out[B,Hq,D], lse[B,Hq]).
    ``trace`` (a list) receives one dict per (CTA, output-tile segment).
    """
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    B, Hq, D = q.shape
    T_m = Hq // Hkv
    # output tiles in batch -> head order, with their iteration counts
    tiles = [(b, h) for b in range(B) for h in range(Hkv)]
    C_n = [math.ceil(seqlens[b] / T_n) for (b, _h) in tiles]
    tile_iter0 = np.concatenate([[0], np.cumsum(C_n)]).astype(np.int64)
    I = int(tile_iter0[-1])
    out = np.zeros((B, Hq, D), dtype=np.float64)
    lse = np.full((B, Hq), -np.inf, dtype=np.float64)
    cta_span = spans(I, G)
    G_eff = len(cta_span)
    Op = [None] * G_eff
    mp = [None] * G_eff
    lp = [None] * G_eff
    flags = [0] * G_eff

    def cta_of_iter(it):
        for c, (s, e) in enumerate(cta_span):
            if s <= it < e:
                return c
        raise AssertionError("iteration outside every span")

    for g in reversed(range(G_eff)):
        cta_start, cta_end = cta_span[g]
        it = cta_start
        stored = 0
        while it < cta_end:
            tile_idx = int(np.searchsorted(tile_iter0, it, side="right") - 1)
            tile_iter = int(tile_iter0[tile_idx])
            tile_iter_end = int(tile_iter0[tile_idx + 1])
            local_iter = it - tile_iter
            local_iter_end = min(tile_iter_end, cta_end) - tile_iter
            b, h = tiles[tile_idx]
            rows = slice(h * T_m, (h + 1) * T_m)
            O, m, l = lean_tile(q[b, rows], k[b, h], v[b, h], seqlens[b], local_iter, local_iter_end,
                                T_n, scale)
            host_block = it == tile_iter
            finishing_block = cta_end >= tile_iter_end
            if trace is not None:
                trace.append(dict(cta=g, tile=tile_idx, b=b, h=h, local_iter=local_iter,
                                  local_iter_end=local_iter_end, host=host_block,
                                  finishing=finishing_block))
            if not host_block:
                stored += 1
                assert stored == 1, "a CTA stores at most one partial: one slot per CTA suffices"
                Op[g], mp[g], lp[g] = O, m, l
                flags[g] = 1
            else:
                if not finishing_block:
                    last_cta = cta_of_iter(tile_iter_end - 1)
                    for cta in range(g + 1, last_cta + 1):
                        assert flags[cta] == 1, "Wait(flags[cta]) would never return"
                        m_cta, l_cta, O_cta = mp[cta], lp[cta], Op[cta]
                        m_new = np.maximum(m_cta, m)
                        w_cta = np.where(np.isneginf(m_cta), 0.0, np.exp(m_cta - m_new))
                        w_own = np.where(np.isneginf(m), 0.0, np.exp(m - m_new))
                        l = w_cta * l_cta + w_own * l
                        O = w_cta[:, None] * O_cta + w_own[:, None] * O
                        m = m_new
                out[b, rows] = O / l[:, None]
                lse[b, rows] = m + np.log(l)
            it = tile_iter_end
    return out, lse
