"""CPU oracle for Dynamic Block-Sparse Attention -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It shares no code with the HIP library and never calls it.

What it computes is the plain definition: dense masked softmax attention in
fp64, where the mask is evaluated per (query row, key) pair from the paper's
statement of the attention pattern:

* Stage 1 (Sec. 2.1): a demonstration group attends (1) the anchor/sink,
  (2) a fixed number ``w`` of preceding groups, (3) itself causally.  Here
  the sink is a token prefix ``[0, S)`` and groups are runs of whole
  demonstrations; inside a group a token sees the earlier demonstrations of
  the group and, causally, its own demonstration.
* Stage 2 (Sec. 2.2): the KV of the selected groups is concatenated behind
  the sink; the test query attends all of it and itself causally, then the
  answer is generated token by token against the same keys.

There is no tiling, no online softmax and no skipping here: every row scores
ALL candidate keys, masked ones get -inf, one softmax, one weighted sum.
numpy's matmul is the only library primitive used.  Rows are independent, so
callers may ask for any subset of rows.

Inputs are fp64 arrays holding the already-rounded bf16/fp32 values, token
major ``[tokens, heads, D]``.  Every function is pinned by tests that do not
go through this module's own formulas (textbook causal attention, closed-form
counts, brute force, the paper's worked example); nothing is "parity unpinned".
"""
from __future__ import annotations

from typing import Iterable, Optional, Sequence, Tuple

import numpy as np

# ---------------------------------------------------------------------------
# token -> demonstration / group maps
# ---------------------------------------------------------------------------


def token_maps(sink_len: int, demo_offsets: np.ndarray, group_demo_offsets: np.ndarray):
    """demo_of[t], group_of[t] for every token t in [0, N); -1 for sink tokens."""
    demo_offsets = np.asarray(demo_offsets, dtype=np.int64)
    group_demo_offsets = np.asarray(group_demo_offsets, dtype=np.int64)
    n = int(demo_offsets[-1])
    assert int(demo_offsets[0]) == sink_len
    demo_of = np.full(n, -1, dtype=np.int64)
    group_of = np.full(n, -1, dtype=np.int64)
    for d in range(len(demo_offsets) - 1):
        demo_of[demo_offsets[d]:demo_offsets[d + 1]] = d
    for g in range(len(group_demo_offsets) - 1):
        lo = demo_offsets[group_demo_offsets[g]]
        hi = demo_offsets[group_demo_offsets[g + 1]]
        group_of[lo:hi] = g
    return demo_of, group_of


# ---------------------------------------------------------------------------
# mask predicates (Sec. 2.1 items (1)-(3); Sec. 2.2)
# ---------------------------------------------------------------------------


def visible_pre(i: int, j: int, sink_len: int, demo_of, group_of, prev_window: int = 0) -> bool:
    """Stage-1 visibility of key j for row i, one pair at a time."""
    if i < sink_len:                       # the anchor is encoded causally with itself
        return j <= i
    if j < sink_len:                       # (1) anchor / sink
        return True
    gi, gj = group_of[i], group_of[j]
    if gj == gi and demo_of[j] < demo_of[i]:           # (3) earlier demonstrations of the own group
        return True
    if demo_of[j] == demo_of[i] and j <= i:            # (3) causal inside the own demonstration
        return True
    if gi - prev_window <= gj < gi:                    # (2) preceding groups
        return True
    return False


def mask_pre(rows: np.ndarray, sink_len: int, demo_of: np.ndarray, group_of: np.ndarray,
             prev_window: int = 0) -> np.ndarray:
    """bool [len(rows), N]: the same predicate as ``visible_pre`` for whole rows."""
    rows = np.asarray(rows, dtype=np.int64)
    n = len(demo_of)
    j = np.arange(n, dtype=np.int64)[None, :]
    i = rows[:, None]
    di, gi = demo_of[rows][:, None], group_of[rows][:, None]
    dj, gj = demo_of[None, :], group_of[None, :]
    j_sink = j < sink_len
    sink_row = i < sink_len
    clause_sink = j_sink
    clause_group = (~j_sink) & (gj == gi) & (dj < di)
    clause_self = (~j_sink) & (dj == di) & (j <= i)
    clause_prev = (~j_sink) & (gi - prev_window <= gj) & (gj < gi)
    pool_rows = clause_sink | clause_group | clause_self | clause_prev
    return np.where(sink_row, j <= i, pool_rows)


def mask_query_pool(selected: Iterable[int], sink_len: int, group_of: np.ndarray) -> np.ndarray:
    """bool [N]: pool key j is visible to a query iff it is a sink token or its
    group is among the query's selected groups (Sec. 2.2)."""
    sel = np.zeros(int(group_of.max()) + 2, dtype=bool)
    for g in selected:
        sel[int(g)] = True
    j = np.arange(len(group_of))
    vis = j < sink_len
    pool = ~vis
    vis[pool] = sel[group_of[pool]]
    return vis


# ---------------------------------------------------------------------------
# dense masked softmax attention
# ---------------------------------------------------------------------------


def masked_softmax_attend(q: np.ndarray, k: np.ndarray, v: np.ndarray, mask: np.ndarray, scale: float,
                          return_probs: bool = False):
    """q [R, D], k [n, D], v [n, Dv], mask bool [R, n] -> O [R, Dv] (and P [R, n]).

    s = scale * q k^T ; masked -> -inf ; p = softmax(s) ; O = p v.
    """
    s = scale * (q @ k.T)
    s = np.where(mask, s, -np.inf)
    m = s.max(axis=1, keepdims=True)
    assert np.all(np.isfinite(m)), "a row with no visible key"
    e = np.exp(s - m)
    l = e.sum(axis=1, keepdims=True)
    p = e / l
    o = p @ v
    if return_probs:
        return o, p
    return o


def log_sum_exp(q: np.ndarray, k: np.ndarray, mask: np.ndarray, scale: float) -> np.ndarray:
    """Natural-log softmax denominator per row: log sum_j exp(scale q.k_j)."""
    s = np.where(mask, scale * (q @ k.T), -np.inf)
    m = s.max(axis=1)
    return m + np.log(np.exp(s - m[:, None]).sum(axis=1))


def _row_chunks(n_rows: int, n_keys: int, budget_elems: int = 24_000_000):
    step = max(1, budget_elems // max(1, n_keys))
    for r0 in range(0, n_rows, step):
        yield r0, min(n_rows, r0 + step)


# ---------------------------------------------------------------------------
# Stage 1: pre-encoding (Sec. 2.1)
# ---------------------------------------------------------------------------


def preencode_attn(q: np.ndarray, k: np.ndarray, v: np.ndarray, sink_len: int, demo_offsets, group_demo_offsets,
                   scale: float, prev_window: int = 0, rows: Optional[np.ndarray] = None,
                   return_lse: bool = False):
    """O[rows, Hq, D] for the stage-1 pattern.  q [N, Hq, D]; k, v [N, Hkv, D]."""
    n, hq, d = q.shape
    hkv = k.shape[1]
    assert hq % hkv == 0
    r = hq // hkv
    demo_of, group_of = token_maps(sink_len, demo_offsets, group_demo_offsets)
    assert len(demo_of) == n
    rows = np.arange(n, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    out = np.empty((len(rows), hq, d), dtype=np.float64)
    lse = np.empty((hq, len(rows)), dtype=np.float64)
    kh = np.ascontiguousarray(np.swapaxes(k, 0, 1))   # [Hkv, N, D], a plain copy for contiguous matmul operands
    vh = np.ascontiguousarray(np.swapaxes(v, 0, 1))
    for a, b in _row_chunks(len(rows), n):
        m = mask_pre(rows[a:b], sink_len, demo_of, group_of, prev_window)
        for h in range(hq):
            kk, vv = kh[h // r], vh[h // r]
            out[a:b, h, :] = masked_softmax_attend(q[rows[a:b], h, :], kk, vv, m, scale)
            if return_lse:
                lse[h, a:b] = log_sum_exp(q[rows[a:b], h, :], kk, m, scale)
    return (out, lse) if return_lse else out


# ---------------------------------------------------------------------------
# Stage 2: query prefill and decode (Sec. 2.2)
# ---------------------------------------------------------------------------


def _query_selected(sel_ptr, sel_idx, u: int) -> np.ndarray:
    return np.asarray(sel_idx[int(sel_ptr[u]):int(sel_ptr[u + 1])], dtype=np.int64)


def query_attn(q_self: np.ndarray, k_self: np.ndarray, v_self: np.ndarray, k_pool: np.ndarray, v_pool: np.ndarray,
               sink_len: int, demo_offsets, group_demo_offsets, cu_qlens, sel_ptr, sel_idx, scale: float,
               queries: Optional[Sequence[int]] = None) -> np.ndarray:
    """Prefill of the test queries.  Token a of query u attends: every sink key,
    every key of u's selected groups (no mask inside the pool part), and its
    own tokens b <= a.  One softmax over the union.

    Returns O [sum T, Hq, D]; rows of queries not in ``queries`` are NaN.
    """
    tot, hq, d = q_self.shape
    hkv = k_pool.shape[1]
    r = hq // hkv
    n = k_pool.shape[0]
    _, group_of = token_maps(sink_len, demo_offsets, group_demo_offsets)
    out = np.full((tot, hq, d), np.nan, dtype=np.float64)
    n_queries = len(cu_qlens) - 1
    for u in (range(n_queries) if queries is None else queries):
        t0, t1 = int(cu_qlens[u]), int(cu_qlens[u + 1])
        t = t1 - t0
        pool_vis = mask_query_pool(_query_selected(sel_ptr, sel_idx, u), sink_len, group_of)
        a = np.arange(t)
        self_vis = a[None, :] <= a[:, None]                     # b <= a
        mask = np.concatenate([np.broadcast_to(pool_vis, (t, n)), self_vis], axis=1)
        for hk in range(hkv):                                   # candidate keys: [pool ; own tokens]
            kk = np.concatenate([k_pool[:, hk, :], k_self[t0:t1, hk, :]], axis=0)
            vv = np.concatenate([v_pool[:, hk, :], v_self[t0:t1, hk, :]], axis=0)
            for h in range(hk * r, (hk + 1) * r):
                out[t0:t1, h, :] = masked_softmax_attend(q_self[t0:t1, h, :], kk, vv, mask, scale)
    return out


def decode_attn(q_step: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, self_len, k_pool: np.ndarray,
                v_pool: np.ndarray, sink_len: int, demo_offsets, group_demo_offsets, sel_ptr, sel_idx,
                scale: float, queries: Optional[Sequence[int]] = None) -> np.ndarray:
    """One generated token per query.  q_step [B, Hq, D]; caches [B, Tmax, Hkv, D];
    self_len[u] counts the query's own keys including the new token.  The new
    token attends the sink, the selected groups and ALL self keys [0, self_len).
    """
    b, hq, d = q_step.shape
    hkv = k_pool.shape[1]
    r = hq // hkv
    n = k_pool.shape[0]
    t_max = k_cache.shape[1]
    _, group_of = token_maps(sink_len, demo_offsets, group_demo_offsets)
    out = np.full((b, hq, d), np.nan, dtype=np.float64)
    for u in (range(b) if queries is None else queries):
        pool_vis = mask_query_pool(_query_selected(sel_ptr, sel_idx, u), sink_len, group_of)
        self_vis = np.arange(t_max) < int(self_len[u])
        mask = np.concatenate([pool_vis, self_vis])[None, :]
        for hk in range(hkv):                                   # candidate keys: [pool ; own cache]
            kk = np.concatenate([k_pool[:, hk, :], k_cache[u, :, hk, :]], axis=0)
            vv = np.concatenate([v_pool[:, hk, :], v_cache[u, :, hk, :]], axis=0)
            out[u, hk * r:(hk + 1) * r, :] = masked_softmax_attend(q_step[u, hk * r:(hk + 1) * r, :], kk, vv,
                                                                   np.broadcast_to(mask, (r, mask.shape[1])), scale)
    return out


# ---------------------------------------------------------------------------
# split-KV partial state and its merge (the decode second pass)
# ---------------------------------------------------------------------------


def partial_state(q: np.ndarray, k: np.ndarray, v: np.ndarray, scale: float):
    """Softmax state of one query row over one chunk of visible keys:
    m = max_j s_j, l = sum_j exp(s_j - m), acc = sum_j exp(s_j - m) v_j."""
    if k.shape[0] == 0:
        return -np.inf, 0.0, np.zeros(v.shape[1])
    s = scale * (k @ q)
    m = s.max()
    e = np.exp(s - m)
    return m, e.sum(), e @ v


def merge_partials(ms: Sequence[float], ls: Sequence[float], accs: Sequence[np.ndarray]) -> np.ndarray:
    """m* = max_s m_s ; l* = sum_s l_s e^{m_s - m*} ; o = sum_s acc_s e^{m_s - m*} / l*."""
    ms = np.asarray(ms, dtype=np.float64)
    m_star = ms.max()
    wts = np.where(np.isneginf(ms), 0.0, np.exp(ms - m_star))
    l_star = float(np.sum(wts * np.asarray(ls, dtype=np.float64)))
    acc = np.sum(wts[:, None] * np.asarray(accs, dtype=np.float64), axis=0)
    return acc / l_star


# ---------------------------------------------------------------------------
# work accounting (visible pairs; 4*D flops per pair per query head)
# ---------------------------------------------------------------------------


def visible_pairs_pre(sink_len: int, demo_offsets, group_demo_offsets, prev_window: int = 0) -> int:
    """Number of visible (row, key) pairs of the stage-1 mask, by counting the mask."""
    demo_of, group_of = token_maps(sink_len, demo_offsets, group_demo_offsets)
    n = len(demo_of)
    total = 0
    for a, b in _row_chunks(n, n):
        total += int(mask_pre(np.arange(a, b), sink_len, demo_of, group_of, prev_window).sum())
    return total


def visible_pairs_query(sink_len: int, demo_offsets, group_demo_offsets, cu_qlens, sel_ptr, sel_idx) -> int:
    _, group_of = token_maps(sink_len, demo_offsets, group_demo_offsets)
    total = 0
    for u in range(len(cu_qlens) - 1):
        t = int(cu_qlens[u + 1] - cu_qlens[u])
        pool_vis = mask_query_pool(_query_selected(sel_ptr, sel_idx, u), sink_len, group_of)
        a = np.arange(t)
        total += t * int(pool_vis.sum()) + int((a[None, :] <= a[:, None]).sum())
    return total
