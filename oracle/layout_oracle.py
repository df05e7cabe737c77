"""Tile-list oracle for the DBSA block layout -- TEST INFRASTRUCTURE ONLY.

Derives, straight from the visibility predicates of ``dbsa_oracle`` and by
scanning every (Q tile, KV tile) pair, the canonical lists the library's layout
builder must reproduce bit for bit.  No code is shared with that builder.

Canonical form (Sec. 2.1 for the stage-1 pattern, Sec. 2.2 for the query stage):

* Q tiles are cut every ``block_m`` tokens inside a segment and never straddle
  segments.  Stage 1: the sink segment ``[0, S)`` first, then each group from
  its first token.  Query stage: each query's own tokens from its first token.
  A row of the Q-tile table is ``(q_start, q_len, owner, 0)`` with owner = -1
  for the sink, the group index at stage 1, the query index at stage 2.
* KV tiles are cut every ``block_n`` tokens inside a segment (sink, each group,
  each query's self tokens) from the segment's first token.
* A KV tile is listed for a Q tile iff at least one (row, key) pair in it is
  visible.  Its kind is FULL iff every pair is visible, else CAUSAL.  Self
  tiles of the query stage carry the SELF bit.
* Order: ascending ``kv_start`` at stage 1; at stage 2 the sink tiles, then the
  selected groups in the caller's order, then the self tiles.
* An entry is two int32 words: ``kv_start`` and ``kv_len | kind << 16``.
* Decode: per query the pool part of the list (sink + selected groups); split s
  of n covers entries ``[s*L // n, (s+1)*L // n)``.
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np

from . import dbsa_oracle as orc

KIND_FULL = 0
KIND_CAUSAL = 1
KIND_SELF_FULL = 2
KIND_SELF_CAUSAL = 3


def _segments(sink_len, demo_offsets, group_demo_offsets) -> List[Tuple[int, int]]:
    """[(start, end)] of the sink segment and of every group, in token order."""
    gb = np.asarray(demo_offsets)[np.asarray(group_demo_offsets)]
    segs = [(0, int(sink_len))]
    for g in range(len(gb) - 1):
        segs.append((int(gb[g]), int(gb[g + 1])))
    return segs


def _cut(start: int, end: int, step: int) -> List[Tuple[int, int]]:
    return [(a, min(step, end - a)) for a in range(start, end, step)]


def _pack(entries) -> np.ndarray:
    out = np.zeros((len(entries), 2), dtype=np.int32)
    for n, (start, length, kind) in enumerate(entries):
        out[n, 0] = start
        out[n, 1] = length | (kind << 16)
    return out


def preencode_layout(sink_len, demo_offsets, group_demo_offsets, prev_window, block_m, block_n):
    """-> (qtile_tab int32 [n,4], list_ptr int64 [n+1], list_ent int32 [E,2])."""
    demo_of, group_of = orc.token_maps(sink_len, demo_offsets, group_demo_offsets)
    segs = _segments(sink_len, demo_offsets, group_demo_offsets)
    kv_tiles = [t for (a, b) in segs for t in _cut(a, b, block_n)]
    qtab, ptr, ents = [], [0], []
    for owner, (a, b) in enumerate(segs):
        for (q0, qn) in _cut(a, b, block_m):
            m = orc.mask_pre(np.arange(q0, q0 + qn), sink_len, demo_of, group_of, prev_window)
            for (k0, kn) in kv_tiles:                      # ascending kv_start
                sub = m[:, k0:k0 + kn]
                if sub.any():
                    ents.append((k0, kn, KIND_FULL if sub.all() else KIND_CAUSAL))
            qtab.append((q0, qn, owner - 1, 0))
            ptr.append(len(ents))
    return (np.asarray(qtab, dtype=np.int32).reshape(-1, 4), np.asarray(ptr, dtype=np.int64), _pack(ents))


def _pool_entries(u, sink_len, demo_offsets, group_demo_offsets, sel_ptr, sel_idx, block_n, group_of):
    segs = _segments(sink_len, demo_offsets, group_demo_offsets)
    sel = [int(g) for g in sel_idx[int(sel_ptr[u]):int(sel_ptr[u + 1])]]
    vis = orc.mask_query_pool(sel, sink_len, group_of)
    ents = []
    for seg_id in [0] + [g + 1 for g in sel]:              # sink, then the caller's order
        a, b = segs[seg_id]
        for (k0, kn) in _cut(a, b, block_n):
            sub = vis[k0:k0 + kn]
            if sub.any():
                assert sub.all()
                ents.append((k0, kn, KIND_FULL))
    return ents


def query_layout(sink_len, demo_offsets, group_demo_offsets, cu_qlens, sel_ptr, sel_idx, block_m, block_n):
    _, group_of = orc.token_maps(sink_len, demo_offsets, group_demo_offsets)
    qtab, ptr, ents = [], [0], []
    for u in range(len(cu_qlens) - 1):
        t0, t1 = int(cu_qlens[u]), int(cu_qlens[u + 1])
        pool = _pool_entries(u, sink_len, demo_offsets, group_demo_offsets, sel_ptr, sel_idx, block_n, group_of)
        for (q0, qn) in _cut(t0, t1, block_m):
            ents.extend(pool)
            a = np.arange(q0, q0 + qn)[:, None]
            for (k0, kn) in _cut(t0, t1, block_n):
                b = np.arange(k0, k0 + kn)[None, :]
                sub = b <= a
                if sub.any():
                    ents.append((k0, kn, KIND_SELF_FULL if sub.all() else KIND_SELF_CAUSAL))
            qtab.append((q0, qn, u, 0))
            ptr.append(len(ents))
    return (np.asarray(qtab, dtype=np.int32).reshape(-1, 4), np.asarray(ptr, dtype=np.int64), _pack(ents))


def decode_layout(sink_len, demo_offsets, group_demo_offsets, n_queries, sel_ptr, sel_idx, block_n, n_split):
    """-> (dec_ptr int64 [B+1], dec_ent int32 [E,2], split_ptr int64 [B, n_split+1])."""
    _, group_of = orc.token_maps(sink_len, demo_offsets, group_demo_offsets)
    ptr, ents = [0], []
    split = np.zeros((n_queries, n_split + 1), dtype=np.int64)
    for u in range(n_queries):
        pool = _pool_entries(u, sink_len, demo_offsets, group_demo_offsets, sel_ptr, sel_idx, block_n, group_of)
        base = len(ents)
        ents.extend(pool)
        ptr.append(len(ents))
        for s in range(n_split + 1):
            split[u, s] = base + (s * len(pool)) // n_split
    return np.asarray(ptr, dtype=np.int64), _pack(ents), split


def decode_group_schedule(sink_len, demo_offsets, group_demo_offsets, n_queries, sel_ptr, sel_idx, block_n,
                          chunk_tiles, item_queries=32):
    """Group-major decode schedule derived from the visibility predicate: a segment (the
    sink, a group) is used by the queries that see its keys; the t KV tiles of a used segment are
    cut into ceil(t / chunk_tiles) runs of equal length to within one tile (run i = tiles
    [i t / n, (i+1) t / n)), and every run is one item per batch of ``item_queries`` users
    (ascending query order); every (item, user) pair takes the user's next slot; a query's last slot is for
    its own cached keys.  -> dict like the library's export."""
    _, group_of = orc.token_maps(sink_len, demo_offsets, group_demo_offsets)
    segs = _segments(sink_len, demo_offsets, group_demo_offsets)
    vis = [orc.mask_query_pool([int(g) for g in sel_idx[int(sel_ptr[u]):int(sel_ptr[u + 1])]], sink_len, group_of)
           for u in range(n_queries)]
    seg_ptr, seg_ent = [0], []
    for (a, b) in segs:
        seg_ent.extend((k0, kn, KIND_FULL) for (k0, kn) in _cut(a, b, block_n))
        seg_ptr.append(len(seg_ent))
    uses, counts = [], np.zeros(n_queries, dtype=np.int64)
    for s, (a, b) in enumerate(segs):
        users = [u for u in range(n_queries) if b > a and vis[u][a:b].any()]
        for u in users:
            assert vis[u][a:b].all()
        t0, t = seg_ptr[s], seg_ptr[s + 1] - seg_ptr[s]
        n_runs = -(-t // chunk_tiles)
        for run in range(n_runs):
            c0, c1 = t0 + (run * t) // n_runs, t0 + ((run + 1) * t) // n_runs
            cn = c1 - c0
            for b0 in range(0, len(users), item_queries):
                uses.append((c0, cn, users[b0:b0 + item_queries]))
                for u in users[b0:b0 + item_queries]:
                    counts[u] += 1
    slot_ptr = np.concatenate([[0], np.cumsum(counts + 1)]).astype(np.int64)
    nxt = np.zeros(n_queries, dtype=np.int64)
    items, qrefs = [], []
    for (c0, cn, users) in uses:
        items.append((c0, cn, len(qrefs), len(users)))
        for u in users:
            qrefs.append((u, int(slot_ptr[u] + nxt[u])))
            nxt[u] += 1
    return dict(seg_ptr=np.asarray(seg_ptr, np.int64), seg_ent=_pack(seg_ent),
                items=np.asarray(items, np.int32).reshape(-1, 4), qrefs=np.asarray(qrefs, np.int32).reshape(-1, 2),
                slot_ptr=slot_ptr)


def position_shifts(sink_len, demo_offsets, group_demo_offsets, cu_qlens, sel_ptr, sel_idx, qtile_tab, list_ptr,
                    list_ent, seg_ent, items, qrefs):
    """Re-positioning data (Sec. 2.2), derived from the new position ids themselves: the
    concatenated cache of query u lists its pool tokens in order and the i-th of them gets id i.
    A list entry (or schedule item) whose first key moves from id j to id j' has displacement
    j' - j; a query row at new id ``cache_len + a`` is rotated at ``cache_len + a - (j' - j)``
    instead.  Returns (list_shift parallel to ``list_ent`` with the tile's first local row
    index folded in, qref_shift parallel to ``qrefs``, cache_len [B])."""
    from . import rope_oracle as ro
    n_queries = len(cu_qlens) - 1
    new_id, cache_len = [], []
    for u in range(n_queries):
        ids = ro.selected_token_ids(sink_len, demo_offsets, group_demo_offsets,
                                    sel_idx[int(sel_ptr[u]):int(sel_ptr[u + 1])])
        new_id.append({int(j): i for i, j in enumerate(ids)})
        cache_len.append(len(ids))
    list_shift = np.zeros(len(list_ent), dtype=np.int32)
    for t in range(len(qtile_tab)):
        q0, _, u, _ = (int(x) for x in qtile_tab[t])
        a0 = q0 - int(cu_qlens[u])
        for e in range(int(list_ptr[t]), int(list_ptr[t + 1])):
            j, kind = int(list_ent[e, 0]), int(list_ent[e, 1]) >> 16
            if kind in (KIND_SELF_FULL, KIND_SELF_CAUSAL):
                list_shift[e] = a0                                  # own keys keep their local ids
            else:
                list_shift[e] = cache_len[u] - (new_id[u][j] - j) + a0
    qref_shift = np.zeros(len(qrefs), dtype=np.int32)
    for (ent_begin, _, ref_begin, n_q) in (tuple(int(x) for x in it) for it in items):
        j = int(seg_ent[ent_begin, 0])
        for ref in range(ref_begin, ref_begin + n_q):
            u = int(qrefs[ref, 0])
            qref_shift[ref] = cache_len[u] - (new_id[u][j] - j)
    return list_shift, qref_shift, np.asarray(cache_len, dtype=np.int32)

