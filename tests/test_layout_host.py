"""Host block-layout builder vs the tile-list oracle (bit-exact), error codes, and
that the C-ABI library exports what include/dbsa.h declares.  CPU only: layouts
are built with DBSA_LAYOUT_HOST_ONLY, no GPU call is made."""
import os
import re

import numpy as np
import pytest

from oracle import dbsa_oracle as orc
from oracle import layout_oracle as lo
from paper_2503_08640_amd import binding as B
from paper_2503_08640_amd import synth


def rand_pool(rng, sink_len, n_groups, demos_per_group=(1, 4), demo_len=(1, 9)):
    lens, gdo = [], [0]
    for _ in range(n_groups):
        nd = int(rng.integers(demos_per_group[0], demos_per_group[1] + 1))
        lens += [int(rng.integers(demo_len[0], demo_len[1] + 1)) for _ in range(nd)]
        gdo.append(len(lens))
    offs = sink_len + np.concatenate([[0], np.cumsum(lens)])
    return synth.Pool(sink_len, offs.astype(np.int32), np.asarray(gdo, np.int32))


def assert_same_lists(got, want):
    for g, w, name in zip(got, want, ("qtile_tab", "list_ptr", "list_ent")):
        assert g.dtype == w.dtype, name
        assert g.shape == w.shape, (name, g.shape, w.shape)
        assert np.array_equal(g, w), name


def test_library_exports_every_declared_symbol():
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    header = open(os.path.join(root, "include", "dbsa.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(dbsa_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTED_SYMBOLS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert B.strerror(B.DBSA_OK) == "ok"
    assert "workspace" in B.strerror(B.DBSA_ERR_WORKSPACE)


@pytest.mark.parametrize("seed", range(8))
def test_preencode_lists_match_oracle_on_random_pools(seed):
    rng = np.random.default_rng(seed)
    pool = rand_pool(rng, sink_len=int(rng.integers(0, 12)), n_groups=int(rng.integers(1, 6)))
    w = int(rng.integers(0, 3))
    bm, bn = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    lay = B.dbsa_layout_build(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, w, block_m=bm, block_n=bn,
                              host_only=True)
    assert_same_lists(lay.export(), lo.preencode_layout(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets,
                                                        w, bm, bn))
    order = lay.export_order()
    tab, ptr, _ = lay.export()
    assert sorted(order.tolist()) == list(range(len(tab)))
    owners, lens = tab[order, 2], np.diff(ptr)[order]
    assert np.all(np.diff(owners) >= 0)                      # owner by owner
    same = owners[:-1] == owners[1:]
    assert np.all(lens[:-1][same] >= lens[1:][same])         # longest list of an owner first


@pytest.mark.parametrize("seed", range(8))
def test_repositioning_shifts_match_the_new_position_ids(seed):
    rng = np.random.default_rng(300 + seed)
    pool = rand_pool(rng, sink_len=int(rng.integers(0, 7)), n_groups=int(rng.integers(1, 7)))
    nq = int(rng.integers(1, 6))
    qlens = rng.integers(1, 12, size=nq)
    cu = np.concatenate([[0], np.cumsum(qlens)]).astype(np.int32)
    sels = [rng.permutation(pool.n_groups)[:int(rng.integers(0, pool.n_groups + 1))] for _ in range(nq)]
    sel_ptr = np.concatenate([[0], np.cumsum([len(s) for s in sels])]).astype(np.int32)
    sel_idx = np.concatenate(sels).astype(np.int32) if sel_ptr[-1] else np.zeros(0, np.int32)
    bm, bn = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    lay = B.dbsa_layout_build(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, cu_qlens=cu, sel_ptr=sel_ptr,
                              sel_idx=sel_idx, n_split=int(rng.integers(0, 4)), block_m=bm, block_n=bn, host_only=True)
    tab, ptr, ent = lay.export()
    g = lay.export_decode_groups(pool.n_groups, nq)
    got = lay.export_positions(nq)
    want = lo.position_shifts(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, cu, sel_ptr, sel_idx, tab, ptr,
                              ent, g["seg_ent"], g["items"], g["qrefs"])
    for a, b, name in zip(got, want, ("list_shift", "qref_shift", "cache_len")):
        assert a.dtype == b.dtype and np.array_equal(a, b), name
    assert np.all(got[0] >= 0) and np.all(got[1] >= 0)


def _arena_pages(rng, pool, needed):
    """Scatter the sink and the groups in ``needed`` over an arena with gaps, in random order;
    other groups are resident or not at random.  -> page_start [G+1]."""
    gb = pool.group_token_bounds()
    lens = [pool.sink_len] + [int(gb[g + 1] - gb[g]) for g in range(pool.n_groups)]
    resident = [s for s in range(pool.n_groups + 1) if s == 0 or (s - 1) in needed or rng.random() < 0.5]
    page_start = np.full(pool.n_groups + 1, -1, dtype=np.int32)
    at = int(rng.integers(0, 5))
    for s in rng.permutation(resident):
        page_start[s] = at
        at += lens[s] + int(rng.integers(0, 7))
    return page_start


@pytest.mark.parametrize("seed", range(8))
def test_paged_layout_names_arena_rows_and_keeps_positions(seed):
    """Sec. 4 (storage cost): groups may be offloaded or re-encoded; the query stage only needs
    the selected ones, wherever they sit."""
    rng = np.random.default_rng(400 + seed)
    pool = rand_pool(rng, sink_len=int(rng.integers(0, 7)), n_groups=int(rng.integers(1, 7)))
    nq = int(rng.integers(1, 5))
    cu = np.concatenate([[0], np.cumsum(rng.integers(1, 12, size=nq))]).astype(np.int32)
    sels = [rng.permutation(pool.n_groups)[:int(rng.integers(0, pool.n_groups + 1))] for _ in range(nq)]
    sel_ptr = np.concatenate([[0], np.cumsum([len(s) for s in sels])]).astype(np.int32)
    sel_idx = np.concatenate(sels).astype(np.int32) if sel_ptr[-1] else np.zeros(0, np.int32)
    bm, bn = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    page_start = _arena_pages(rng, pool, set(int(g) for g in sel_idx))
    kw = dict(cu_qlens=cu, sel_ptr=sel_ptr, sel_idx=sel_idx, n_split=2, block_m=bm, block_n=bn, host_only=True)
    plain = B.dbsa_layout_build(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, **kw)
    paged = B.dbsa_layout_build(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, page_start=page_start, **kw)
    gb = pool.group_token_bounds()
    seg_lo = np.concatenate([[0], gb[:-1]]).astype(np.int64)        # logical first token of sink, groups

    def to_arena(ent, self_kinds=True):
        out = ent.copy()
        for i in range(len(ent)):
            if self_kinds and (int(ent[i, 1]) >> 16) >= lo.KIND_SELF_FULL:
                continue                                             # a query's own tokens are not paged
            j = int(ent[i, 0])
            s = 0 if j < pool.sink_len else 1 + int(np.searchsorted(gb, j, side="right") - 1)
            out[i, 0] = page_start[s] + (j - seg_lo[s])
        return out

    tab, ptr, ent = plain.export()
    assert_same_lists(paged.export(), (tab, ptr, to_arena(ent)))
    dp, de, sp = plain.export_decode(nq)
    dp2, de2, sp2 = paged.export_decode(nq)
    assert np.array_equal(dp, dp2) and np.array_equal(sp, sp2) and np.array_equal(de2, to_arena(de, False))
    g1, g2 = plain.export_decode_groups(pool.n_groups, nq), paged.export_decode_groups(pool.n_groups, nq)
    for key in ("seg_ptr", "items", "qrefs", "slot_ptr"):
        assert np.array_equal(g1[key], g2[key]), key
    used = np.unique(np.concatenate([np.arange(int(a), int(a) + int(n)) for a, n in g1["items"][:, :2]] + [[]]))
    used = used.astype(np.int64)
    assert np.array_equal(g2["seg_ent"][used], to_arena(g1["seg_ent"][used], False))
    for a, b in zip(plain.export_positions(nq), paged.export_positions(nq)):
        assert np.array_equal(a, b)                                  # positions are about token ids, not rows
    if sel_ptr[-1]:
        gone = page_start.copy()
        gone[int(sel_idx[0]) + 1] = -1
        with pytest.raises(B.DbsaError) as ei:
            B.dbsa_layout_build(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, page_start=gone, **kw)
        assert ei.value.code == B.DBSA_ERR_BAD_SELECTION
    res = np.nonzero(page_start >= 0)[0]
    if len(res) >= 2:
        clash = page_start.copy()
        clash[res[1]] = clash[res[0]]
        lens = [pool.sink_len] + [int(gb[g + 1] - gb[g]) for g in range(pool.n_groups)]
        if lens[res[0]] > 0 and lens[res[1]] > 0:
            with pytest.raises(B.DbsaError) as ei:
                B.dbsa_layout_build(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, page_start=clash, **kw)
            assert ei.value.code == B.DBSA_ERR_BAD_BOUNDS


@pytest.mark.parametrize("seed", range(6))
def test_append_layout_is_the_tail_of_the_full_layout(seed):
    """Sec. 2.1: an added group attends the anchor, its window and itself, and nothing encoded
    earlier attends it: its Q tiles and lists are those of the full pre-encode layout."""
    rng = np.random.default_rng(200 + seed)
    pool = rand_pool(rng, sink_len=int(rng.integers(0, 12)), n_groups=int(rng.integers(2, 7)))
    w = int(rng.integers(0, 3))
    bm, bn = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    g0 = int(rng.integers(0, pool.n_groups))
    lay = B.dbsa_layout_build_append(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, w, g0, block_m=bm,
                                     block_n=bn, host_only=True)
    tab, ptr, ent = lo.preencode_layout(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, w, bm, bn)
    keep = np.nonzero(tab[:, 2] >= g0)[0]
    assert len(keep) > 0 and np.array_equal(keep, np.arange(keep[0], len(tab)))   # a suffix of the tile table
    e0 = ptr[keep[0]]
    assert_same_lists(lay.export(), (tab[keep], ptr[keep[0]:] - e0, ent[e0:]))
    # the oracle's predicate says the same thing: no row before the new groups sees a key inside them
    first_new = int(pool.group_token_bounds()[g0])
    demo_of, group_of = orc.token_maps(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets)
    vis = orc.mask_pre(np.arange(first_new), pool.sink_len, demo_of, group_of, w)
    assert not vis[:, first_new:].any()
    for bad in (-1, pool.n_groups):
        with pytest.raises(B.DbsaError):
            B.dbsa_layout_build_append(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, w, bad, block_m=bm,
                                       block_n=bn, host_only=True)


@pytest.mark.parametrize("seed", range(8))
def test_query_and_decode_lists_match_oracle_on_random_inputs(seed):
    rng = np.random.default_rng(50 + seed)
    pool = rand_pool(rng, sink_len=int(rng.integers(0, 7)), n_groups=int(rng.integers(1, 7)))
    nq = int(rng.integers(1, 5))
    qlens = rng.integers(1, 12, size=nq)
    cu = np.concatenate([[0], np.cumsum(qlens)]).astype(np.int32)
    sels = [rng.permutation(pool.n_groups)[:int(rng.integers(0, pool.n_groups + 1))] for _ in range(nq)]
    sel_ptr = np.concatenate([[0], np.cumsum([len(s) for s in sels])]).astype(np.int32)
    sel_idx = np.concatenate(sels).astype(np.int32) if sel_ptr[-1] else np.zeros(0, np.int32)
    bm, bn, ns = int(rng.integers(1, 7)), int(rng.integers(1, 7)), int(rng.integers(1, 5))
    lay = B.dbsa_layout_build(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, cu_qlens=cu,
                              sel_ptr=sel_ptr, sel_idx=sel_idx, n_split=ns, block_m=bm, block_n=bn, host_only=True)
    assert_same_lists(lay.export(), lo.query_layout(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, cu,
                                                    sel_ptr, sel_idx, bm, bn))
    dec_ptr, dec_ent, split = lay.export_decode(nq)
    o_ptr, o_ent, o_split = lo.decode_layout(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, nq, sel_ptr,
                                             sel_idx, bn, ns)
    assert np.array_equal(dec_ptr, o_ptr) and np.array_equal(dec_ent, o_ent) and np.array_equal(split, o_split)
    got = lay.export_decode_groups(pool.n_groups, nq)
    segs = np.diff(got["seg_ptr"])
    used = [0] * (pool.sink_len > 0) + [int(g) + 1 for g in set(sel_idx.tolist())]
    longest = max([int(segs[s]) for s in used] + [1])
    assert got["chunk_tiles"] == max(1, -(-longest // ns))               # ceil(longest used segment / n_split)
    want = lo.decode_group_schedule(pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, nq, sel_ptr, sel_idx,
                                    bn, got["chunk_tiles"])
    for key in ("seg_ptr", "seg_ent", "items", "qrefs", "slot_ptr"):
        assert got[key].dtype == want[key].dtype and np.array_equal(got[key], want[key]), key
    # what any valid schedule must satisfy, whatever the cutting rule: every (used segment, user)
    # pair sees each tile of the segment exactly once, runs stay inside a segment, hold at most
    # chunk_tiles tiles, are as few as that allows and differ by at most one tile within a segment
    seen = {}
    for (c0, cn, r0, nu) in got["items"].tolist():
        s = int(np.searchsorted(got["seg_ptr"], c0, side="right")) - 1
        assert got["seg_ptr"][s] <= c0 and c0 + cn <= got["seg_ptr"][s + 1] and 1 <= cn <= got["chunk_tiles"]
        for (u, _) in got["qrefs"][r0:r0 + nu].tolist():
            seen.setdefault((s, u), []).append((c0, cn))
    for u in range(nq):
        mine = [0] * (pool.sink_len > 0) + [int(g) + 1 for g in sels[u]]
        assert sorted(s for (s, v) in seen if v == u) == sorted(s for s in mine if segs[s] > 0)
    for (s, u), runs in seen.items():
        assert [c0 for c0, _ in runs] == list(np.cumsum([got["seg_ptr"][s]] + [cn for _, cn in runs[:-1]]))
        assert sum(cn for _, cn in runs) == segs[s] and len(runs) == -(-int(segs[s]) // got["chunk_tiles"])
        assert max(cn for _, cn in runs) - min(cn for _, cn in runs) <= 1


def test_config0_lists_match_oracle_and_counts():
    pc = synth.config0_pool()
    p = pc.pool
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, block_m=64, block_n=64,
                              host_only=True)
    got = lay.export()
    assert_same_lists(got, lo.preencode_layout(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, 64, 64))
    tab, ptr, ent = got
    # sink tile + 2 groups x 2 tiles; lists: [sink], then per group (sink, diag), (sink, full, diag)
    assert tab.tolist() == [[0, 4, -1, 0], [4, 64, 0, 0], [68, 64, 0, 0], [132, 64, 1, 0], [196, 64, 1, 0]]
    assert np.diff(ptr).tolist() == [1, 2, 3, 2, 3]
    qc = synth.config0_query(pc)
    layq = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                               sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=2, block_m=64, block_n=64,
                               host_only=True)
    assert_same_lists(layq.export(), lo.query_layout(p.sink_len, p.demo_offsets, p.group_demo_offsets, qc.cu_qlens,
                                                     qc.sel_ptr, qc.sel_idx, 64, 64))
    _, _, qent = layq.export()
    # sink, the two tiles of group 1, then the query's own 16 tokens under the causal rule
    assert qent.tolist() == [[0, 4], [132, 64], [196, 64], [0, 16 | (3 << 16)]]


def test_ragged_bf16_shape_lists_match_oracle():
    """A cut-down config-1 pool (ragged demo lengths, groups that are no tile multiple)."""
    pc_pool = synth.pack_groups(64, synth.draw_demo_lengths(np.random.default_rng(3), 4096, 32, 128), 4)
    for bm in (64, 256):
        lay = B.dbsa_layout_build(pc_pool.sink_len, pc_pool.demo_offsets, pc_pool.group_demo_offsets, 0, block_m=bm,
                                  block_n=64, host_only=True)
        assert_same_lists(lay.export(), lo.preencode_layout(pc_pool.sink_len, pc_pool.demo_offsets,
                                                            pc_pool.group_demo_offsets, 0, bm, 64))


def test_permuted_selection_gives_permuted_lists():
    pc = synth.config0_pool()
    p = pc.pool
    cu, sel_ptr = np.array([0, 5], np.int32), np.array([0, 2], np.int32)
    ents = []
    for sel in ([0, 1], [1, 0]):
        lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=cu, sel_ptr=sel_ptr,
                                  sel_idx=np.array(sel, np.int32), n_split=1, block_m=64, block_n=64, host_only=True)
        ents.append(lay.export()[2])
    a, b = ents
    assert a[0].tolist() == b[0].tolist()                      # sink first in both
    assert a[1:3].tolist() == b[3:5].tolist() and a[3:5].tolist() == b[1:3].tolist()
    assert a[5:].tolist() == b[5:].tolist()                    # self tiles last


def _build(pool_kw=None, sel_kw=None, **kw):
    pc = synth.config0_pool().pool
    args = dict(sink_len=pc.sink_len, demo_offsets=pc.demo_offsets, group_demo_offsets=pc.group_demo_offsets)
    args.update(pool_kw or {})
    return B.dbsa_layout_build(args["sink_len"], args["demo_offsets"], args["group_demo_offsets"], 0,
                               host_only=True, **(sel_kw or {}), **kw)


@pytest.mark.parametrize("pool_kw,sel_kw,code", [
    (dict(sink_len=3), None, B.DBSA_ERR_BAD_BOUNDS),                                   # demo_offsets[0] != S
    (dict(demo_offsets=[4, 36, 36, 100]), None, B.DBSA_ERR_BAD_BOUNDS),                # not strictly increasing
    (dict(group_demo_offsets=[0, 4, 9]), None, B.DBSA_ERR_BAD_BOUNDS),                 # last != n_demos
    (dict(group_demo_offsets=[1, 4, 8]), None, B.DBSA_ERR_BAD_BOUNDS),                 # first != 0
    (None, dict(cu_qlens=[0, 4], sel_ptr=[0, 2], sel_idx=[1, 1]), B.DBSA_ERR_BAD_SELECTION),   # duplicate
    (None, dict(cu_qlens=[0, 4], sel_ptr=[0, 1], sel_idx=[2]), B.DBSA_ERR_BAD_SELECTION),      # out of range
    (None, dict(cu_qlens=[0, 4], sel_ptr=[0, 1], sel_idx=[-1]), B.DBSA_ERR_BAD_SELECTION),
    (None, dict(cu_qlens=[0, 4, 4], sel_ptr=[0, 0, 0], sel_idx=[]), B.DBSA_ERR_BAD_BOUNDS),    # empty query
    (None, dict(cu_qlens=[1, 4], sel_ptr=[0, 0], sel_idx=[]), B.DBSA_ERR_BAD_BOUNDS),
    (None, dict(cu_qlens=[0, 4], sel_ptr=[0, 0], sel_idx=[], n_split=-1), B.DBSA_ERR_INVALID_ARG),
])
def test_malformed_inputs_are_rejected(pool_kw, sel_kw, code):
    with pytest.raises(B.DbsaError) as ei:
        _build(pool_kw, sel_kw)
    assert ei.value.code == code


def test_bad_tile_sizes_and_flags_are_rejected():
    for kw in (dict(block_m=0), dict(block_n=0), dict(block_n=1 << 16)):
        with pytest.raises(B.DbsaError) as ei:
            _build(**kw)
        assert ei.value.code == B.DBSA_ERR_INVALID_ARG


def test_empty_selection_and_same_group_in_two_queries_are_valid():
    lay = _build(sel_kw=dict(cu_qlens=[0, 4, 9], sel_ptr=[0, 0, 1], sel_idx=[1]))
    tab, ptr, ent = lay.export()
    assert np.diff(ptr).tolist() == [2, 4]          # (sink, self) and (sink, 2 group tiles, self)
    lay2 = _build(sel_kw=dict(cu_qlens=[0, 4, 9], sel_ptr=[0, 1, 2], sel_idx=[1, 1]))
    assert lay2.export()[0].shape[0] == 2


def test_host_only_layout_cannot_run_attention_and_workspace_size():
    lay = _build(sel_kw=dict(cu_qlens=[0, 4, 9], sel_ptr=[0, 0, 1], sel_idx=[1], n_split=3))
    # decode: one slot per (query, split) or per schedule slot; a split query prefill: up to 4 per query token
    slots = max(2 * 3, int(lay.export_decode_groups(2, 2)['slot_ptr'][-1]), 9 * 4)
    assert lay.workspace_bytes(32, 128) == slots * 32 * 132 * 4
    pre = _build()
    assert pre.workspace_bytes(32, 128) == 0
    t = B.Tensor(16, 8, 8)
    rc = B.lib().dbsa_preencode_attn(pre.handle, t, t, t, t, None, B.DBSA_BF16, 2, 2, 64, 0.125, None, 0, None)
    assert rc == B.DBSA_ERR_INVALID_ARG


def test_default_split_count_is_bounded_by_list_length():
    lay = _build(sel_kw=dict(cu_qlens=[0, 4], sel_ptr=[0, 0], sel_idx=[]))   # one sink tile only
    _, _, split = lay.export_decode(1)
    assert split.shape == (1, 2)


def test_group_major_schedule_batches_users_and_defaults_to_a_bounded_chunk():
    """40 queries on one group: two items per run (32 + 8 users); every slot is used once."""
    pc = synth.config0_pool().pool
    nq = 40
    cu = np.arange(nq + 1, dtype=np.int32)
    sel_ptr = np.arange(nq + 1, dtype=np.int32)
    sel_idx = np.ones(nq, np.int32)
    lay = B.dbsa_layout_build(pc.sink_len, pc.demo_offsets, pc.group_demo_offsets, cu_qlens=cu, sel_ptr=sel_ptr,
                              sel_idx=sel_idx, n_split=0, block_m=64, block_n=64, host_only=True)
    got = lay.export_decode_groups(pc.n_groups, nq)
    want = lo.decode_group_schedule(pc.sink_len, pc.demo_offsets, pc.group_demo_offsets, nq, sel_ptr, sel_idx, 64,
                                    got["chunk_tiles"])
    for key in ("seg_ptr", "seg_ent", "items", "qrefs", "slot_ptr"):
        assert np.array_equal(got[key], want[key]), key
    assert 1 <= got["chunk_tiles"] <= 64
    # so little work that a run is one tile: the sink tile and the group's two tiles, each for 32 + 8 users
    assert sorted(got["items"][:, 3].tolist()) == [8, 8, 8, 32, 32, 32]
    assert got["items"][:, 1].tolist() == [1] * 6
    # 40 of 64 rows filled: the contraction's records are whole segments (nothing worth cutting), with slots of their own
    rec, fill = lay.export_matrix_records()
    plan, nominal, refs, mx_slots = lay.export_matrix_plan(nq)
    assert fill >= 0.22 and rec[:, 1].tolist() == [40, 40] and rec[:, 3].tolist() == [1, 2] and plan.tolist() == [0, 2]
    assert np.diff(mx_slots).tolist() == [3] * nq
    slots = np.sort(got["qrefs"][:, 1])
    own = got["slot_ptr"][1:] - 1
    assert np.array_equal(np.sort(np.concatenate([slots, own])), np.arange(got["slot_ptr"][-1]))
    # the larger of the decode step's partial states and the split prefill's (up to 4 runs per prompt token)
    assert lay.workspace_bytes(4, 64) == max(int(got["slot_ptr"][-1]), 4 * nq) * 4 * 68 * 4


def test_rotary_calls_reject_bad_arguments_before_touching_the_device():
    import ctypes as C
    L = B.lib()
    f = (C.c_double * 64)(*([1.0] * 64))
    assert L.dbsa_rope_table(None, 128, 16, C.c_void_p(16), None) == B.DBSA_ERR_INVALID_ARG
    assert L.dbsa_rope_table(f, 128, 16, None, None) == B.DBSA_ERR_INVALID_ARG
    assert L.dbsa_rope_table(f, 128, 0, C.c_void_p(16), None) == B.DBSA_ERR_INVALID_ARG
    assert L.dbsa_rope_table(f, 130, 16, C.c_void_p(16), None) == B.DBSA_ERR_INVALID_ARG     # more pairs than the table argument holds
    t = B.Tensor(16, 256, 128)
    assert L.dbsa_rope_apply(t, t, 4, 2, 128, 7, None, 0, C.c_void_p(16), 8, None) == B.DBSA_ERR_UNSUPPORTED   # dtype
    assert L.dbsa_rope_apply(t, t, 4, 2, 24, B.DBSA_BF16, None, 0, C.c_void_p(16), 8, None) == B.DBSA_ERR_UNSUPPORTED
    assert L.dbsa_rope_apply(t, t, 4, 2, 128, B.DBSA_BF16, None, 0, None, 8, None) == B.DBSA_ERR_INVALID_ARG
    assert L.dbsa_rope_apply(B.Tensor(None, 256, 128), t, 4, 2, 128, B.DBSA_BF16, None, 0, C.c_void_p(16), 8, None) == \
        B.DBSA_ERR_INVALID_ARG
    # a host-only layout has no device lists: the re-positioning calls refuse it like the plain ones
    lay = _build(sel_kw=dict(cu_qlens=[0, 4, 9], sel_ptr=[0, 0, 1], sel_idx=[1]))
    tail = (B.DBSA_BF16, 4, 2, 128, C.c_float(0.1), None, 0, None)
    assert L.dbsa_query_attn_rope(lay.handle, t, t, t, t, t, t, None, C.c_void_p(16), 100000, *tail) == B.DBSA_ERR_INVALID_ARG
    assert L.dbsa_query_attn_rope(lay.handle, t, t, t, t, t, t, None, None, 100000, *tail) == B.DBSA_ERR_INVALID_ARG
    assert L.dbsa_decode_attn_rope(lay.handle, t, t, t, C.c_void_p(16), 1024, t, t, t, None, 0, *tail) == \
        B.DBSA_ERR_INVALID_ARG



def test_rotation_ids_known_to_the_host_must_lie_inside_the_table():
    """With positions == NULL the ids are first_id .. first_id + n_tokens - 1: checked before any launch."""
    import ctypes as C
    L = B.lib()
    t = B.Tensor(16, 256, 128)
    tab = C.c_void_p(16)
    assert L.dbsa_rope_apply(t, t, 4, 2, 128, B.DBSA_BF16, None, 5, tab, 8, None) == B.DBSA_ERR_INVALID_ARG    # ids 5..8, table of 8
    assert L.dbsa_rope_apply(t, t, 4, 2, 128, B.DBSA_BF16, None, -1, tab, 8, None) == B.DBSA_ERR_INVALID_ARG
    assert L.dbsa_rope_apply(t, t, 2 ** 31 - 1, 2, 128, B.DBSA_BF16, None, 2 ** 31 - 1, tab, 8, None) == \
        B.DBSA_ERR_INVALID_ARG                                                                               # no 32-bit wrap


def expected_decode_chunk(tiles, users, compute_units):
    """The default run length of the decode schedule, restated: tiles[s] / users[s] = tiles of segment s and
    queries that use it (segments without users or tiles left out)."""
    run_slots = max(1, compute_units * 6 // 8 * 3 // 4)
    batches = sum(t * -(-u // 32) for t, u in zip(tiles, users))
    return max(1, min(32, -(-batches // run_slots)))


def expected_matrix_plan(tiles, users, compute_units):
    """Runs cut to measure, restated: the (segment, 64 queries) units are walked in order; a worker takes tiles
    until its cost (tiles + 4.5 per run) reaches the share, a unit that does not fit is cut there, no run is shorter
    than 4 tiles; the share is the smallest (by bisection) that leaves the last worker no more than the others + 4.
    -> (run lengths in order, plan_ptr)."""
    k_run, k_snap, k_min_share = 4.5, 4, 12
    units = [t for t, u in zip(tiles, users) for _ in range(-(-u // 64))]
    line = sum(units)
    workers = max(1, min(max(1, compute_units // 8), line // k_min_share))

    def deal(target):
        plan, runs, acc = [0], [], 0.0
        for t in units:
            pos = 0
            while pos < t:
                room, rem = target - acc - k_run, t - pos
                if len(plan) >= workers or rem <= room + k_snap:
                    acc += k_run + rem
                    runs.append(rem)
                    pos = t
                elif room < k_snap and acc > 0.0:
                    plan.append(len(runs))
                    acc = 0.0
                else:
                    take = min(rem - k_snap, max(k_snap, int(room)))
                    pos += take
                    runs.append(take)
                    plan.append(len(runs))
                    acc = 0.0
        last = acc if len(plan) >= workers else 0.0
        plan += [len(runs)] * (workers + 1 - len(plan))
        return runs, plan, last

    lo = line / workers
    hi = (line + k_run * (len(units) + workers)) / workers + k_run + 2.0 * k_snap
    for _ in range(24):
        mid = 0.5 * (lo + hi)
        if deal(mid)[2] <= mid + k_snap:
            hi = mid
        else:
            lo = mid
    runs, plan, _ = deal(hi)
    return runs, plan


def test_default_decode_chunk_follows_the_compute_unit_count():
    """A layout built without a device is sized for 256 compute units.  Few queries per group: runs of pool
    tiles are cut so that about 144 single-wave workgroups per KV head (six per compute unit over eight KV
    heads, three quarters of them for pool runs) cover the step, never longer than 32 tiles.  Most of 64 rows
    filled: runs cut to measure for 32 workers per KV head, every worker within a few tiles of the mean cost."""
    pc = synth.make_pool_case("chunkpool", 11, dtype="bf16", n_q_heads=2, n_kv_heads=1, head_dim=16, sink_len=64,
                              pool_tokens=60000, demo_len_range=(200, 600), n_groups=6).pool
    assert 256 * 6 // 8 * 3 // 4 == 144
    seen = set()
    for nq in (1, 8, 20, 34, 40, 100, 200):
        cu = np.arange(nq + 1, dtype=np.int32)
        sel_ptr = (np.arange(nq + 1) * pc.n_groups).astype(np.int32)
        sel_idx = np.tile(np.arange(pc.n_groups, dtype=np.int32), nq)
        lay = B.dbsa_layout_build(pc.sink_len, pc.demo_offsets, pc.group_demo_offsets, cu_qlens=cu, sel_ptr=sel_ptr,
                                  sel_idx=sel_idx, n_split=0, block_m=64, block_n=64, host_only=True)
        got = lay.export_decode_groups(pc.n_groups, nq)
        tiles = np.diff(got["seg_ptr"]).tolist()
        want = expected_decode_chunk(tiles, [nq] * len(tiles), 256)     # every segment serves all nq queries
        assert got["chunk_tiles"] == want, (nq, got["chunk_tiles"], want)
        seen.add(want)
        assert got["items"][:, 1].max() <= want                         # no run is longer than the chunk
        rec, fill = lay.export_matrix_records()
        plan, nominal = lay.export_matrix_plan()
        assert (fill >= 0.22) == (nq in (20, 34, 40, 100, 200)), (nq, fill)
        assert nominal == (32 if fill >= 0.22 else 0) and (len(plan) > 0) == (fill >= 0.22)
        if fill >= 0.22:
            runs, want_plan = expected_matrix_plan(tiles, [nq] * len(tiles), 256)
            assert rec[:, 3].tolist() == runs and plan.tolist() == want_plan
            # every unit's runs tile its segment in order; a worker's records are consecutive
            assert plan[0] == 0 and plan[-1] == len(rec) and np.all(np.diff(plan) >= 0)
            cost = np.array([rec[plan[c]:plan[c + 1], 3].sum() + 4.5 * (plan[c + 1] - plan[c]) for c in range(len(plan) - 1)])
            assert cost.max() <= cost.mean() + 8.5, (nq, cost.max(), cost.mean())
            assert rec[:, 3].min() >= min(4, min(tiles))
    assert len(seen) >= 3


@pytest.mark.parametrize("seed", range(12))
def test_runs_cut_to_measure_tile_every_unit_and_balance_the_workers(seed):
    """Random pools (a few huge groups, many tiny ones, ragged user counts): wherever a layout cuts its runs to
    measure, the runs of a (segment, 64 users) unit tile it in order, none is shorter than 4 tiles unless the unit is,
    the plan hands every record to one worker, and no worker but the last carries more than the share allows."""
    rng = np.random.default_rng(100 + seed)
    n_groups = int(rng.integers(1, 40))
    small = seed % 3 == 0                      # many groups of a tile or two / a few long ones
    pc = synth.make_pool_case("planpool", 200 + seed, dtype="bf16", n_q_heads=2, n_kv_heads=1, head_dim=16,
                              sink_len=int(rng.integers(1, 300)), pool_tokens=int(n_groups * (60 if small else rng.integers(300, 5000))),
                              demo_len_range=(5, 40) if small else (30, 400), n_groups=n_groups).pool
    n_groups = pc.n_groups
    n_q = int(rng.integers(40, 400))
    sels = [np.sort(rng.choice(n_groups, size=int(rng.integers(max(1, n_groups // 2), n_groups + 1)), replace=False)) for _ in range(n_q)]
    sel_ptr = np.concatenate([[0], np.cumsum([len(x) for x in sels])]).astype(np.int32)
    sel_idx = np.concatenate(sels).astype(np.int32)
    cu = np.arange(n_q + 1, dtype=np.int32)
    lay = B.dbsa_layout_build(pc.sink_len, pc.demo_offsets, pc.group_demo_offsets, cu_qlens=cu, sel_ptr=sel_ptr,
                              sel_idx=sel_idx, n_split=0, block_m=64, block_n=64, host_only=True)
    got = lay.export_decode_groups(n_groups, n_q)
    rec, fill = lay.export_matrix_records()
    plan, nominal = lay.export_matrix_plan()
    if fill < 0.22:
        assert len(plan) == 0 and nominal == 0
        return
    assert nominal == 32 and plan[0] == 0 and plan[-1] == len(rec) and np.all(np.diff(plan) >= 0) and len(plan) - 1 <= 32
    seg_ptr = got["seg_ptr"]
    users = [n_q] + [int((sel_idx == g).sum()) for g in range(n_groups)]
    tiles = np.diff(seg_ptr).tolist()
    # the records, in order, walk the units (segment, batch of 64 users) and tile each of them
    i = 0
    for s, (t, u) in enumerate(zip(tiles, users)):
        if t == 0 or u == 0:
            continue
        for b in range(-(-u // 64)):
            at = int(seg_ptr[s])
            while at < seg_ptr[s + 1]:
                r0, nq, e0, en = rec[i]
                assert e0 == at and nq == min(64, u - 64 * b) and en >= min(4, t), (s, b, rec[i].tolist())
                at += int(en)
                i += 1
            assert at == seg_ptr[s + 1]
    assert i == len(rec)
    runs, want_plan = expected_matrix_plan(tiles, users, 256)
    assert rec[:, 3].tolist() == runs and plan.tolist() == want_plan
    _, _, plan_refs, plan_slots = lay.export_matrix_plan(n_q)
    _check_plan_covers_segments(rec, plan_refs, plan_slots, seg_ptr, sel_ptr, sel_idx, n_q)
    # the work items keep runs of one length
    assert got["items"][:, 1].max() <= got["chunk_tiles"] <= 32
    cost = np.array([rec[plan[c]:plan[c + 1], 3].sum() + 4.5 * (plan[c + 1] - plan[c]) for c in range(len(plan) - 1)])
    assert cost[:-1].max(initial=0.0) <= cost.mean() + 4.5 + 2 * 4 + 4.5 * 2 or len(cost) == 1, (cost.max(), cost.mean())


@pytest.mark.parametrize("n_classes", [1, 7, 64, 512])
def test_persistent_schedule_deals_every_tile_once_and_balances(n_classes):
    """Records repeat the layout's own tables; every Q tile is served by exactly one worker; no worker
    carries more than the mean load plus one round's spread."""
    pc = synth.make_pool_case("schedpool", 5, dtype="bf16", n_q_heads=2, n_kv_heads=1, head_dim=16, sink_len=100,
                              pool_tokens=40000, demo_len_range=(100, 900), n_groups=9).pool
    lay = B.dbsa_layout_build(pc.sink_len, pc.demo_offsets, pc.group_demo_offsets, block_m=64, block_n=64,
                              host_only=True)
    tab, ptr, _ = lay.export()
    cptr, rec = lay.export_schedule(n_classes)
    n = tab.shape[0]
    assert cptr[0] == 0 and cptr[-1] == n and np.all(np.diff(cptr) >= 0)
    entries = np.diff(ptr)
    by_key = {(int(tab[t, 0]), int(tab[t, 1])): t for t in range(n)}
    assert len(by_key) == n
    served = np.zeros(n, np.int32)
    load = np.zeros(n_classes)
    for c in range(n_classes):
        for q_start, q_len, first, count in rec[cptr[c]:cptr[c + 1]]:
            t = by_key[(int(q_start), int(q_len))]
            served[t] += 1
            assert first == ptr[t] and count == entries[t]
            load[c] += count + 3
    assert np.all(served == 1)
    # greedy dealing: the heaviest worker is at most one tile's cost above the lightest ... within
    # a round; over the launch the spread stays below the cost of the largest tile
    assert load.max() - load.min() <= entries.max() + 3
    # a layout keeps one schedule
    import ctypes as C
    assert B.lib().dbsa_layout_export_schedule(lay.handle, n_classes + 1, None, None) == B.DBSA_ERR_INVALID_ARG
    assert B.lib().dbsa_layout_export_schedule(lay.handle, n_classes, None, None) == B.DBSA_OK
    assert B.lib().dbsa_layout_export_schedule(lay.handle, 0, None, None) == B.DBSA_ERR_INVALID_ARG
    assert B.lib().dbsa_layout_export_schedule(None, 4, None, None) == B.DBSA_ERR_INVALID_ARG


def _check_plan_covers_segments(rec, refs, slots, seg_ptr, sel_ptr, sel_idx, n_queries):
    assert rec[0, 0] == 0 and np.array_equal(rec[1:, 0], (rec[:, 0] + rec[:, 1])[:-1]) and rec[-1, 0] + rec[-1, 1] == len(refs)
    seen = {}                      # (segment, query) -> tiles covered so far
    used_slots = [[] for _ in range(n_queries)]
    seg_of_tile = np.searchsorted(seg_ptr, np.arange(seg_ptr[-1]), side="right") - 1
    for r0, nq, e0, en in rec:
        s = int(seg_of_tile[e0])
        assert seg_ptr[s] <= e0 and e0 + en <= seg_ptr[s + 1]
        for q, slot in refs[r0:r0 + nq]:
            assert seen.get((s, int(q)), int(seg_ptr[s])) == e0, "a user's runs of a segment follow each other"
            seen[(s, int(q))] = int(e0 + en)
            used_slots[int(q)].append(int(slot))
    for u in range(n_queries):
        segs = [0] + [int(g) + 1 for g in sel_idx[sel_ptr[u]:sel_ptr[u + 1]]]
        for s in segs:
            if seg_ptr[s + 1] > seg_ptr[s]:
                assert seen.pop((s, u)) == seg_ptr[s + 1], (s, u)
        assert used_slots[u] == list(range(int(slots[u]), int(slots[u + 1]) - 1)), u
    assert not seen


@pytest.mark.parametrize("n_queries,n_select", [(5, 2), (70, 2), (130, 3), (300, 1)])
def test_matrix_records_cover_every_item_query_pair_once(n_queries, n_select):
    """The decode schedule's runs with up to 64 queries per record: each (item, query) pair of the 32-query
    schedule appears in exactly one record with the same tiles and the same slot; references are contiguous."""
    pc = synth.make_pool_case("mxhost", 21, dtype="bf16", n_q_heads=2, n_kv_heads=1, head_dim=16, sink_len=70,
                              pool_tokens=9000, demo_len_range=(30, 140), n_groups=4).pool
    rng = np.random.default_rng(n_queries)
    sel_ptr, sel_idx = synth.draw_selections(rng, n_queries, pc.n_groups, n_select)
    cu = np.arange(n_queries + 1, dtype=np.int32)
    lay = B.dbsa_layout_build(pc.sink_len, pc.demo_offsets, pc.group_demo_offsets, cu_qlens=cu, sel_ptr=sel_ptr,
                              sel_idx=sel_idx, n_split=0, block_m=32, block_n=64, host_only=True)
    got = lay.export_decode_groups(pc.n_groups, n_queries)
    rec, fill = lay.export_matrix_records()
    items, qrefs = got["items"], got["qrefs"]
    assert np.all(rec[:, 1] >= 1) and np.all(rec[:, 1] <= 64)
    plan, _, plan_refs, plan_slots = lay.export_matrix_plan(n_queries)
    if len(plan):
        # runs, references and slots of the records' own: every (segment, user) pair sees each tile of the segment once,
        # a query's slots are its records in order plus one for its own cache
        assert fill >= 0.22
        _check_plan_covers_segments(rec, plan_refs, plan_slots, got["seg_ptr"], sel_ptr, sel_idx, n_queries)
        return
    assert fill < 0.22
    # references of the records tile the reference array in order, without gaps
    assert rec[0, 0] == 0 and np.array_equal(rec[1:, 0], (rec[:, 0] + rec[:, 1])[:-1]) and rec[-1, 0] + rec[-1, 1] == len(qrefs)
    pairs_items = sorted((int(e0), int(en), int(q), int(s)) for e0, en, r0, nq in items for q, s in qrefs[r0:r0 + nq])
    pairs_rec = sorted((int(e0), int(en), int(q), int(s)) for r0, nq, e0, en in rec for q, s in qrefs[r0:r0 + nq])
    assert pairs_items == pairs_rec
    want_fill = float((rec[:, 1] * rec[:, 3]).sum()) / float((64 * rec[:, 3]).sum())
    assert abs(fill - want_fill) < 1e-6
    # a record is one item or two consecutive ones of the same run
    assert len(rec) >= (len(items) + 1) // 2


def test_query_stage_launch_order_groups_queries_by_their_selections():
    """The order is a permutation; an owner's tiles stay together, longest list first; owners follow each other in
    the order of their selection lists (word by word, ties by query index)."""
    pc = synth.make_pool_case("ordpool", 31, dtype="bf16", n_q_heads=2, n_kv_heads=1, head_dim=16, sink_len=10,
                              pool_tokens=3000, demo_len_range=(30, 140), n_groups=6).pool
    rng = np.random.default_rng(3)
    n_q = 40
    sels = [sorted(rng.choice(6, size=int(rng.integers(0, 4)), replace=False).tolist()) for _ in range(n_q)]
    sel_ptr = np.concatenate([[0], np.cumsum([len(s) for s in sels])]).astype(np.int32)
    sel_idx = np.array([g for s in sels for g in s], dtype=np.int32)
    q_len = rng.integers(1, 150, size=n_q)
    cu = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    lay = B.dbsa_layout_build(pc.sink_len, pc.demo_offsets, pc.group_demo_offsets, cu_qlens=cu, sel_ptr=sel_ptr,
                              sel_idx=sel_idx, n_split=0, block_m=64, block_n=64, host_only=True)
    order = lay.export_order()
    tab, ptr, _ = lay.export()
    assert sorted(order.tolist()) == list(range(len(tab)))
    owners, lens = tab[order, 2], np.diff(ptr)[order]
    firsts = [int(o) for i, o in enumerate(owners) if i == 0 or owners[i - 1] != o]
    assert sorted(firsts) == list(range(n_q))                                   # every owner is one contiguous stretch
    assert firsts == sorted(range(n_q), key=lambda u: (sels[u], u))
    same = owners[:-1] == owners[1:]
    assert np.all(lens[:-1][same] >= lens[1:][same])
