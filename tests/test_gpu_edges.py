"""GPU tests of the calls' edges: log-sum-exp of the query stage against the oracle, split query
prefill with large Q tiles, scores that jump by more than fp32's exponent range from one key to
the next, the alternation of the decode walk across rejected calls, table bounds of the
re-positioning decode, recycling of list blocks, chip-size constants.  Tolerances as in the parity
suite (bf16 inputs vs the fp64 oracle: max-abs 2e-2, mean-abs 2e-3), for the log-sum-exp too: the
kernels fold the softmax scale into Q and round it to bf16 again, so a score of size |s| carries an
error of about |s| * 2^-9 / sqrt(D) * sqrt(3) (a few 1e-3 at |s| ~ 20), and the log-sum-exp inherits
the error of the row's largest scores."""
import numpy as np
import pytest
import torch

from oracle import dbsa_oracle as orc
from paper_2503_08640_amd import binding as B
from paper_2503_08640_amd import synth
from gpu_util import assert_close, to_dev, to_f64
from test_gpu_parity import _oracle_query, _query_setup, _run_decode_steps, oracle_preencode, run_preencode, small_pool_case

pytestmark = pytest.mark.gpu


def oracle_query_lse(pc, qc):
    """[Hq, sum T]: log of the softmax denominator of every query row over sink, selected groups and own tokens."""
    p = pc.pool
    _, group_of = orc.token_maps(p.sink_len, p.demo_offsets, p.group_demo_offsets)
    q, ks, kp = synth.as_f64(qc.q), synth.as_f64(qc.k), synth.as_f64(pc.k)
    hq, hkv = q.shape[1], kp.shape[1]
    out = np.zeros((hq, q.shape[0]))
    for u in range(qc.n_queries):
        t0, t1 = int(qc.cu_qlens[u]), int(qc.cu_qlens[u + 1])
        sel = qc.sel_idx[int(qc.sel_ptr[u]):int(qc.sel_ptr[u + 1])]
        pool_vis = orc.mask_query_pool(sel, p.sink_len, group_of)
        a = np.arange(t1 - t0)
        mask = np.concatenate([np.broadcast_to(pool_vis, (t1 - t0, len(pool_vis))), a[None, :] <= a[:, None]], axis=1)
        for h in range(hq):
            kk = np.concatenate([kp[:, h // (hq // hkv)], ks[t0:t1, h // (hq // hkv)]], axis=0)
            out[h, t0:t1] = orc.log_sum_exp(q[t0:t1, h], kk, mask, pc.scale)
    return out


@pytest.mark.parametrize("hq,hkv,block_m", [(8, 2, 32), (8, 2, 64), (4, 4, 128), (4, 2, 256)])
def test_query_stage_log_sum_exp_matches_the_oracle(hq, hkv, block_m):
    """Single pass and split lists (the merge pass writes it there), ragged queries."""
    pc = small_pool_case("lsepool", 3100 + block_m, hq=hq, hkv=hkv, pool_tokens=9000, groups=4, lens=(32, 200), sigma=0.5)
    qc = synth.make_query_case("lseq", 3101, pc, n_queries=3, q_len=[300, 70, 9], selections=[[0, 1, 2, 3], [2, 0], [3, 1]])
    want = oracle_query_lse(pc, qc)
    ref = _oracle_query(pc, qc)
    lay, kp, vp = _query_setup(pc, qc, block_m, 0)
    qs, ks, vs = to_dev(qc.q), to_dev(qc.k), to_dev(qc.v)
    for ws, what in ((False, "single pass"), (None, "split lists")):
        lse = torch.zeros(hq, qs.shape[0], device="cuda")
        o = B.dbsa_query_attn(lay, qs, ks, vs, kp, vp, pc.scale, lse=lse, **({"workspace": False} if ws is False else {}))
        assert_close(to_f64(o), ref, f"{what} bm={block_m}")
        assert_close(to_f64(lse), want, f"query-stage lse, {what}, bm={block_m}")


@pytest.mark.parametrize("hq,hkv,block_m,q_len", [(4, 4, 128, [1500, 1283]), (8, 2, 128, [1990]), (4, 2, 256, [1700, 1201]),
                                                  (2, 2, 256, [1999])])
def test_split_query_prefill_with_large_q_tiles(hq, hkv, block_m, q_len):
    """Long queries under Q tiles of 128 and 256 rows: the last block_m / 64 list entries of a Q tile lie
    on its diagonal and hide keys from its upper rows, and the lists are cut into runs.  Every run
    must start at a tile all of its rows see; the result must not depend on the cut."""
    pc = small_pool_case("bigtile", 3200 + block_m + hq, hq=hq, hkv=hkv, pool_tokens=6000, groups=3, lens=(64, 300), sigma=0.5)
    sels = [[0, 1, 2], [1]][:len(q_len)]
    qc = synth.make_query_case("bigq", 3201, pc, n_queries=len(q_len), q_len=q_len, selections=sels)
    ref = _oracle_query(pc, qc)
    want_lse = oracle_query_lse(pc, qc)
    lay, kp, vp = _query_setup(pc, qc, block_m, 0)
    qs, ks, vs = to_dev(qc.q), to_dev(qc.k), to_dev(qc.v)
    lse = torch.zeros(hq, qs.shape[0], device="cuda")
    one = B.dbsa_query_attn(lay, qs, ks, vs, kp, vp, pc.scale, workspace=False)
    cut = B.dbsa_query_attn(lay, qs, ks, vs, kp, vp, pc.scale, lse=lse)
    assert not torch.equal(one, cut), "the workspace did not switch the split path on"
    assert_close(to_f64(one), ref, f"single pass bm={block_m} T={q_len}")
    assert_close(to_f64(cut), ref, f"split lists bm={block_m} T={q_len}")
    assert_close(to_f64(lse), want_lse, f"split lists lse bm={block_m} T={q_len}")


def _step_keys(k_bits, seg_bounds, direction, top, rng):
    """Keys whose score against a query along `direction` is about 0 up to a point inside each segment
    (not on a tile boundary) and about scale * |q| * top from there on, plus small noise."""
    n, hkv, d = k_bits.shape
    level = np.zeros(n, dtype=np.float32)
    for a, b in seg_bounds:
        if b - a >= 8:
            level[a + (b - a) * 5 // 8 + 3:b] = 1.0
    k = level[:, None, None] * top * direction[None, None, :] + 0.3 * rng.standard_normal((n, hkv, d)).astype(np.float32)
    return synth.f32_to_bf16_bits(k)


@pytest.mark.parametrize("hq,hkv,block_m,jump", [(8, 2, 32, 300.0), (4, 4, 128, 300.0), (8, 1, 64, 300.0), (8, 2, 32, 40.0),
                                                 (4, 4, 128, 40.0), (4, 2, 256, 300.0)])
def test_scores_that_jump_beyond_the_exponent_range(hq, hkv, block_m, jump):
    """Inside every segment the scores jump by `jump` (natural-log units): 300 is more than exp2 can
    represent relative to the running maximum (the unscaled probabilities overflow to infinity before the
    maximum catches up), 40 is far beyond the rescale slack but finite.  Pre-encode, query prefill, decode."""
    rng = np.random.default_rng(91)
    pc = small_pool_case("jump", 3300 + hq + block_m, hq=hq, hkv=hkv, pool_tokens=3000, groups=3, lens=(32, 128))
    p = pc.pool
    d = pc.head_dim
    u = rng.standard_normal(d).astype(np.float32)
    u /= np.linalg.norm(u)
    c = 32.0
    top = jump / (pc.scale * c)
    gb = p.group_token_bounds()
    segs = [(0, p.sink_len)] + [(int(gb[g]), int(gb[g + 1])) for g in range(p.n_groups)]
    pc.k = _step_keys(pc.k, segs, u, top, rng)
    pc.q = synth.f32_to_bf16_bits(c * u[None, None, :] + rng.standard_normal(pc.q.shape).astype(np.float32))
    row = int(gb[1]) - 1
    s_row = (synth.as_f64(pc.k)[int(gb[0]):row + 1, 0] @ synth.as_f64(pc.q)[row, 0]) * pc.scale * np.log2(np.e)
    assert s_row.max() - s_row[:64].max() > (128.0 if jump > 100 else 32.0)      # the inputs do what they are meant to
    _, o, _ = run_preencode(pc, block_m)
    assert_close(to_f64(o), oracle_preencode(pc), f"jump {jump} pre-encode bm={block_m}")

    n_q = 5
    qc = synth.make_query_case("jumpq", 3301, pc, n_queries=n_q, q_len=[300, 40, 129, 64, 7], n_select=2, n_decode=2)
    lens = np.diff(qc.cu_qlens)
    qc.k = _step_keys(qc.k, [(int(qc.cu_qlens[i]), int(qc.cu_qlens[i + 1])) for i in range(n_q)], u, top, rng)
    qc.q = synth.f32_to_bf16_bits(c * u[None, None, :] + rng.standard_normal(qc.q.shape).astype(np.float32))
    qc.dec_q = synth.f32_to_bf16_bits(c * u[None, None, None, :] + rng.standard_normal(qc.dec_q.shape).astype(np.float32))
    t_max = qc.k_cache.shape[1]
    cache = _step_keys(qc.k_cache.reshape(n_q * t_max, hkv, d), [(i * t_max, i * t_max + int(lens[i]) + 2) for i in range(n_q)],
                       u, top, rng)
    qc.k_cache = cache.reshape(qc.k_cache.shape)
    lay, kp, vp = _query_setup(pc, qc, block_m, 0)
    qs, ks, vs = to_dev(qc.q), to_dev(qc.k), to_dev(qc.v)
    ref = _oracle_query(pc, qc)
    assert_close(to_f64(B.dbsa_query_attn(lay, qs, ks, vs, kp, vp, pc.scale, workspace=False)), ref,
                 f"jump {jump} query prefill bm={block_m}")
    assert_close(to_f64(B.dbsa_query_attn(lay, qs, ks, vs, kp, vp, pc.scale)), ref, f"jump {jump} split query prefill bm={block_m}")
    if 32 % (hq // hkv) == 0:
        _run_decode_steps(pc, qc, lay, kp, vp, range(2), f"jump {jump} Hq={hq} Hkv={hkv}")


# ---------------------------------------------------------------------------
# API edges
# ---------------------------------------------------------------------------
def _decode_case(seed=3400, n_decode=4):
    pc = small_pool_case("edgepool", seed, hq=8, hkv=2, pool_tokens=5000, groups=4, lens=(32, 200), sigma=0.5)
    qc = synth.make_query_case("edgeq", seed + 1, pc, n_queries=4, q_len=[33, 64, 5, 100], n_select=2, n_decode=n_decode)
    shp = qc.k_cache.shape
    kc = to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
    vc = to_dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    return pc, qc, kc, vc


def test_a_rejected_decode_call_leaves_the_walk_direction_alone():
    """Twin layouts: one sees valid, REJECTED, REJECTED, valid; the other valid, valid.  The second valid calls
    walk the keys in the same direction, so the fp32 partial states they leave in the workspace are bitwise
    equal; the same step walked the other way leaves different bits."""
    pc, qc, kc, vc = _decode_case()
    lens = np.diff(qc.cu_qlens)
    kp, vp = to_dev(pc.k), to_dev(pc.v)
    lay_a, _, _ = _query_setup(pc, qc, 64, 0)
    lay_b, _, _ = _query_setup(pc, qc, 64, 0)
    sl = [torch.from_numpy((lens + s + 1).astype(np.int32)).cuda() for s in range(2)]
    q0, q1 = to_dev(qc.dec_q[0]), to_dev(qc.dec_q[1])
    n_ws = lay_a.workspace_bytes(pc.n_q_heads, pc.head_dim)
    ws_a = torch.zeros(n_ws, dtype=torch.uint8, device="cuda")
    ws_b = torch.zeros_like(ws_a)
    tiny = torch.empty(16, dtype=torch.uint8, device="cuda")
    a0 = B.dbsa_decode_attn(lay_a, q0, kc, vc, sl[0], kp, vp, pc.scale, workspace=ws_a)
    with pytest.raises(B.DbsaError) as ei:
        B.dbsa_decode_attn(lay_a, q1, kc, vc, sl[1], kp, vp, pc.scale, workspace=tiny)
    assert ei.value.code == B.DBSA_ERR_WORKSPACE
    tab = B.dbsa_rope_table(np.ones(64), 4)                        # far too short: rejected as well
    with pytest.raises(B.DbsaError) as ei:
        B.dbsa_decode_attn_rope(lay_a, q1, kc, vc, sl[1], kp, vp, tab, pc.scale)
    assert ei.value.code == B.DBSA_ERR_INVALID_ARG
    a1 = B.dbsa_decode_attn(lay_a, q1, kc, vc, sl[1], kp, vp, pc.scale, workspace=ws_a)
    b0 = B.dbsa_decode_attn(lay_b, q0, kc, vc, sl[0], kp, vp, pc.scale, workspace=ws_b)
    b1 = B.dbsa_decode_attn(lay_b, q1, kc, vc, sl[1], kp, vp, pc.scale, workspace=ws_b)
    torch.cuda.synchronize()
    assert torch.equal(a0, b0) and torch.equal(a1, b1)
    assert torch.equal(ws_a, ws_b)
    forward = ws_b.clone()
    b1_again = B.dbsa_decode_attn(lay_b, q1, kc, vc, sl[1], kp, vp, pc.scale, workspace=ws_b)
    torch.cuda.synchronize()
    assert not torch.equal(forward, ws_b), "the two walk directions left the same bits: the check above shows nothing"
    assert_close(to_f64(b1_again), to_f64(b1), "two walk directions")


def test_repositioning_decode_rejects_a_table_shorter_than_the_ids_in_reach():
    """A decode row looks up id shift + self_len - 1 <= max shift + Tmax - 1 (Tmax: tokens a query's cache holds)."""
    pc, qc, kc, vc = _decode_case(3410)
    lens = np.diff(qc.cu_qlens)
    kp, vp = to_dev(pc.k), to_dev(pc.v)
    lay, _, _ = _query_setup(pc, qc, 64, 0)
    _, qref_shift, _ = lay.export_positions(qc.n_queries)
    t_max = qc.k_cache.shape[1]
    need = int(qref_shift.max()) + t_max                              # ids 0 .. max shift + Tmax - 1
    f = np.ones(64)
    sl = torch.from_numpy((lens + 1).astype(np.int32)).cuda()
    q0 = to_dev(qc.dec_q[0])
    for fn, extra in ((B.dbsa_decode_attn_rope, {}),):
        with pytest.raises(B.DbsaError) as ei:
            fn(lay, q0, kc, vc, sl, kp, vp, B.dbsa_rope_table(f, need - 1), pc.scale, **extra)
        assert ei.value.code == B.DBSA_ERR_INVALID_ARG
        fn(lay, q0, kc, vc, sl, kp, vp, B.dbsa_rope_table(f, need), pc.scale, **extra)     # exactly enough: accepted
    torch.cuda.synchronize()


def test_list_blocks_of_destroyed_layouts_are_recycled_and_the_pool_stays_bounded():
    """Twenty layouts alive at once own twenty blocks; destroyed, all twenty go back to the pool, which keeps
    sixteen and frees the rest.  A layout built afterwards takes one of them."""
    pc = small_pool_case("poolpool", 3420, hq=2, hkv=2, pool_tokens=2000, groups=3, lens=(32, 64)).pool
    lays = [B.dbsa_layout_build(pc.sink_len, pc.demo_offsets, pc.group_demo_offsets, block_m=32, block_n=64)
            for _ in range(20)]
    torch.cuda.synchronize()
    for lay in lays:
        lay.destroy()
    # a block counts as idle once the events recorded at its layout's destruction have completed
    torch.cuda.synchronize()
    assert B.lib().dbsa_pooled_list_blocks() >= 16
    lay = B.dbsa_layout_build(pc.sink_len, pc.demo_offsets, pc.group_demo_offsets, block_m=32, block_n=64)
    lay.destroy()
    assert B.lib().dbsa_pooled_list_blocks() == 16
    torch.cuda.synchronize()
    lay = B.dbsa_layout_build(pc.sink_len, pc.demo_offsets, pc.group_demo_offsets, block_m=32, block_n=64)
    assert B.lib().dbsa_pooled_list_blocks() == 15
    lay.destroy()


def test_default_decode_chunk_uses_the_devices_compute_unit_count():
    from test_layout_host import expected_decode_chunk
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    pc = synth.make_pool_case("chunkdev", 12, dtype="bf16", n_q_heads=2, n_kv_heads=1, head_dim=128, sink_len=64,
                              pool_tokens=60000, demo_len_range=(200, 600), n_groups=6).pool
    for nq in (20, 100):
        cu = np.arange(nq + 1, dtype=np.int32)
        sel_ptr = (np.arange(nq + 1) * pc.n_groups).astype(np.int32)
        sel_idx = np.tile(np.arange(pc.n_groups, dtype=np.int32), nq)
        lay = B.dbsa_layout_build(pc.sink_len, pc.demo_offsets, pc.group_demo_offsets, cu_qlens=cu, sel_ptr=sel_ptr,
                                  sel_idx=sel_idx, n_split=0, block_m=64, block_n=64)
        got = lay.export_decode_groups(pc.n_groups, nq)
        tiles = np.diff(got["seg_ptr"]).tolist()
        assert got["chunk_tiles"] == expected_decode_chunk(tiles, [nq] * len(tiles), cus)


@pytest.mark.parametrize("n_queries,n_select,groups,hq,hkv", [(70, 2, 3, 8, 2), (130, 3, 3, 8, 2), (64, 2, 2, 8, 2),
                                                              (200, 4, 5, 8, 2), (100, 2, 3, 16, 2), (100, 3, 3, 8, 1)])
def test_decode_with_many_queries_per_group_as_a_contraction(n_queries, n_select, groups, hq, hkv):
    """Four (or eight) query heads per KV head and groups that each serve dozens of queries: the step runs its pool items
    with 64 queries per wave (batches of 64 + a ragged rest) and the queries' own caches in the single-wave
    kernel.  Every query, two steps (own caches of 10 and 11 keys ... and longer), against the oracle."""
    pc = small_pool_case("mxpool", 3500 + n_queries + hq, hq=hq, hkv=hkv, pool_tokens=2600, groups=groups, lens=(30, 140), sigma=0.5)
    rng = np.random.default_rng(n_queries)
    q_len = rng.integers(1, 80, size=n_queries).tolist()
    qc = synth.make_query_case("mxq", 3501, pc, n_queries=n_queries, q_len=q_len, n_select=n_select, n_decode=2)
    lay, kp, vp = _query_setup(pc, qc, 32, 0)
    rec, fill = lay.export_matrix_records()
    assert fill >= 0.22 and rec[:, 1].max() > 32, "this case is meant to take the contraction path"
    _run_decode_steps(pc, qc, lay, kp, vp, range(2), f"{n_queries} queries x {n_select} of {groups} groups")
    # twice the same step on twin layouts: bitwise equal (static schedule, no atomics)
    lay2, _, _ = _query_setup(pc, qc, 32, 0)
    shp = qc.k_cache.shape
    kc = to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
    vc = to_dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    sl = torch.from_numpy((np.diff(qc.cu_qlens) + 1).astype(np.int32)).cuda()
    lay3, _, _ = _query_setup(pc, qc, 32, 0)
    a = B.dbsa_decode_attn(lay2, to_dev(qc.dec_q[0]), kc, vc, sl, kp, vp, pc.scale)
    b = B.dbsa_decode_attn(lay3, to_dev(qc.dec_q[0]), kc, vc, sl, kp, vp, pc.scale)
    assert torch.equal(a, b)


# ---------------------------------------------------------------------------
# persistent prefill launches on ragged mid-size inputs (the full-size configs have regular shapes)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("hq,hkv,block_m,window", [(8, 2, 32, 0), (8, 2, 64, 0), (8, 2, 64, 2), (4, 4, 128, 0)])
def test_persistent_preencode_on_a_pool_of_many_short_groups(hq, hkv, block_m, window):
    """Enough Q tiles for the launch to run persistently (at least two per workgroup place), groups of a few
    hundred tokens with ragged ends: lists of 1 to ~10 tiles, short last Q tiles, a new owner every few records.
    Sampled rows (all of the sink, the first and last rows of many groups, random others) against the oracle."""
    tokens = {32: 18000, 64: 18000, 128: 34000}[block_m]
    pc = synth.make_pool_case("persist", 3600 + block_m + hq + window, dtype="bf16", n_q_heads=hq, n_kv_heads=hkv, head_dim=128,
                              sink_len=37, pool_tokens=tokens, demo_len_range=(20, 150), n_groups=45, k_channel_sigma=0.5,
                              prev_window=window)
    p = pc.pool
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, window, block_m=block_m, block_n=64)
    tab, _, _ = lay.export()
    heads_per_block = {(8, 2, 32): 4, (8, 2, 64): 4, (4, 4, 128): 1}[(hq, hkv, block_m)]
    places = torch.cuda.get_device_properties(0).multi_processor_count * (1 if heads_per_block * block_m // 32 == 8 else 2)
    classes = places // (hq // heads_per_block)
    assert tab.shape[0] >= 2 * classes, "this case is meant to launch persistently"
    o = B.dbsa_preencode_attn(lay, to_dev(pc.q), to_dev(pc.k), to_dev(pc.v), pc.scale)
    rng = np.random.default_rng(5)
    gb = p.group_token_bounds()
    rows = set(range(p.sink_len)) | set(rng.choice(p.n_tokens, size=700, replace=False).tolist())
    for g in range(0, p.n_groups, 3):
        rows |= set(range(int(gb[g]), int(gb[g]) + 3)) | set(range(int(gb[g + 1]) - 3, int(gb[g + 1])))
    rows = np.array(sorted(rows))
    ref = orc.preencode_attn(synth.as_f64(pc.q), synth.as_f64(pc.k), synth.as_f64(pc.v), p.sink_len, p.demo_offsets,
                             p.group_demo_offsets, pc.scale, window, rows=rows)
    assert_close(to_f64(o)[rows], ref, f"persistent pre-encode bm={block_m} Hq={hq} Hkv={hkv} w={window}")
    o2 = B.dbsa_preencode_attn(lay, to_dev(pc.q), to_dev(pc.k), to_dev(pc.v), pc.scale)
    assert torch.equal(o, o2)


def test_persistent_query_prefill_with_hundreds_of_ragged_queries():
    """700 queries of 1 to 64 tokens with selections of 0 to 4 groups (some empty, some all): one Q tile or two per
    query, more than two Q tiles per workgroup place, so the launch is persistent and its records end in tiles of
    the queries' own keys.  Every 7th query against the oracle."""
    pc = small_pool_case("persistq", 3700, hq=8, hkv=2, pool_tokens=3000, groups=4, lens=(30, 200), sigma=0.5)
    rng = np.random.default_rng(11)
    n_q = 700
    q_len = rng.integers(1, 65, size=n_q).tolist()
    sels = [sorted(rng.choice(4, size=int(rng.integers(0, 5)), replace=False).tolist()) for _ in range(n_q)]
    qc = synth.make_query_case("persistqq", 3701, pc, n_queries=n_q, q_len=q_len, selections=sels)
    lay, kp, vp = _query_setup(pc, qc, 32, 0)
    tab, _, _ = lay.export()
    assert tab.shape[0] >= 2 * (2 * torch.cuda.get_device_properties(0).multi_processor_count // 2)
    queries = list(range(0, n_q, 7))
    oq = B.dbsa_query_attn(lay, to_dev(qc.q), to_dev(qc.k), to_dev(qc.v), kp, vp, pc.scale, workspace=False)
    ref = _oracle_query(pc, qc, queries=queries)
    rows = np.concatenate([np.arange(qc.cu_qlens[u], qc.cu_qlens[u + 1]) for u in queries])
    assert_close(to_f64(oq)[rows], ref[rows], "persistent query prefill, 700 ragged queries")
