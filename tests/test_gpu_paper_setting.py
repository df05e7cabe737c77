"""GPU parity for the pool structure the paper itself runs (Sec. 3, implementation details:
blocks of 50 demonstrations, the first block is the attention sink, every block also sees
the two blocks before it) and for the four encoding patterns of the attention ablation
(Sec. 5.2: Full, Sink + Prev + Self, Sink + Self, Self).  All four are the same layout
builder with different (sink, window) arguments; the kernels are the ones the benchmark
configurations use."""
import numpy as np
import pytest
import torch

from oracle import dbsa_oracle as orc
from oracle import layout_oracle as lo
from paper_2503_08640_amd import binding as B
from paper_2503_08640_amd import synth
from gpu_util import assert_close, to_dev, to_f64

pytestmark = pytest.mark.gpu


def _preencode(pc, block_m):
    p = pc.pool
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, pc.prev_window, block_m=block_m,
                              block_n=64)
    return lay, B.dbsa_preencode_attn(lay, to_dev(pc.q), to_dev(pc.k), to_dev(pc.v), pc.scale)


def _oracle(pc, rows=None):
    p = pc.pool
    return orc.preencode_attn(synth.as_f64(pc.q), synth.as_f64(pc.k), synth.as_f64(pc.v), p.sink_len, p.demo_offsets,
                              p.group_demo_offsets, pc.scale, pc.prev_window, rows=rows)


# name -> (first block is the sink, preceding blocks visible); 9 blocks of 6 demos
PATTERNS = {"full": (True, 8), "sink+prev+self": (True, 2), "sink+self": (True, 0), "self": (False, 0)}


@pytest.mark.parametrize("pattern", list(PATTERNS))
@pytest.mark.parametrize("block_m", [32, 64])
def test_sec52_encoding_patterns_all_rows(pattern, block_m):
    sink_first, w = PATTERNS[pattern]
    pc = synth.make_block_pool_case(f"sec52-{pattern}", 3000, n_demos=54, demos_per_block=6, demo_len_range=(28, 47),
                                    prev_window=w, sink_is_first_block=sink_first, n_q_heads=8, n_kv_heads=2)
    p = pc.pool
    assert p.n_groups == (8 if sink_first else 9) and (p.sink_len > 0) == sink_first
    lay, o = _preencode(pc, block_m)
    tab, ptr, ent = lay.export()
    otab, optr, oent = lo.preencode_layout(p.sink_len, p.demo_offsets, p.group_demo_offsets, w, block_m, 64)
    assert np.array_equal(tab, otab) and np.array_equal(ptr, optr) and np.array_equal(ent, oent)
    ref = _oracle(pc)
    assert_close(to_f64(o), ref, f"Sec. 5.2 pattern {pattern}, bm={block_m}")
    if pattern == "full":
        # every block sees every earlier block: dense causal attention over the whole pool
        q, k, v = (torch.from_numpy(synth.as_f64(x)).permute(1, 0, 2) for x in (pc.q, pc.k, pc.v))
        r = pc.n_q_heads // pc.n_kv_heads
        dense = torch.nn.functional.scaled_dot_product_attention(
            q, k.repeat_interleave(r, 0), v.repeat_interleave(r, 0), is_causal=True, scale=pc.scale)
        assert_close(to_f64(o), dense.permute(1, 0, 2).numpy(), "full pattern vs dense causal routine")


def test_paper_setting_query_and_decode_small():
    """Whole-block sink, window 2, 30 % of the blocks per query, ragged query lengths."""
    pc = synth.make_block_pool_case("paper-small", 3001, n_demos=88, demos_per_block=8, demo_len_range=(28, 47),
                                    prev_window=2, n_q_heads=8, n_kv_heads=2)
    p = pc.pool
    qc = synth.make_query_case("paper-small-q", 3002, pc, n_queries=5, q_len=[64, 33, 1, 40, 17],
                               n_select=synth.select_count(0.30, p.n_groups), n_decode=3)
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, 2, cu_qlens=qc.cu_qlens,
                              sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=32, block_n=64)
    kp, vp = to_dev(pc.k), to_dev(pc.v)
    kp64, vp64 = synth.as_f64(pc.k), synth.as_f64(pc.v)
    oq = B.dbsa_query_attn(lay, to_dev(qc.q), to_dev(qc.k), to_dev(qc.v), kp, vp, pc.scale)
    ref = orc.query_attn(synth.as_f64(qc.q), synth.as_f64(qc.k), synth.as_f64(qc.v), kp64, vp64, p.sink_len,
                         p.demo_offsets, p.group_demo_offsets, qc.cu_qlens, qc.sel_ptr, qc.sel_idx, pc.scale)
    assert_close(to_f64(oq), ref, "paper setting (small) query prefill")
    shp = qc.k_cache.shape
    kc = to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
    vc = to_dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    lens = np.diff(qc.cu_qlens)
    for s in range(3):
        self_len = (lens + s + 1).astype(np.int32)
        od = B.dbsa_decode_attn(lay, to_dev(qc.dec_q[s]), kc, vc, torch.from_numpy(self_len).cuda(), kp, vp, pc.scale)
        refd = orc.decode_attn(synth.as_f64(qc.dec_q[s]), synth.as_f64(qc.k_cache), synth.as_f64(qc.v_cache),
                               self_len, kp64, vp64, p.sink_len, p.demo_offsets, p.group_demo_offsets, qc.sel_ptr,
                               qc.sel_idx, pc.scale)
        assert_close(to_f64(od), refd, f"paper setting (small) decode step {s}")


def test_paper_setting_full_size():
    """2400 demonstrations / 90k tokens, 48 blocks of 50, sink = first block, window 2:
    sampled rows against the oracle, every row against the closed-form Q = 0 probe."""
    pc = synth.paper_setting_pool()
    p = pc.pool
    w = pc.prev_window
    gb = p.group_token_bounds().astype(np.int64)
    print(f"[case] paper setting: N={p.n_tokens} S={p.sink_len} G={p.n_groups} w={w}", flush=True)
    lay, o = _preencode(pc, B.BENCH_BLOCK_M_PREENCODE)
    rng = np.random.default_rng(pc.seed)
    rows = set(rng.choice(p.n_tokens, size=512, replace=False).tolist())
    rows |= set(range(0, p.sink_len, 7)) | {p.sink_len - 1}
    for g in (0, 1, 2, p.n_groups // 2, p.n_groups - 1):      # groups 0-2 have a shorter window than the rest
        rows |= set(range(int(gb[g]), int(gb[g]) + 66)) | set(range(int(gb[g + 1]) - 66, int(gb[g + 1])))
    rows = np.array(sorted(rows), dtype=np.int64)
    assert_close(to_f64(o[torch.from_numpy(rows).cuda()]), _oracle(pc, rows),
                 f"paper setting pre-encode, {len(rows)} sampled rows")

    # Q = 0: uniform weights over the visible set = sink + up to w preceding blocks + own block causally
    tok = np.arange(p.n_tokens, dtype=np.int64)
    grp = np.maximum(np.searchsorted(gb, tok, side="right") - 1, 0)
    first_vis_group = np.maximum(grp - w, 0)
    n_vis = np.where(tok < p.sink_len, tok + 1, p.sink_len + tok - gb[first_vis_group] + 1)
    v = to_dev(pc.v)
    vprobe = torch.zeros_like(v)
    vprobe[:, :, 0] = 1.0
    vprobe[: p.sink_len, :, 1] = 1.0
    oz = to_f64(B.dbsa_preencode_attn(lay, torch.zeros_like(to_dev(pc.q)), to_dev(pc.k), vprobe, pc.scale))
    assert np.abs(oz[:, :, 0] - 1.0).max() <= 2 ** -8
    sink_seen = np.minimum(tok + 1, p.sink_len)
    # relative output rounding 2^-8: the recovered sink share is exact to that
    assert np.abs(oz[:, :, 1] - (sink_seen / n_vis)[:, None]).max() <= 2 ** -8

    qc = synth.paper_setting_query(pc)
    assert int(qc.sel_ptr[1]) == 14
    layq = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, w, cu_qlens=qc.cu_qlens,
                               sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=B.BENCH_BLOCK_M_QUERY,
                               block_n=64)
    kp, vp = to_dev(pc.k), v
    kp64, vp64 = synth.as_f64(pc.k), synth.as_f64(pc.v)
    queries = (0, 5, 10, 15)
    oq = B.dbsa_query_attn(layq, to_dev(qc.q), to_dev(qc.k), to_dev(qc.v), kp, vp, pc.scale)
    ref = orc.query_attn(synth.as_f64(qc.q), synth.as_f64(qc.k), synth.as_f64(qc.v), kp64, vp64, p.sink_len,
                         p.demo_offsets, p.group_demo_offsets, qc.cu_qlens, qc.sel_ptr, qc.sel_idx, pc.scale,
                         queries=queries)
    qrows = np.concatenate([np.arange(qc.cu_qlens[u], qc.cu_qlens[u + 1]) for u in queries])
    assert_close(to_f64(oq)[qrows], ref[qrows], f"paper setting query prefill, queries {list(queries)}")
    shp = qc.k_cache.shape
    kc = to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
    vc = to_dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    lens = np.diff(qc.cu_qlens)
    for s in (0, 31):
        self_len = (lens + s + 1).astype(np.int32)
        od = B.dbsa_decode_attn(layq, to_dev(qc.dec_q[s]), kc, vc, torch.from_numpy(self_len).cuda(), kp, vp, pc.scale)
        refd = orc.decode_attn(synth.as_f64(qc.dec_q[s]), synth.as_f64(qc.k_cache), synth.as_f64(qc.v_cache),
                               self_len, kp64, vp64, p.sink_len, p.demo_offsets, p.group_demo_offsets, qc.sel_ptr,
                               qc.sel_idx, pc.scale, queries=queries)
        assert_close(to_f64(od)[list(queries)], refd[list(queries)], f"paper setting decode step {s}")


@pytest.mark.parametrize("w", [0, 2])
def test_appending_groups_reproduces_the_full_encoding(w):
    """Sec. 1 / Sec. 2.1: new demonstrations are added by encoding one more block with the same
    pattern.  Encode all but the last two groups, then append them: the appended rows equal the
    oracle, the rows written are exactly the new groups', and the result is bitwise the one a
    single pass over the whole pool produces."""
    pc = synth.make_block_pool_case("append", 3010 + w, n_demos=70, demos_per_block=10, demo_len_range=(28, 47),
                                    prev_window=w, n_q_heads=8, n_kv_heads=2)
    p = pc.pool
    g0 = p.n_groups - 2
    first_new = int(p.group_token_bounds()[g0])
    q, k, v = to_dev(pc.q), to_dev(pc.k), to_dev(pc.v)
    full = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, w, block_m=32, block_n=64)
    o_full = B.dbsa_preencode_attn(full, q, k, v, pc.scale)
    # the pool as it was before the addition: its description stops at group g0
    old = B.dbsa_layout_build(p.sink_len, p.demo_offsets[: p.group_demo_offsets[g0] + 1],
                              p.group_demo_offsets[: g0 + 1], w, block_m=32, block_n=64)
    o = torch.full_like(q, float("nan"))
    B.dbsa_preencode_attn(old, q[:first_new], k[:first_new], v[:first_new], pc.scale, out=o[:first_new])
    assert torch.isnan(o[first_new:]).all()
    app = B.dbsa_layout_build_append(p.sink_len, p.demo_offsets, p.group_demo_offsets, w, g0, block_m=32, block_n=64)
    B.dbsa_preencode_attn(app, q, k, v, pc.scale, out=o)
    assert torch.equal(o.view(torch.int16), o_full.view(torch.int16))
    assert_close(to_f64(o[first_new:]), _oracle(pc, np.arange(first_new, p.n_tokens)), f"appended groups, w={w}")
