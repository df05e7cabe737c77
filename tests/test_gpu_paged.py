"""Groups kept in pages of an arena (Sec. 4, storage cost: caches may be offloaded or
re-encoded): the query stage reads the selected groups wherever they sit and never touches
rows that belong to nobody.  Same kernels, same tile order, same values => bitwise equal to
the contiguous run; one oracle comparison on top."""
import numpy as np
import pytest
import torch

from oracle import dbsa_oracle as orc
from paper_2503_08640_amd import binding as B
from paper_2503_08640_amd import synth
from gpu_util import assert_close, to_dev, to_f64

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("rope", [False, True])
def test_query_stage_over_an_arena_equals_the_contiguous_run(rope):
    pc = synth.make_pool_case("arena", 5000, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, sink_len=70,
                              pool_tokens=4000, demo_len_range=(30, 120), n_groups=6, k_channel_sigma=0.5)
    p = pc.pool
    sels = [[3, 0], [5], [0, 3, 5], []]                 # groups 1, 2, 4 are selected by nobody
    qc = synth.make_query_case("arenaq", 5001, pc, n_queries=4, q_len=[64, 37, 100, 5], selections=sels, n_decode=2)
    gb = p.group_token_bounds().astype(np.int64)
    seg = [(0, p.sink_len)] + [(int(gb[g]), int(gb[g + 1])) for g in range(p.n_groups)]
    # arena: group 5, a hole, the sink, group 0, a hole, group 3, group 2 (resident but unused); 1 and 4 offloaded
    order, page_start, at = [6, 0, 1, 4, 3], np.full(p.n_groups + 1, -1, dtype=np.int32), 13
    for s in order:
        page_start[s] = at
        at += seg[s][1] - seg[s][0] + 29
    kp, vp = to_dev(pc.k), to_dev(pc.v)
    if rope:
        from oracle import rope_oracle as ro
        tab = B.dbsa_rope_table(ro.inv_freq(500000.0, 128), 2 * p.n_tokens + 200)
        kp = B.dbsa_rope_apply(kp, tab)                 # keys carry their encoding ids, wherever they are stored
    k_arena = torch.full((at, pc.n_kv_heads, pc.head_dim), float("nan"), dtype=kp.dtype, device="cuda")
    v_arena = torch.full_like(k_arena, float("nan"))
    for s in order:
        a, b = seg[s]
        k_arena[page_start[s]: page_start[s] + b - a] = kp[a:b]
        v_arena[page_start[s]: page_start[s] + b - a] = vp[a:b]
    kw = dict(cu_qlens=qc.cu_qlens, sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=32, block_n=64)
    plain = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, **kw)
    paged = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, page_start=page_start, **kw)
    qs, ks, vs = to_dev(qc.q), to_dev(qc.k), to_dev(qc.v)
    shp = qc.k_cache.shape
    kc = to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
    vc = to_dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    self_len = torch.from_numpy((np.diff(qc.cu_qlens) + 1).astype(np.int32)).cuda()
    if rope:
        a = B.dbsa_query_attn_rope(plain, qs, ks, vs, kp, vp, tab, pc.scale)
        b = B.dbsa_query_attn_rope(paged, qs, ks, vs, k_arena, v_arena, tab, pc.scale)
        da = B.dbsa_decode_attn_rope(plain, to_dev(qc.dec_q[0]), kc, vc, self_len, kp, vp, tab, pc.scale)
        db = B.dbsa_decode_attn_rope(paged, to_dev(qc.dec_q[0]), kc, vc, self_len, k_arena, v_arena, tab, pc.scale)
    else:
        a = B.dbsa_query_attn(plain, qs, ks, vs, kp, vp, pc.scale)
        b = B.dbsa_query_attn(paged, qs, ks, vs, k_arena, v_arena, pc.scale)
        da = B.dbsa_decode_attn(plain, to_dev(qc.dec_q[0]), kc, vc, self_len, kp, vp, pc.scale)
        db = B.dbsa_decode_attn(paged, to_dev(qc.dec_q[0]), kc, vc, self_len, k_arena, v_arena, pc.scale)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16)), "prefill differs between arena and contiguous pool"
    assert torch.equal(da.view(torch.int16), db.view(torch.int16)), "decode differs between arena and contiguous pool"
    if not rope:
        ref = orc.query_attn(synth.as_f64(qc.q), synth.as_f64(qc.k), synth.as_f64(qc.v), synth.as_f64(pc.k),
                             synth.as_f64(pc.v), p.sink_len, p.demo_offsets, p.group_demo_offsets, qc.cu_qlens,
                             qc.sel_ptr, qc.sel_idx, pc.scale)
        assert_close(to_f64(b), ref, "query prefill over the arena")
