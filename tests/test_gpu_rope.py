"""GPU parity of the query stage with re-positioning (Sec. 2.2) against oracle/rope_oracle.py.

The oracle gathers the un-rotated keys of [sink ; selected groups], rotates them at new
in-order ids and attends.  The library never gathers: pool keys are rotated ONCE at their
encoding ids (dbsa_rope_apply), and the query rows are rotated per segment instead."""
import numpy as np
import pytest
import torch

from oracle import rope_oracle as ro
from paper_2503_08640_amd import binding as B
from paper_2503_08640_amd import synth
from gpu_util import assert_close, to_dev, to_f64

pytestmark = pytest.mark.gpu


def test_rope_table_matches_fp64_angles():
    f = ro.inv_freq(500000.0, 128)
    n_pos = 100000
    tab = B.dbsa_rope_table(f, n_pos).cpu().numpy().astype(np.float64)
    ids = np.array([0, 1, 2, 63, 64, 4097, 65535, 65536, 99999])
    ang = ids[:, None] * f[None, :]
    assert np.abs(tab[ids, :, 0] - np.cos(ang)).max() <= 2 ** -23
    assert np.abs(tab[ids, :, 1] - np.sin(ang)).max() <= 2 ** -23


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rope_apply_matches_the_oracle_rotation(dtype):
    rng = np.random.default_rng(5)
    t, h, d = 300, 3, 128
    x = synth._store(rng.standard_normal((t, h, d)).astype(np.float32), dtype)
    f = ro.inv_freq(10000.0, d)
    tab = B.dbsa_rope_table(f, 5000)
    tol = 2 ** -8 * 6 if dtype == "bf16" else 1e-5      # |x| <~ 6; output rounded to bf16
    got = to_f64(B.dbsa_rope_apply(to_dev(x), tab, first_id=1000))
    assert np.abs(got - ro.rope(synth.as_f64(x), 1000 + np.arange(t), f)).max() <= tol
    pos = rng.integers(0, 5000, size=t).astype(np.int32)
    got = to_f64(B.dbsa_rope_apply(to_dev(x), tab, positions=torch.from_numpy(pos).cuda()))
    assert np.abs(got - ro.rope(synth.as_f64(x), pos, f)).max() <= tol


def _repositioned_case(pc, qc, block_m, base, n_split=0, queries=None, decode_steps=(0,), what=""):
    p = pc.pool
    d = pc.head_dim
    f = ro.inv_freq(base, d)
    lens = np.diff(qc.cu_qlens)
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, pc.prev_window, cu_qlens=qc.cu_qlens,
                              sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=n_split, block_m=block_m, block_n=64)
    list_shift, qref_shift, _ = lay.export_positions(qc.n_queries)
    # ids in use: pool keys up to N-1; rows up to shift + rows per tile; decode rows up to shift + self_len - 1
    n_pos = int(max(p.n_tokens, list_shift.max() + block_m, max(qref_shift.max(initial=0), 0) + lens.max() + qc.n_decode) + 1)
    tab = B.dbsa_rope_table(f, n_pos)
    # what the encoding pass leaves behind: keys rotated at their sequential ids (Sec. 2.1)
    kp = B.dbsa_rope_apply(to_dev(pc.k), tab, first_id=0)
    vp = to_dev(pc.v)
    local = np.concatenate([np.arange(n) for n in lens]).astype(np.int32)
    ks = B.dbsa_rope_apply(to_dev(qc.k), tab, positions=torch.from_numpy(local).cuda())
    oq = B.dbsa_query_attn_rope(lay, to_dev(qc.q), ks, to_dev(qc.v), kp, vp, tab, pc.scale)
    kp64, vp64 = synth.as_f64(pc.k), synth.as_f64(pc.v)
    ref = ro.query_attn_repositioned(synth.as_f64(qc.q), synth.as_f64(qc.k), synth.as_f64(qc.v), kp64, vp64,
                                     p.sink_len, p.demo_offsets, p.group_demo_offsets, qc.cu_qlens, qc.sel_ptr,
                                     qc.sel_idx, f, pc.scale, queries=queries)
    us = range(qc.n_queries) if queries is None else queries
    rows = np.concatenate([np.arange(qc.cu_qlens[u], qc.cu_qlens[u + 1]) for u in us])
    assert_close(to_f64(oq)[rows], ref[rows], f"{what} re-positioned prefill bm={block_m}")
    if qc.n_decode == 0:
        return
    shp = qc.k_cache.shape
    t_max = shp[1]
    cache_pos = torch.from_numpy(np.tile(np.arange(t_max, dtype=np.int32), shp[0])).cuda()
    kc = B.dbsa_rope_apply(to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])), tab, positions=cache_pos).view(shp)
    vc = to_dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    for s in decode_steps:
        self_len = (lens + s + 1).astype(np.int32)
        od = B.dbsa_decode_attn_rope(lay, to_dev(qc.dec_q[s]), kc, vc, torch.from_numpy(self_len).cuda(), kp, vp, tab,
                                     pc.scale)
        refd = ro.decode_attn_repositioned(synth.as_f64(qc.dec_q[s]), synth.as_f64(qc.k_cache),
                                           synth.as_f64(qc.v_cache), self_len, kp64, vp64, p.sink_len, p.demo_offsets,
                                           p.group_demo_offsets, qc.sel_ptr, qc.sel_idx, f, pc.scale, queries=queries)
        assert_close(to_f64(od)[list(us)], refd[list(us)], f"{what} re-positioned decode step {s}")


@pytest.mark.parametrize("hq,hkv,block_m,base", [(8, 2, 32, 500000.0), (8, 2, 64, 10000.0), (4, 4, 128, 10000.0),
                                                 (4, 4, 256, 500000.0), (8, 1, 32, 10000.0)])
def test_repositioned_query_and_decode_small(hq, hkv, block_m, base):
    """Permuted, empty and full selections, ragged query lengths, several head ratios: every row."""
    pc = synth.make_pool_case("ropepool", 4000 + hq + hkv, dtype="bf16", n_q_heads=hq, n_kv_heads=hkv, head_dim=128,
                              sink_len=70, pool_tokens=3000, demo_len_range=(30, 120), n_groups=5,
                              k_channel_sigma=0.5)
    sels = [[3, 0], [], [4, 1, 2, 0, 3], [2], [0, 1, 2, 3, 4], [1, 4]]
    qc = synth.make_query_case("ropeq", 4001, pc, n_queries=6, q_len=[64, 37, 100, 1, 33, 70], selections=sels,
                               n_decode=3)
    _repositioned_case(pc, qc, block_m, base, decode_steps=range(3), what=f"Hq={hq} Hkv={hkv}")


@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 2), (16, 2)])
def test_repositioned_decode_with_many_queries_per_group(hq, hkv):
    """40 queries on 3 groups: every group serves several batches of 32 / r queries, so the decode step runs the
    kernel whose waves share an item's tiles (r = 2) or, with query heads in fours per KV head, the contraction."""
    # (channel scales of sigma 0.35: with 0.5 one of the 16 heads of the third case gets scores beyond +-60,
    # where rounding the rotated, pre-scaled Q to bf16 alone moves single outputs by up to 2e-2, the whole
    # tolerance; the kernels agree with each other there to 7e-3)
    pc = synth.make_pool_case("ropemany", 4020 + hq, dtype="bf16", n_q_heads=hq, n_kv_heads=hkv, head_dim=128,
                              sink_len=40, pool_tokens=2500, demo_len_range=(30, 120), n_groups=3,
                              k_channel_sigma=0.35)
    qc = synth.make_query_case("ropemanyq", 4021, pc, n_queries=40, q_len=9, n_select=2, n_decode=2)
    if (hq // hkv) % 4 == 0:
        # query heads in fours per KV head and 27 of 64 rows filled: the pool items run as the contraction, whose
        # rows are rotated once per record, each at its own id
        p = pc.pool
        host = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, pc.prev_window, cu_qlens=qc.cu_qlens,
                                   sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=32, block_n=64, host_only=True)
        assert host.export_matrix_records()[1] >= 0.22
    _repositioned_case(pc, qc, 32, 10000.0, decode_steps=range(2), what=f"many queries Hq={hq} Hkv={hkv}")


@pytest.mark.parametrize("hq,hkv,block_m,q_len", [(4, 4, 128, [1500, 1283]), (4, 2, 256, [1700, 1201]), (2, 2, 256, [1999])])
def test_repositioned_split_prefill_with_large_q_tiles(hq, hkv, block_m, q_len):
    """Few long queries under Q tiles of 128 / 256 rows: the lists are cut into runs (the workspace is given),
    and the last block_m / 64 entries of every list hide keys from the Q tile's upper rows.  No run may start
    among them behind the first: the kernel takes a row's first maximum from the first tile of its run."""
    pc = synth.make_pool_case("ropebig", 4030 + block_m + hq, dtype="bf16", n_q_heads=hq, n_kv_heads=hkv, head_dim=128,
                              sink_len=70, pool_tokens=6000, demo_len_range=(64, 300), n_groups=3)
    sels = [[2, 0, 1], [1]][:len(q_len)]
    qc = synth.make_query_case("ropebigq", 4031, pc, n_queries=len(q_len), q_len=q_len, selections=sels)
    _repositioned_case(pc, qc, block_m, 500000.0, what=f"split, bm={block_m} T={q_len}")


def test_repositioned_stage_matches_the_position_free_stage_when_ids_do_not_move():
    """All groups in pool order: new ids = encoding ids, so the re-positioned calls must agree
    with the position-free calls on explicitly rotated inputs (same kernels, other code path)."""
    pc = synth.make_pool_case("ropeid", 4010, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, sink_len=64,
                              pool_tokens=2000, demo_len_range=(30, 120), n_groups=4)
    p = pc.pool
    sel = [list(range(4))] * 3
    qc = synth.make_query_case("ropeidq", 4011, pc, n_queries=3, q_len=[50, 64, 9], selections=sel)
    f = ro.inv_freq(10000.0, 128)
    tab = B.dbsa_rope_table(f, 2 * p.n_tokens + 100)
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                              sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, block_m=32, block_n=64)
    lens = np.diff(qc.cu_qlens)
    local = np.concatenate([np.arange(n) for n in lens]).astype(np.int32)
    kp = B.dbsa_rope_apply(to_dev(pc.k), tab)
    ks_local = B.dbsa_rope_apply(to_dev(qc.k), tab, positions=torch.from_numpy(local).cuda())
    got = B.dbsa_query_attn_rope(lay, to_dev(qc.q), ks_local, to_dev(qc.v), kp, to_dev(pc.v), tab, pc.scale)
    absolute = torch.from_numpy(local + p.n_tokens).cuda()
    q_abs = B.dbsa_rope_apply(to_dev(qc.q), tab, positions=absolute)
    ks_abs = B.dbsa_rope_apply(to_dev(qc.k), tab, positions=absolute)
    want = B.dbsa_query_attn(lay, q_abs, ks_abs, to_dev(qc.v), kp, to_dev(pc.v), pc.scale)
    # both sides round Q and K to bf16 at different points: a few output quanta
    assert_close(to_f64(got), to_f64(want), "re-positioned vs position-free on rotated inputs")


def test_repositioned_calls_reject_a_table_shorter_than_the_ids_in_use():
    pc = synth.config0_pool()                      # fp32, head_dim 64
    qc = synth.config0_query(pc)
    p = pc.pool
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                              sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, block_m=64, block_n=64)
    small = B.dbsa_rope_table(ro.inv_freq(10000.0, 64), 8)
    with pytest.raises(B.DbsaError) as ei:
        B.dbsa_query_attn_rope(lay, to_dev(qc.q), to_dev(qc.k), to_dev(qc.v), to_dev(pc.k), to_dev(pc.v), small,
                               pc.scale)
    assert ei.value.code == B.DBSA_ERR_INVALID_ARG


@pytest.mark.parametrize("dtype,hq,hkv,d,block_m", [("f32", 4, 2, 64, 64), ("f32", 6, 2, 128, 32), ("bf16", 4, 2, 64, 64),
                                                    ("bf16", 6, 2, 128, 64), ("bf16", 3, 1, 64, 32)])
def test_repositioned_query_and_decode_on_the_shapes_of_the_plain_kernels(dtype, hq, hkv, d, block_m):
    """fp32 storage, head_dim 64, three query heads per KV head (32 % 3 != 0: no group-major decode): the shapes
    the matrix kernels with re-positioning do not serve run the plain fp32-arithmetic kernels, prefill and decode,
    against the same oracle (bf16 with head_dim 128 and r = 3: the prefill is the pipelined kernel, the decode the
    plain one)."""
    pc = synth.make_pool_case("ropeplain", 4100 + hq + d, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d,
                              sink_len=70, pool_tokens=2500, demo_len_range=(30, 120), n_groups=5)
    sels = [[3, 0], [], [4, 1, 2, 0, 3], [2], [1, 4]]
    qc = synth.make_query_case("ropeplainq", 4101, pc, n_queries=5, q_len=[64, 37, 70, 1, 33], selections=sels,
                               n_decode=2)
    _repositioned_case(pc, qc, block_m, 10000.0, decode_steps=range(2), what=f"{dtype} Hq={hq} Hkv={hkv} D={d}")


def test_repositioned_config3_full_size():
    """Config 3 (90k pool, 16 queries x 64 tokens, 7 of 22 groups, Llama-3.1 rotary base) with
    new in-order ids: sampled queries against the oracle, first and last decode step."""
    pc = synth.config2_pool()
    qc = synth.config3_query(pc)
    _repositioned_case(pc, qc, B.BENCH_BLOCK_M_QUERY, 500000.0, queries=(0, 5, 10, 15), decode_steps=(0, 31),
                       what="cfg3")
