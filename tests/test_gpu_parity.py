"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle on
the same seeded inputs, element by element.  Sizes here are ones the oracle
finishes in seconds but that still span several tiles, ragged tails and every
tile kind.  Tolerance (bf16 inputs): max-abs 2e-2, mean-abs 2e-3; layouts bit-exact."""
import numpy as np
import pytest
import torch

from oracle import dbsa_oracle as orc
from oracle import layout_oracle as lo
from paper_2503_08640_amd import binding as B
from paper_2503_08640_amd import synth
from gpu_util import assert_close, pool_f64, to_dev, to_f64

pytestmark = pytest.mark.gpu


def run_preencode(pc, block_m, block_n=64, lse=False):
    p = pc.pool
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, pc.prev_window, block_m=block_m,
                              block_n=block_n)
    q, k, v = to_dev(pc.q), to_dev(pc.k), to_dev(pc.v)
    lse_t = torch.zeros(pc.n_q_heads, p.n_tokens, device="cuda", dtype=torch.float32) if lse else None
    o = B.dbsa_preencode_attn(lay, q, k, v, pc.scale, lse=lse_t)
    torch.cuda.synchronize()
    return lay, o, lse_t


def oracle_preencode(pc, rows=None, lse=False):
    q, k, v = pool_f64(pc)
    p = pc.pool
    return orc.preencode_attn(q, k, v, p.sink_len, p.demo_offsets, p.group_demo_offsets, pc.scale, pc.prev_window,
                              rows=rows, return_lse=lse)


def small_pool_case(name, seed, *, dtype="bf16", hq=4, hkv=4, d=128, sink=64, pool_tokens=4096, groups=4,
                    lens=(32, 128), sigma=0.0, w=0):
    return synth.make_pool_case(name, seed, dtype=dtype, n_q_heads=hq, n_kv_heads=hkv, head_dim=d, sink_len=sink,
                                pool_tokens=pool_tokens, demo_len_range=lens, n_groups=groups, k_channel_sigma=sigma,
                                prev_window=w)


# ---------------------------------------------------------------------------
# config 0: tiny fp32 case, every row
# ---------------------------------------------------------------------------

def test_config0_fp32_preencode_query_decode():
    pc = synth.config0_pool()
    qc = synth.config0_query(pc)
    p = pc.pool
    lay, o, lse = run_preencode(pc, block_m=64, lse=True)
    ref, ref_lse = oracle_preencode(pc, lse=True)
    assert_close(to_f64(o), ref, "cfg0 preencode fp32", max_tol=2e-5, mean_tol=2e-6)
    assert_close(to_f64(lse), ref_lse, "cfg0 preencode lse", max_tol=2e-5, mean_tol=2e-6)
    tab, ptr, ent = lay.export()
    otab, optr, oent = lo.preencode_layout(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, 64, 64)
    assert np.array_equal(tab, otab) and np.array_equal(ptr, optr) and np.array_equal(ent, oent)

    layq = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                               sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=2, block_m=64, block_n=64)
    kp, vp = to_dev(pc.k), to_dev(pc.v)
    oq = B.dbsa_query_attn(layq, to_dev(qc.q), to_dev(qc.k), to_dev(qc.v), kp, vp, pc.scale)
    refq = orc.query_attn(synth.as_f64(qc.q), synth.as_f64(qc.k), synth.as_f64(qc.v), synth.as_f64(pc.k),
                          synth.as_f64(pc.v), p.sink_len, p.demo_offsets, p.group_demo_offsets, qc.cu_qlens,
                          qc.sel_ptr, qc.sel_idx, pc.scale)
    assert_close(to_f64(oq), refq, "cfg0 query fp32", max_tol=2e-5, mean_tol=2e-6)
    kc, vc = to_dev(qc.k_cache.reshape(-1, *qc.k_cache.shape[2:])), to_dev(qc.v_cache.reshape(-1, *qc.v_cache.shape[2:]))
    kc, vc = kc.view(qc.k_cache.shape), vc.view(qc.v_cache.shape)
    t = int(qc.cu_qlens[1])
    for s in range(qc.n_decode):
        self_len = torch.tensor([t + s + 1], dtype=torch.int32, device="cuda")
        od = B.dbsa_decode_attn(layq, to_dev(qc.dec_q[s]), kc, vc, self_len, kp, vp, pc.scale)
        refd = orc.decode_attn(synth.as_f64(qc.dec_q[s]), synth.as_f64(qc.k_cache), synth.as_f64(qc.v_cache),
                               [t + s + 1], synth.as_f64(pc.k), synth.as_f64(pc.v), p.sink_len, p.demo_offsets,
                               p.group_demo_offsets, qc.sel_ptr, qc.sel_idx, pc.scale)
        assert_close(to_f64(od), refd, f"cfg0 decode step {s} fp32", max_tol=2e-5, mean_tol=2e-6)


def test_fp32_kernel_accepts_odd_tile_sizes():
    pc = synth.config0_pool()
    _, o, _ = run_preencode(pc, block_m=24, block_n=40)
    assert_close(to_f64(o), oracle_preencode(pc), "cfg0 preencode fp32, 24x40 tiles", max_tol=2e-5, mean_tol=2e-6)


# ---------------------------------------------------------------------------
# bf16 MFMA pre-encode on cut-down configs 1 and 2, every row
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("block_m", [32, 64, 128, 256])
def test_preencode_bf16_mha_ragged_groups_all_rows(block_m):
    pc = small_pool_case("cfg1_small", 2001)
    lay, o, lse = run_preencode(pc, block_m, lse=True)
    ref, ref_lse = oracle_preencode(pc, lse=True)
    assert_close(to_f64(o), ref, f"cfg1-small preencode bm={block_m}")
    assert_close(to_f64(lse), ref_lse, f"cfg1-small lse bm={block_m}", max_tol=2e-2, mean_tol=2e-3)
    p = pc.pool
    got = lay.export()
    want = lo.preencode_layout(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, block_m, 64)
    assert all(np.array_equal(a, b) for a, b in zip(got, want))


@pytest.mark.parametrize("block_m", [32, 64, 128])
def test_preencode_bf16_gqa_with_k_outliers_all_rows(block_m):
    pc = small_pool_case("cfg2_small", 2002, hq=8, hkv=2, pool_tokens=6000, groups=3, lens=(32, 256), sigma=0.5)
    _, o, _ = run_preencode(pc, block_m)
    assert_close(to_f64(o), oracle_preencode(pc), f"cfg2-small preencode bm={block_m}")


def test_preencode_bf16_head_dim_64():
    pc = small_pool_case("d64", 2003, hq=4, hkv=2, d=64, sink=4, pool_tokens=1000, groups=3, lens=(8, 40))
    _, o, _ = run_preencode(pc, 64)
    assert_close(to_f64(o), oracle_preencode(pc), "d64 preencode")


@pytest.mark.parametrize("sink,groups,w", [(0, 3, 0), (64, 1, 0), (5, 4, 2), (130, 3, 1)])
def test_preencode_bf16_degenerate_pools(sink, groups, w):
    pc = small_pool_case("edge", 2004 + sink, hq=2, hkv=1, sink=sink, pool_tokens=1500, groups=groups,
                         lens=(16, 90), w=w)
    _, o, _ = run_preencode(pc, 64)
    assert_close(to_f64(o), oracle_preencode(pc), f"edge preencode S={sink} G={groups} w={w}")


def test_preencode_bf16_strided_head_major_tensors():
    """Strides are API parameters: a head-major cache must give the same result."""
    pc = small_pool_case("strided", 2010, hq=4, hkv=2, pool_tokens=1200, groups=2)
    p = pc.pool
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, block_m=64, block_n=64)
    q = to_dev(pc.q)
    k = to_dev(pc.k).permute(1, 0, 2).contiguous().permute(1, 0, 2)   # [N, Hkv, D] view of head-major memory
    v = to_dev(pc.v).permute(1, 0, 2).contiguous().permute(1, 0, 2)
    o = B.dbsa_preencode_attn(lay, q, k, v, pc.scale)
    assert_close(to_f64(o), oracle_preencode(pc), "head-major K/V")


# ---------------------------------------------------------------------------
# query stage + decode, small
# ---------------------------------------------------------------------------

def _query_setup(pc, qc, block_m, n_split):
    p = pc.pool
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                              sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=n_split, block_m=block_m, block_n=64)
    return lay, to_dev(pc.k), to_dev(pc.v)


def _oracle_query(pc, qc, queries=None):
    p = pc.pool
    return orc.query_attn(synth.as_f64(qc.q), synth.as_f64(qc.k), synth.as_f64(qc.v), synth.as_f64(pc.k),
                          synth.as_f64(pc.v), p.sink_len, p.demo_offsets, p.group_demo_offsets, qc.cu_qlens,
                          qc.sel_ptr, qc.sel_idx, pc.scale, queries=queries)


def _run_decode_steps(pc, qc, lay, kp, vp, steps, what, queries=None):
    p = pc.pool
    shp = qc.k_cache.shape
    kc = to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
    vc = to_dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    lens = np.diff(qc.cu_qlens)
    kc64, vc64 = synth.as_f64(qc.k_cache), synth.as_f64(qc.v_cache)
    kp64, vp64 = synth.as_f64(pc.k), synth.as_f64(pc.v)
    for s in steps:
        self_len = (lens + s + 1).astype(np.int32)
        od = B.dbsa_decode_attn(lay, to_dev(qc.dec_q[s]), kc, vc, torch.from_numpy(self_len).cuda(), kp, vp, pc.scale)
        refd = orc.decode_attn(synth.as_f64(qc.dec_q[s]), kc64, vc64, self_len, kp64, vp64, p.sink_len,
                               p.demo_offsets, p.group_demo_offsets, qc.sel_ptr, qc.sel_idx, pc.scale,
                               queries=queries)
        got = to_f64(od)
        if queries is not None:
            got, refd = got[list(queries)], refd[list(queries)]
        assert_close(got, refd, f"{what} decode step {s}")


@pytest.mark.parametrize("block_m,n_split", [(32, 1), (64, 3), (128, 0)])
def test_query_and_decode_bf16_ragged_queries(block_m, n_split):
    pc = small_pool_case("qpool", 2020, hq=8, hkv=2, pool_tokens=5000, groups=5, lens=(32, 200), sigma=0.5)
    sels = [[3, 0], [], [4, 1, 2, 0, 3], [2]]
    qc = synth.make_query_case("q", 2021, pc, n_queries=4, q_len=[64, 37, 100, 1], selections=sels, n_decode=3)
    lay, kp, vp = _query_setup(pc, qc, block_m, n_split)
    oq = B.dbsa_query_attn(lay, to_dev(qc.q), to_dev(qc.k), to_dev(qc.v), kp, vp, pc.scale)
    assert_close(to_f64(oq), _oracle_query(pc, qc), f"query bm={block_m}")
    p = pc.pool
    got = lay.export()
    want = lo.query_layout(p.sink_len, p.demo_offsets, p.group_demo_offsets, qc.cu_qlens, qc.sel_ptr, qc.sel_idx,
                           block_m, 64)
    assert all(np.array_equal(a, b) for a, b in zip(got, want))
    _run_decode_steps(pc, qc, lay, kp, vp, range(3), f"bm={block_m} ns={n_split}")


@pytest.mark.parametrize("hq,hkv,block_m", [(4, 4, 128), (4, 4, 32), (4, 2, 64), (8, 1, 32), (16, 1, 32)])
def test_query_and_decode_bf16_head_ratios(hq, hkv, block_m):
    """MHA (one query head per KV head) up to 16 query heads per KV head; 40 queries on few
    groups so that decode items serve more queries than one wave has columns."""
    pc = small_pool_case("ratio", 2060 + hq + hkv, hq=hq, hkv=hkv, pool_tokens=2500, groups=3, lens=(32, 128))
    qc = synth.make_query_case("qr", 2061, pc, n_queries=40, q_len=9, n_select=2, n_decode=2)
    lay, kp, vp = _query_setup(pc, qc, block_m, 0)
    oq = B.dbsa_query_attn(lay, to_dev(qc.q), to_dev(qc.k), to_dev(qc.v), kp, vp, pc.scale)
    assert_close(to_f64(oq), _oracle_query(pc, qc), f"query Hq={hq} Hkv={hkv} bm={block_m}")
    _run_decode_steps(pc, qc, lay, kp, vp, range(2), f"Hq={hq} Hkv={hkv}")


@pytest.mark.parametrize("hq,hkv,d,n_split", [(4, 2, 64, 0), (6, 2, 128, 3), (6, 2, 64, 2)])
def test_query_and_decode_bf16_fallback_kernels(hq, hkv, d, n_split):
    """head_dim 64 and head ratios that do not divide 32 take the non-pipelined MFMA kernels and
    the per-(query, split) decode with its own merge."""
    pc = small_pool_case("fb", 2080 + hq + d, hq=hq, hkv=hkv, d=d, sink=20, pool_tokens=3000, groups=4, lens=(32, 150))
    qc = synth.make_query_case("qfb", 2081, pc, n_queries=4, q_len=[64, 37, 70, 1], selections=[[3, 0], [], [2, 1, 0, 3], [2]],
                               n_decode=2)
    lay, kp, vp = _query_setup(pc, qc, 64, n_split)
    oq = B.dbsa_query_attn(lay, to_dev(qc.q), to_dev(qc.k), to_dev(qc.v), kp, vp, pc.scale)
    assert_close(to_f64(oq), _oracle_query(pc, qc), f"fallback query Hq={hq} Hkv={hkv} D={d}")
    _run_decode_steps(pc, qc, lay, kp, vp, range(2), f"fallback Hq={hq} Hkv={hkv} D={d} ns={n_split}")


def test_token_strides_beyond_the_pipelined_kernels_reach_take_the_fallback():
    """The pipelined kernels address a tile's rows with 32-bit byte offsets (token stride < 2^24
    elements); a pool viewed with a larger stride must still give the right answer."""
    pc = small_pool_case("wide", 2090, hq=4, hkv=2, sink=8, pool_tokens=200, groups=2, lens=(16, 60))
    p = pc.pool
    stride = (1 << 24) + 256
    n = p.n_tokens

    def widen(x):                      # [N, H, D] -> the same values at a token stride of `stride` elements
        flat = torch.zeros(n * stride, dtype=x.dtype, device="cuda")
        view = flat.as_strided((n, x.shape[1], x.shape[2]), (stride, x.shape[2], 1))
        view.copy_(x)
        return view

    k, v = widen(to_dev(pc.k)), widen(to_dev(pc.v))
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, block_m=64, block_n=64)
    o = B.dbsa_preencode_attn(lay, to_dev(pc.q), k, v, pc.scale)
    assert_close(to_f64(o), oracle_preencode(pc), "pre-encode, token stride 2^24 + 256")
    qc = synth.make_query_case("qwide", 2091, pc, n_queries=2, q_len=[40, 3], selections=[[1], [0, 1]], n_decode=1)
    layq = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                               sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=2, block_m=64, block_n=64)
    oq = B.dbsa_query_attn(layq, to_dev(qc.q), to_dev(qc.k), to_dev(qc.v), k, v, pc.scale)
    assert_close(to_f64(oq), _oracle_query(pc, qc), "query prefill, token stride 2^24 + 256")
    _run_decode_steps(pc, qc, layq, k, v, range(1), "token stride 2^24 + 256")


def test_query_prefill_with_split_lists_agrees_with_the_single_pass():
    """Few Q tiles: with a workspace every list is cut into runs whose partial states are merged;
    without one the same call runs each list in one pass.  Both must match the oracle, and each
    other's log-sum-exp."""
    pc = small_pool_case("splitpool", 2070, hq=8, hkv=2, pool_tokens=9000, groups=4, lens=(32, 200), sigma=0.5)
    qc = synth.make_query_case("qs", 2071, pc, n_queries=3, q_len=[64, 50, 7], selections=[[0, 1, 2, 3], [2], [3, 1]])
    ref = _oracle_query(pc, qc)
    for bm in (32, 64):
        lay, kp, vp = _query_setup(pc, qc, bm, 0)
        qs, ks, vs = to_dev(qc.q), to_dev(qc.k), to_dev(qc.v)
        lse_a = torch.zeros(pc.n_q_heads, qs.shape[0], device="cuda")
        lse_b = torch.zeros_like(lse_a)
        one = B.dbsa_query_attn(lay, qs, ks, vs, kp, vp, pc.scale, lse=lse_a, workspace=False)
        cut = B.dbsa_query_attn(lay, qs, ks, vs, kp, vp, pc.scale, lse=lse_b)
        assert_close(to_f64(one), ref, f"single pass bm={bm}")
        assert_close(to_f64(cut), ref, f"split lists bm={bm}")
        assert not torch.equal(one, cut), "the workspace did not switch the split path on"
        assert (lse_a - lse_b).abs().max().item() <= 1e-3


def test_all_groups_selected_matches_dense_causal_oracle_and_order_is_irrelevant():
    pc = small_pool_case("full", 2030, hq=4, hkv=1, pool_tokens=3000, groups=4, lens=(32, 128))
    outs = []
    for sel in ([0, 1, 2, 3], [2, 0, 3, 1]):
        qc = synth.make_query_case("qfull", 2031, pc, n_queries=2, q_len=48, selections=[sel, sel[::-1]], n_decode=1)
        lay, kp, vp = _query_setup(pc, qc, 64, 2)
        oq = B.dbsa_query_attn(lay, to_dev(qc.q), to_dev(qc.k), to_dev(qc.v), kp, vp, pc.scale)
        assert_close(to_f64(oq), _oracle_query(pc, qc), f"all groups, order {sel}")
        outs.append(to_f64(oq))
    # a permuted selection re-orders the KV walk: equal up to fp32 summation order
    assert np.abs(outs[0] - outs[1]).max() <= 2e-2


def test_decode_with_self_cache_longer_than_one_tile():
    pc = small_pool_case("dpool", 2040, hq=8, hkv=2, pool_tokens=2000, groups=2, lens=(32, 128))
    qc = synth.make_query_case("qd", 2041, pc, n_queries=3, q_len=[130, 64, 7], n_select=1, n_decode=2)
    lay, kp, vp = _query_setup(pc, qc, 64, 4)
    _run_decode_steps(pc, qc, lay, kp, vp, range(2), "long self cache")


def test_attention_calls_reject_what_the_kernels_do_not_implement():
    pc = small_pool_case("rej", 2050, hq=4, hkv=2, pool_tokens=600, groups=2)
    p = pc.pool
    q, k, v = to_dev(pc.q), to_dev(pc.k), to_dev(pc.v)
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, block_m=48, block_n=64)
    with pytest.raises(B.DbsaError) as ei:
        B.dbsa_preencode_attn(lay, q, k, v, pc.scale)
    assert ei.value.code == B.DBSA_ERR_UNSUPPORTED
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, block_m=64, block_n=64)
    with pytest.raises(B.DbsaError) as ei:                      # 3 query heads over 2 KV heads
        B.dbsa_preencode_attn(lay, q[:, :3], k, v, pc.scale)
    assert ei.value.code == B.DBSA_ERR_UNSUPPORTED
    with pytest.raises(B.DbsaError) as ei:                      # a query-stage call on a pre-encode layout
        B.dbsa_query_attn(lay, q, k, v, k, v, pc.scale)
    assert ei.value.code == B.DBSA_ERR_INVALID_ARG
    qc = synth.make_query_case("qrej", 2051, pc, n_queries=2, q_len=8, n_select=1, n_decode=1)
    layq, kp, vp = _query_setup(pc, qc, 64, 2)
    shp = qc.k_cache.shape
    kc = to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
    with pytest.raises(B.DbsaError) as ei:                      # workspace too small
        B.dbsa_decode_attn(layq, to_dev(qc.dec_q[0]), kc, kc, torch.tensor([9, 9], dtype=torch.int32, device="cuda"),
                           kp, vp, pc.scale, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert ei.value.code == B.DBSA_ERR_WORKSPACE


# ---------------------------------------------------------------------------
# rows whose maximum keeps growing: the lazy-rescale path of every kernel
# ---------------------------------------------------------------------------
def _ramp_keys(k_bits, seg_bounds, direction, top, rng):
    """Keys = ramp(position inside its segment) * direction + small noise: with queries along
    `direction` the scores of a segment rise from 0 to about scale * |q| * `top`, i.e. by
    far more than the kernels' rescale slack (8 in log2 units) from one 64-key tile to the next."""
    n, hkv, d = k_bits.shape
    ramp = np.zeros(n, dtype=np.float32)
    for a, b in seg_bounds:
        if b > a:
            ramp[a:b] = np.arange(b - a, dtype=np.float32) / max(1, b - a - 1)
    k = ramp[:, None, None] * top * direction[None, None, :] + 0.3 * rng.standard_normal((n, hkv, d)).astype(np.float32)
    return synth.f32_to_bf16_bits(k)


@pytest.mark.parametrize("hq,hkv,block_m", [(8, 2, 32), (4, 4, 128), (8, 1, 64)])
def test_growing_row_maxima_take_the_rescale_path(hq, hkv, block_m):
    rng = np.random.default_rng(77)
    pc = small_pool_case("ramp", 2090 + hq, hq=hq, hkv=hkv, pool_tokens=3000, groups=3, lens=(32, 128))
    p = pc.pool
    d = pc.head_dim
    u = rng.standard_normal(d).astype(np.float32)
    u /= np.linalg.norm(u)
    c = 32.0                                            # |q . u|
    top = 200.0 / (pc.scale * c)                        # scores reach ~200
    gb = p.group_token_bounds()
    segs = [(0, p.sink_len)] + [(int(gb[g]), int(gb[g + 1])) for g in range(p.n_groups)]
    pc.k = _ramp_keys(pc.k, segs, u, top, rng)
    pc.q = synth.f32_to_bf16_bits(c * u[None, None, :] + rng.standard_normal(pc.q.shape).astype(np.float32))
    # the inputs do what they are meant to: along the keys of a group the tile maxima of a row rise by
    # more than the slack of 8 (log2 units) at nearly every 64-key tile
    row = int(gb[1]) - 1
    s_row = (synth.as_f64(pc.k)[int(gb[0]):row + 1, 0] @ synth.as_f64(pc.q)[row, 0]) * pc.scale * np.log2(np.e)
    tile_max = np.array([s_row[t:t + 64].max() for t in range(0, len(s_row), 64)])
    assert (np.diff(tile_max) > 8.0).mean() > 0.8 and len(tile_max) >= 8
    _, o, _ = run_preencode(pc, block_m)
    assert_close(to_f64(o), oracle_preencode(pc), f"ramped pre-encode bm={block_m}")

    n_q = 36 if hq // hkv >= 4 else 5                   # many queries per group: the shared-tile decode kernels too
    qc = synth.make_query_case("rampq", 2091, pc, n_queries=n_q, q_len=40, n_select=2, n_decode=2)
    lens = np.diff(qc.cu_qlens)
    qc.k = _ramp_keys(qc.k, [(int(qc.cu_qlens[i]), int(qc.cu_qlens[i + 1])) for i in range(n_q)], u, top, rng)
    qc.q = synth.f32_to_bf16_bits(c * u[None, None, :] + rng.standard_normal(qc.q.shape).astype(np.float32))
    qc.dec_q = synth.f32_to_bf16_bits(c * u[None, None, None, :] + rng.standard_normal(qc.dec_q.shape).astype(np.float32))
    t_max = qc.k_cache.shape[1]
    cache = _ramp_keys(qc.k_cache.reshape(n_q * t_max, hkv, d), [(i * t_max, i * t_max + int(lens[i]) + 2) for i in range(n_q)],
                       u, top, rng)
    qc.k_cache = cache.reshape(qc.k_cache.shape)
    lay, kp, vp = _query_setup(pc, qc, block_m if block_m <= 64 else 64, 0)
    oq = B.dbsa_query_attn(lay, to_dev(qc.q), to_dev(qc.k), to_dev(qc.v), kp, vp, pc.scale)
    assert_close(to_f64(oq), _oracle_query(pc, qc), f"ramped query prefill Hq={hq} Hkv={hkv}")
    _run_decode_steps(pc, qc, lay, kp, vp, range(2), f"ramped Hq={hq} Hkv={hkv}")   # one step per walk direction
