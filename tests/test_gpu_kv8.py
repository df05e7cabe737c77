"""Decode over a pool stored as 8-bit floats (e4m3) with per-KV-head scales.  Quantising is
input preparation, like rounding to bf16: the oracle receives the DE-quantised pool, so the
comparison charges the kernel only for its own arithmetic."""
import numpy as np
import pytest
import torch

from oracle import dbsa_oracle as orc
from paper_2503_08640_amd import binding as B
from paper_2503_08640_amd import synth
from gpu_util import assert_close, to_dev, to_f64

pytestmark = pytest.mark.gpu


def quantise_per_head(x: torch.Tensor):
    """[N, H, D] bf16 -> (float8_e4m3fn [N, H, D], float32 scale [H]) with absmax -> 448."""
    scale = (x.float().abs().amax(dim=(0, 2)) / 448.0).clamp_min(1e-12)
    x8 = (x.float() / scale[None, :, None]).to(torch.float8_e4m3fn)
    return x8, scale.contiguous()


def dequantise(x8: torch.Tensor, scale: torch.Tensor) -> np.ndarray:
    return (x8.float() * scale[None, :, None]).double().cpu().numpy()


def _decode_case(pc, qc, steps, queries=None, what=""):
    p = pc.pool
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                              sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=32, block_n=64)
    k8, ks = quantise_per_head(to_dev(pc.k))
    v8, vs = quantise_per_head(to_dev(pc.v))
    kq, vq = dequantise(k8, ks), dequantise(v8, vs)
    shp = qc.k_cache.shape
    kc = to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
    vc = to_dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    lens = np.diff(qc.cu_qlens)
    us = list(range(qc.n_queries)) if queries is None else list(queries)
    for s in steps:
        self_len = (lens + s + 1).astype(np.int32)
        od = B.dbsa_decode_attn_kv8(lay, to_dev(qc.dec_q[s]), kc, vc, torch.from_numpy(self_len).cuda(), k8, v8, ks, vs,
                                    pc.scale)
        ref = orc.decode_attn(synth.as_f64(qc.dec_q[s]), synth.as_f64(qc.k_cache), synth.as_f64(qc.v_cache), self_len,
                              kq, vq, p.sink_len, p.demo_offsets, p.group_demo_offsets, qc.sel_ptr, qc.sel_idx,
                              pc.scale, queries=queries)
        assert_close(to_f64(od)[us], ref[us], f"{what} fp8-pool decode step {s}")


@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4), (8, 1)])
def test_decode_over_an_fp8_pool_small(hq, hkv):
    pc = synth.make_pool_case("kv8", 6000 + hq + hkv, dtype="bf16", n_q_heads=hq, n_kv_heads=hkv, head_dim=128,
                              sink_len=70, pool_tokens=5000, demo_len_range=(30, 200), n_groups=5,
                              k_channel_sigma=0.5)
    sels = [[3, 0], [], [4, 1, 2, 0, 3], [2]] + [[1, 4]] * 36        # 40 queries: items with more users than columns
    qc = synth.make_query_case("kv8q", 6001, pc, n_queries=40, q_len=[64, 37, 100, 1] + [9] * 36, selections=sels,
                               n_decode=3)
    _decode_case(pc, qc, range(3), what=f"Hq={hq} Hkv={hkv}")


def test_fp8_decode_rejects_what_it_does_not_implement():
    pc = synth.make_pool_case("kv8r", 6010, dtype="bf16", n_q_heads=6, n_kv_heads=2, head_dim=128, sink_len=8,
                              pool_tokens=600, demo_len_range=(30, 100), n_groups=2)      # 3 query heads per KV head
    qc = synth.make_query_case("kv8rq", 6011, pc, n_queries=2, q_len=4, n_select=1, n_decode=1)
    p = pc.pool
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                              sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, block_m=32, block_n=64)
    k8, ks = quantise_per_head(to_dev(pc.k))
    shp = qc.k_cache.shape
    kc = to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
    with pytest.raises(B.DbsaError) as ei:
        B.dbsa_decode_attn_kv8(lay, to_dev(qc.dec_q[0]), kc, kc, torch.ones(2, dtype=torch.int32, device="cuda"), k8, k8,
                               ks, ks, pc.scale)
    assert ei.value.code == B.DBSA_ERR_UNSUPPORTED


def test_decode_over_an_fp8_pool_config3_full_size():
    pc = synth.config2_pool()
    qc = synth.config3_query(pc)
    _decode_case(pc, qc, (0, 31), queries=(0, 7, 15), what="cfg3")


@pytest.mark.parametrize("hq,hkv", [(8, 2), (4, 4)])
def test_repositioned_decode_over_an_fp8_pool(hq, hkv):
    """Re-positioning (Sec. 2.2) over a quantised pool: the keys are rotated at their encoding
    ids, THEN quantised.  The oracle gets the de-quantised keys rotated back in fp64 (a rotation
    is undone by the opposite angle), i.e. the un-rotated keys whose encoding-time rotation
    gives exactly the stored values, and rotates them at the new in-order ids itself."""
    from oracle import rope_oracle as ro
    pc = synth.make_pool_case("kv8rope", 6020 + hq, dtype="bf16", n_q_heads=hq, n_kv_heads=hkv, head_dim=128,
                              sink_len=70, pool_tokens=4000, demo_len_range=(30, 200), n_groups=5,
                              k_channel_sigma=0.5)
    sels = [[3, 0], [], [4, 1, 2, 0, 3], [2]] + [[4, 1]] * 20
    qc = synth.make_query_case("kv8ropeq", 6021, pc, n_queries=24, q_len=[64, 37, 100, 1] + [9] * 20, selections=sels,
                               n_decode=2)
    p = pc.pool
    f = ro.inv_freq(500000.0, 128)
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                              sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=32, block_n=64)
    tab = B.dbsa_rope_table(f, 2 * p.n_tokens + 200)
    k8, ks = quantise_per_head(B.dbsa_rope_apply(to_dev(pc.k), tab, first_id=0))
    v8, vs = quantise_per_head(to_dev(pc.v))
    k_unrot = ro.rope(dequantise(k8, ks), -np.arange(p.n_tokens), f)
    vq = dequantise(v8, vs)
    shp = qc.k_cache.shape
    cache_pos = torch.from_numpy(np.tile(np.arange(shp[1], dtype=np.int32), shp[0])).cuda()
    kc = B.dbsa_rope_apply(to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])), tab, positions=cache_pos).view(shp)
    vc = to_dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    lens = np.diff(qc.cu_qlens)
    for s in range(2):
        self_len = (lens + s + 1).astype(np.int32)
        od = B.dbsa_decode_attn_kv8(lay, to_dev(qc.dec_q[s]), kc, vc, torch.from_numpy(self_len).cuda(), k8, v8, ks, vs,
                                    pc.scale, rope_table=tab)
        ref = ro.decode_attn_repositioned(synth.as_f64(qc.dec_q[s]), synth.as_f64(qc.k_cache), synth.as_f64(qc.v_cache),
                                          self_len, k_unrot, vq, p.sink_len, p.demo_offsets, p.group_demo_offsets,
                                          qc.sel_ptr, qc.sel_idx, f, pc.scale)
        assert_close(to_f64(od), ref, f"Hq={hq} Hkv={hkv} re-positioned fp8-pool decode step {s}")


def test_fp8_decode_takes_the_rescale_path_when_row_maxima_keep_growing():
    """Keys ramped along a fixed direction inside every segment and queries along that direction:
    the scores of a run rise by more than the kernel's rescale slack from one half tile to the
    next (forward walk; the backward walk of the other step starts at the maximum)."""
    rng = np.random.default_rng(78)
    pc = synth.make_pool_case("kv8ramp", 6030, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, sink_len=64,
                              pool_tokens=3000, demo_len_range=(32, 128), n_groups=3)
    p = pc.pool
    u = rng.standard_normal(128).astype(np.float32)
    u /= np.linalg.norm(u)
    c = 32.0
    top = 200.0 / (pc.scale * c)
    gb = p.group_token_bounds()
    ramp = np.zeros(p.n_tokens, dtype=np.float32)
    for a, b in [(0, p.sink_len)] + [(int(gb[g]), int(gb[g + 1])) for g in range(p.n_groups)]:
        ramp[a:b] = np.arange(b - a, dtype=np.float32) / max(1, b - a - 1)
    k = ramp[:, None, None] * top * u[None, None, :] + 0.3 * rng.standard_normal(pc.k.shape).astype(np.float32)
    pc.k = synth.f32_to_bf16_bits(k)
    qc = synth.make_query_case("kv8rampq", 6031, pc, n_queries=12, q_len=20, n_select=2, n_decode=2)
    qc.dec_q = synth.f32_to_bf16_bits(c * u[None, None, None, :] + rng.standard_normal(qc.dec_q.shape).astype(np.float32))
    _decode_case(pc, qc, range(2), what="ramped keys")


def test_decode_over_an_fp8_pool_config4_full_size():
    """128 concurrent queries at 30 %: a group serves ~40 of them, so the step runs the kernel whose
    four waves share (and share the widening of) an item's half tiles."""
    pc = synth.config2_pool()
    qc = synth.config4_query(pc, 0.30)
    _decode_case(pc, qc, (0,), queries=(0, 31, 64, 127), what="cfg4 30 %")
