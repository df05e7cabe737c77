"""dbsa_decode_attn_static (the decode step that allocates nothing: partial states in the
library's fixed buffer) against dbsa_decode_attn, through the C ABI.

Two calls in a row share the buffer, the second on a smaller input; each is compared with the
workspace entry point bit for bit (two layouts of the same selections walk their keys in the
same direction on their n-th call, so the arithmetic is identical) and with the fp64 oracle
to the usual tolerance."""
import numpy as np
import pytest
import torch

from oracle import dbsa_oracle as orc
from paper_2503_08640_amd import binding as B
from paper_2503_08640_amd import synth

from gpu_util import assert_close, to_dev, to_f64

pytestmark = pytest.mark.gpu


def _case(seed, n_queries, q_len, n_select, hq=8, hkv=2):
    pc = synth.make_pool_case("na_pool", seed, dtype="bf16", n_q_heads=hq, n_kv_heads=hkv, head_dim=128, sink_len=64,
                              pool_tokens=6000, demo_len_range=(32, 200), n_groups=6, k_channel_sigma=0.5)
    qc = synth.make_query_case("na_q", seed + 1, pc, n_queries=n_queries, q_len=q_len, n_select=n_select, n_decode=2)
    return pc, qc


def _layout(pc, qc):
    p = pc.pool
    return B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                               sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=32, block_n=64)


def _step(pc, qc, step, what):
    p = pc.pool
    kp, vp = to_dev(pc.k), to_dev(pc.v)
    shp = qc.k_cache.shape
    kc = to_dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
    vc = to_dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    self_len = (np.diff(qc.cu_qlens) + step + 1).astype(np.int32)
    sl = torch.from_numpy(self_len).cuda()
    q = to_dev(qc.dec_q[step])
    lay_ws, lay_static = _layout(pc, qc), _layout(pc, qc)
    want = B.dbsa_decode_attn(lay_ws, q, kc, vc, sl, kp, vp, pc.scale)
    got = torch.full_like(q, float("nan"))
    before = torch.cuda.memory_allocated()
    B.dbsa_decode_attn_static(lay_static, q, kc, vc, sl, kp, vp, pc.scale, out=got)
    assert torch.cuda.memory_allocated() == before, "the call went through torch's allocator"
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), want.view(torch.int16)), f"{what}: differs from dbsa_decode_attn"
    ref = orc.decode_attn(synth.as_f64(qc.dec_q[step]), synth.as_f64(qc.k_cache), synth.as_f64(qc.v_cache), self_len,
                          synth.as_f64(pc.k), synth.as_f64(pc.v), p.sink_len, p.demo_offsets, p.group_demo_offsets,
                          qc.sel_ptr, qc.sel_idx, pc.scale)
    assert_close(to_f64(got), ref, what)


def test_static_decode_two_calls_second_smaller():
    big = _case(4100, n_queries=24, q_len=40, n_select=3)
    small = _case(4200, n_queries=3, q_len=[5, 70, 17], n_select=1)
    _step(*big, 0, "static decode, 24 queries x 3 groups")
    _step(*small, 1, "static decode, 3 queries x 1 group (after the larger call)")


def test_static_decode_rejects_what_does_not_fit():
    """A step whose partial states exceed the fixed buffer is refused before anything is launched."""
    pc, qc = _case(4300, n_queries=2, q_len=8, n_select=1)
    p = pc.pool
    # n_split = 4096 per query and 4096 query heads: 2 * 4096 slots * 4096 heads * 132 floats > 32 MiB
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                              sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=4096, block_m=32, block_n=64)
    q = torch.zeros(2, 4096, 128, dtype=torch.bfloat16, device="cuda")
    kc = torch.zeros(2, 16, 2, 128, dtype=torch.bfloat16, device="cuda")
    sl = torch.tensor([9, 9], dtype=torch.int32, device="cuda")
    with pytest.raises(B.DbsaError) as err:
        B.dbsa_decode_attn_static(lay, q, kc, kc, sl, to_dev(pc.k), to_dev(pc.v), pc.scale, out=torch.empty_like(q))
    assert err.value.code == B.DBSA_ERR_WORKSPACE
