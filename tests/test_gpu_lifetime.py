"""Layout lifetime on the GPU: building, using and destroying layouts never waits for the
device, so the lists of a destroyed layout must stay intact until the kernels that read
them have finished, and a call on another stream must see the uploaded lists."""
import numpy as np
import pytest
import torch

from paper_2503_08640_amd import binding as B
from paper_2503_08640_amd import synth
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def _case():
    pc = synth.make_pool_case("lifepool", 5100, dtype="bf16", n_q_heads=8, n_kv_heads=2, head_dim=128, sink_len=64,
                              pool_tokens=24000, demo_len_range=(30, 120), n_groups=12)
    sels_a = [[0, 3, 5, 7], [1, 2, 3, 4], [11, 10, 9, 8], [0, 1, 10, 11]]
    sels_b = [[2, 4, 6, 8], [5, 6, 7, 8], [0, 11, 5, 6], [3, 4, 7, 9]]
    qa = synth.make_query_case("lifeq_a", 5101, pc, n_queries=4, q_len=64, selections=sels_a, n_decode=1)
    qb = synth.make_query_case("lifeq_b", 5102, pc, n_queries=4, q_len=64, selections=sels_b, n_decode=1)
    return pc, qa, qb


def _build(pc, qc):
    p = pc.pool
    return B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                               sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, block_m=32, block_n=64)


def test_destroying_a_layout_right_after_the_launch_keeps_its_lists_alive():
    """Alternate two selections many times without ever synchronising: every layout is destroyed
    while its kernels are still queued and the next build wants a block of the same size.  All
    outputs must equal those of a run that synchronises around every call."""
    pc, qa, qb = _case()
    k, v = to_dev(pc.k), to_dev(pc.v)
    dev = {}
    for name, qc in (("a", qa), ("b", qb)):
        lens = np.diff(qc.cu_qlens)
        dev[name] = dict(q=to_dev(qc.q), ks=to_dev(qc.k), vs=to_dev(qc.v), dq=to_dev(qc.dec_q[0]),
                         kc=to_dev(qc.k_cache), vc=to_dev(qc.v_cache),
                         sl=torch.from_numpy((lens + 1).astype(np.int32)).cuda())
    want = {}
    for name, qc in (("a", qa), ("b", qb)):
        t = dev[name]
        lay = _build(pc, qc)
        torch.cuda.synchronize()
        oq = B.dbsa_query_attn(lay, t["q"], t["ks"], t["vs"], k, v, pc.scale)
        od = B.dbsa_decode_attn(lay, t["dq"], t["kc"], t["vc"], t["sl"], k, v, pc.scale)
        torch.cuda.synchronize()
        lay.destroy()
        want[name] = (oq.clone(), od.clone())
    # a long kernel first, so that everything below is queued behind running work
    pl = pc.pool
    lay_pre = B.dbsa_layout_build(pl.sink_len, pl.demo_offsets, pl.group_demo_offsets, 0, block_m=32, block_n=64)
    for _ in range(3):
        B.dbsa_preencode_attn(lay_pre, to_dev(pc.q), k, v, pc.scale)
    got = []
    for i in range(24):
        name, qc = (("a", qa), ("b", qb))[i % 2]
        t = dev[name]
        lay = _build(pc, qc)
        oq = B.dbsa_query_attn(lay, t["q"], t["ks"], t["vs"], k, v, pc.scale)
        od = B.dbsa_decode_attn(lay, t["dq"], t["kc"], t["vc"], t["sl"], k, v, pc.scale)
        lay.destroy()
        got.append((name, oq, od))
    lay_pre.destroy()
    torch.cuda.synchronize()
    for i, (name, oq, od) in enumerate(got):
        # the decode walk direction alternates per layout and both runs start it the same way
        assert torch.equal(oq, want[name][0]), f"query prefill of round {i} ({name}) differs"
        assert torch.equal(od, want[name][1]), f"decode step of round {i} ({name}) differs"


def test_a_call_on_another_stream_sees_the_uploaded_lists():
    pc, qa, _ = _case()
    k, v = to_dev(pc.k), to_dev(pc.v)
    q, ks, vs = to_dev(qa.q), to_dev(qa.k), to_dev(qa.v)
    lay = _build(pc, qa)
    torch.cuda.synchronize()
    want = B.dbsa_query_attn(lay, q, ks, vs, k, v, pc.scale)
    torch.cuda.synchronize()
    lay.destroy()
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(6):
        lay = _build(pc, qa)                        # lists copied on the default stream
        with torch.cuda.stream(side):
            got = B.dbsa_query_attn(lay, q, ks, vs, k, v, pc.scale)
        lay.destroy()                               # while the side stream may still be running
        side.synchronize()
        assert torch.equal(got, want)
    torch.cuda.synchronize()


def test_decode_steps_replayed_from_a_hip_graph_match_the_eager_steps():
    """Two decode steps (one per walk direction) captured into a HIP graph: the calls launch
    kernels only (no allocation, no memset, workspace from the caller), so replays, with eager
    work and synchronisations in between, must reproduce the eager results bit for bit."""
    pc, qa, _ = _case()
    k, v = to_dev(pc.k), to_dev(pc.v)
    lens = np.diff(qa.cu_qlens)
    shp = qa.k_cache.shape
    kc = to_dev(qa.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
    vc = to_dev(qa.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    dq = to_dev(qa.dec_q[0])
    sl = torch.from_numpy((lens + 1).astype(np.int32)).cuda()
    lay = _build(pc, qa)
    ws = torch.empty(lay.workspace_bytes(pc.n_q_heads, pc.head_dim), dtype=torch.uint8, device="cuda")
    out = [torch.empty_like(dq), torch.empty_like(dq)]
    # eager: the first decode call on a fresh layout walks backwards, the second forwards
    for o in out:
        B.dbsa_decode_attn(lay, dq, kc, vc, sl, k, v, pc.scale, out=o, workspace=ws)
    torch.cuda.synchronize()
    want = [o.clone() for o in out]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for o in out:
            B.dbsa_decode_attn(lay, dq, kc, vc, sl, k, v, pc.scale, out=o, workspace=ws)
    for rep in range(4):
        for o in out:
            o.fill_(float("nan"))
        ws.random_(0, 255)                              # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i in range(2):
            assert torch.equal(out[i], want[i]), f"replay {rep}, step {i}"
    lay.destroy()
