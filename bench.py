#!/usr/bin/env python3
"""Benchmark of the DBSA attention hot path on one MI355X.

One step = one pass of the whole path over one batch of seeded synthetic input at
the 90k-token / 30 %-retrieval workload: pre-encode layout build + block-sparse
pre-encode attention over the 90k pool (Llama-3.1-8B shape, GQA 32/8 x 128), then
query layout build + query prefill (16 queries x 64 tokens, 7 of 22 groups each)
+ 32 split-KV decode steps against the same selections.  Inputs are resident in
HBM before the timed region.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# tokens per Q tile (x 4 query heads of one KV head per workgroup); 32-token queries (config 4) take 32-token tiles
from paper_2503_08640_amd.binding import BENCH_BLOCK_M_PREENCODE as PRE_BLOCK_M  # noqa: E402
from paper_2503_08640_amd.binding import BENCH_BLOCK_M_QUERY as QUERY_BLOCK_M  # noqa: E402
from paper_2503_08640_amd.binding import BENCH_BLOCK_M_SHORT_QUERY as SHORT_QUERY_BLOCK_M  # noqa: E402


def visible_pairs_pre(pool, prev_window: int = 0) -> int:
    """Closed-form count of visible (row, key) pairs of the stage-1 pattern: sink triangle +
    per group L*(S + the w groups before it) + L(L+1)/2."""
    s = int(pool.sink_len)
    lens = np.diff(pool.group_token_bounds()).astype(np.int64)
    csum = np.concatenate([[0], np.cumsum(lens)])
    g = np.arange(len(lens))
    prev = csum[g] - csum[np.maximum(g - prev_window, 0)]
    return s * (s + 1) // 2 + int((lens * (s + prev) + lens * (lens + 1) // 2).sum())


def selected_keys(pool, qc) -> np.ndarray:
    lens = np.diff(pool.group_token_bounds()).astype(np.int64)
    return np.array([pool.sink_len + int(lens[qc.sel_idx[qc.sel_ptr[u]:qc.sel_ptr[u + 1]]].sum())
                     for u in range(qc.n_queries)], dtype=np.int64)


MIN_STAGE_LAUNCHES = 50     # timed launches behind every headline stage figure


def load_traffic():
    """HBM bytes per launch counted offline with rocprofv3 --pmc (profiles/hbm_traffic.json, written by
    `python -m paper_2503_08640_amd.profsum`).  The file carries the commit and a digest of the kernel sources it
    was measured at: if the sources in this tree differ, the figures are stale and every one reads as None."""
    from paper_2503_08640_amd import profsum
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        rec = json.load(open(path))
    except Exception:
        return {}, None
    at = {"git_commit": rec.get("git_commit"), "sources_sha256": rec.get("sources_sha256"),
          "current": rec.get("sources_sha256") == profsum.kernel_sources_digest()}
    if not at["current"]:
        return {}, at
    return {k: v.get("bytes_per_launch") for k, v in rec.items() if isinstance(v, dict)}, at


def launch_samples(torch, fn, n: int, warmup: int = 3):
    """ms of n single launches of fn, each bracketed by its own pair of events on the launch stream."""
    for _ in range(warmup):
        fn()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return [a.elapsed_time(b) for a, b in ev]


def stats(samples):
    x = np.asarray(samples, dtype=np.float64)
    return {"n": int(x.size), "mean_ms": float(x.mean()), "median_ms": float(np.median(x)), "min_ms": float(x.min())}


def affine_fit(keys, t):
    """t = alpha + beta * keys by least squares -> (alpha ms, beta ms per key, R^2)."""
    keys, t = np.asarray(keys, dtype=np.float64), np.asarray(t, dtype=np.float64)
    beta, alpha = np.polyfit(keys, t, 1)
    r2 = 1.0 - float(((t - (alpha + beta * keys)) ** 2).sum()) / float(((t - t.mean()) ** 2).sum())
    return {"alpha_ms": float(alpha), "beta_us_per_key": float(beta) * 1e3, "r2": r2,
            "t10_over_t100": float(t[0] / t[-1]), "keys10_over_keys100": float(keys[0] / keys[-1]),
            "t10_minus_alpha_over_t100_minus_alpha": float((t[0] - alpha) / (t[-1] - alpha))}


def extra_setting(torch, B, pc, qc, workload: str, bm_pre: int, bm_query: int, iters: int = 10):
    """Pre-encode, query prefill and one decode step of another workload through the same entry
    points and kernels.  Timed outside the benchmark step; reported beside it."""
    p, w = pc.pool, pc.prev_window
    hq, hkv, d = pc.n_q_heads, pc.n_kv_heads, pc.head_dim

    def dev(x):
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)

    q, k, v = dev(pc.q), dev(pc.k), dev(pc.v)
    o = torch.empty_like(q)
    qs, ks, vs = dev(qc.q), dev(qc.k), dev(qc.v)
    oq = torch.empty_like(qs)
    shp = qc.k_cache.shape
    kc, vc = dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp), dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    dq = dev(qc.dec_q.reshape(-1, hq, d)).view(qc.dec_q.shape)
    od = torch.empty_like(dq[0])
    lens = np.diff(qc.cu_qlens)
    self_len = torch.from_numpy((lens + 1).astype(np.int32)).cuda()
    lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, w, block_m=bm_pre, block_n=64)
    layq = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, w, cu_qlens=qc.cu_qlens,
                               sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=bm_query, block_n=64)
    ws = torch.empty(max(16, layq.workspace_bytes(hq, d)), dtype=torch.uint8, device="cuda")
    # adding the last group to a pool that already holds the others (Sec. 1: constant cost per addition)
    lay_app = B.dbsa_layout_build_append(p.sink_len, p.demo_offsets, p.group_demo_offsets, w, p.n_groups - 1,
                                         block_m=bm_pre, block_n=64)
    # the same pre-encode call on head-major storage ([heads, tokens, D] behind the same [tokens, heads, D] strides:
    # how caches are often kept); a 64-key tile then spans 16 KiB of addresses instead of 64 x heads x 256 bytes
    qh, kh, vh = (t.permute(1, 0, 2).contiguous().permute(1, 0, 2) for t in (q, k, v))
    oh = torch.empty_like(qh)
    calls = (lambda: B.dbsa_preencode_attn(lay, q, k, v, pc.scale, out=o),
             lambda: B.dbsa_query_attn(layq, qs, ks, vs, k, v, pc.scale, out=oq, workspace=ws),
             lambda: B.dbsa_decode_attn(layq, dq[0], kc, vc, self_len, k, v, pc.scale, out=od, workspace=ws),
             lambda: B.dbsa_preencode_attn(lay_app, q, k, v, pc.scale, out=o),
             lambda: B.dbsa_preencode_attn(lay, qh, kh, vh, pc.scale, out=oh))
    # medians over single launches (the inputs above were drawn on the host: the warm-up lets the clocks come back up)
    st = [stats(launch_samples(torch, fn, max(n, MIN_STAGE_LAUNCHES))) for fn, n in zip(calls, (iters, 4 * iters, 20 * iters, 4 * iters, iters))]
    ms = [x["median_ms"] for x in st]
    keys = selected_keys(p, qc)
    flops_pre = 4.0 * d * visible_pairs_pre(p, w) * hq
    flops_query = 4.0 * d * hq * float((lens * keys).sum() + (lens * (lens + 1) // 2).sum())
    bytes_dec = float((keys + lens + 1).sum()) * hkv * d * 2 * 2
    return {
        "workload": workload, "heads": f"{hq}/{hkv} x {d}", "block_m_preencode": bm_pre, "block_m_query": bm_query,
        "pool_tokens": int(p.n_tokens), "sink_len": int(p.sink_len), "n_groups": int(p.n_groups), "prev_window": w,
        "preencode_ms": ms[0], "preencode_useful_tflops": flops_pre / ms[0] / 1e9,
        "preencode_frac_of_mfma_peak": flops_pre / ms[0] / 1e9 / PEAK_BF16_TFLOPS,
        "preencode_head_major_ms": ms[4], "preencode_head_major_frac_of_mfma_peak": flops_pre / ms[4] / 1e9 / PEAK_BF16_TFLOPS,
        "query_prefill_ms": ms[1], "query_prefill_useful_tflops": flops_query / ms[1] / 1e9,
        "query_prefill_frac_of_mfma_peak": flops_query / ms[1] / 1e9 / PEAK_BF16_TFLOPS,
        "decode_step_ms": ms[2], "decode_per_query_gbs": bytes_dec / ms[2] / 1e6,
        "append_last_group_ms": ms[3],
        "timing": "median of single launches", "launch_stats": dict(zip(("preencode", "query_prefill", "decode_step", "append", "preencode_head_major"), st)),
    }


def config4_sweep(torch, B, pc, k, v, iters: int = 20):
    """Config 4: 128 concurrent queries x 32 prompt tokens + 1 decode token over the config-2 pool at 10 / 30 /
    50 / 100 % of the groups per query: query prefill, one decode step, and both per unit of retrieval ratio."""
    from paper_2503_08640_amd import synth
    p = pc.pool
    hq, hkv, d = pc.n_q_heads, pc.n_kv_heads, pc.head_dim

    def dev(x):
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)

    rows = []
    # rotary table for the re-positioned decode step (timing only: the keys are used as they are)
    tab = B.dbsa_rope_table(500000.0 ** (-np.arange(0, d, 2, dtype=np.float64) / d), 2 * p.n_tokens + 256)
    for ratio in synth.RETRIEVAL_RATIOS:
        qc = synth.config4_query(pc, ratio)
        qs, ks, vs = dev(qc.q), dev(qc.k), dev(qc.v)
        oq = torch.empty_like(qs)
        shp = qc.k_cache.shape
        kc = dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp)
        vc = dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
        dq = dev(qc.dec_q.reshape(-1, hq, d)).view(qc.dec_q.shape)
        od = torch.empty_like(dq[0])
        lens = np.diff(qc.cu_qlens)
        self_len = torch.from_numpy((lens + 1).astype(np.int32)).cuda()
        lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                                  sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=SHORT_QUERY_BLOCK_M, block_n=64)
        ws = torch.empty(max(16, lay.workspace_bytes(hq, d)), dtype=torch.uint8, device="cuda")
        st = [stats(launch_samples(torch, fn, n)) for fn, n in
              ((lambda: B.dbsa_query_attn(lay, qs, ks, vs, k, v, pc.scale, out=oq, workspace=ws), max(iters, MIN_STAGE_LAUNCHES)),
               (lambda: B.dbsa_decode_attn(lay, dq[0], kc, vc, self_len, k, v, pc.scale, out=od, workspace=ws),
                max(5 * iters, MIN_STAGE_LAUNCHES)))]
        ms = [x["median_ms"] for x in st]
        rope_ms = stats(launch_samples(torch, lambda: B.dbsa_decode_attn_rope(lay, dq[0], kc, vc, self_len, k, v, tab, pc.scale,
                                                                              out=od, workspace=ws), MIN_STAGE_LAUNCHES))["median_ms"]
        keys = selected_keys(p, qc)
        flops = 4.0 * d * hq * float((lens * keys).sum() + (lens * (lens + 1) // 2).sum())
        # a decode row scores and weighs every key it attends: 4 D flops per (query head, key)
        flops_dec = 4.0 * d * hq * float((keys + lens + 1).sum())
        glens = np.diff(p.group_token_bounds()).astype(np.int64)
        union = p.sink_len + int(glens[np.unique(qc.sel_idx)].sum())
        unique_bytes = (union + float((lens + 1).sum())) * hkv * d * 2 * 2
        rows.append({"retrieval_ratio": ratio, "groups_per_query": int(qc.sel_ptr[1]), "mean_keys_per_query": float(keys.mean()),
                     "query_prefill_ms": ms[0], "query_prefill_useful_tflops": flops / ms[0] / 1e9,
                     "decode_step_ms": ms[1], "decode_step_repositioned_ms": rope_ms,
                     "decode_useful_tflops": flops_dec / ms[1] / 1e9,
                     "decode_frac_of_mfma_peak": flops_dec / ms[1] / 1e9 / PEAK_BF16_TFLOPS,
                     "decode_unique_gbs": unique_bytes / ms[1] / 1e6,
                     "decode_frac_of_hbm_peak_unique_bytes": unique_bytes / ms[1] / 1e6 / PEAK_HBM_GBS,
                     "decode_effective_gbs": float((keys + lens + 1).sum()) * hkv * d * 2 * 2 / ms[1] / 1e6,
                     "query_stage_ms": ms[0] + ms[1], "query_stage_ms_per_ratio": (ms[0] + ms[1]) / ratio,
                     "launch_stats": {"query_prefill": st[0], "decode_step": st[1]}})
        lay.destroy()
    mk = [r["mean_keys_per_query"] for r in rows]
    full = rows[-1]
    return {"workload": "config 4: 128 queries x (32 prompt tokens + 1 decode token) over the config-2 pool, "
                        "independent random selections", "timing": "median of single launches", "rows": rows,
            # cost against the keys one query retrieves (Sec. 1: proportional to the retrieval ratio): alpha is what
            # a smaller selection does not shrink.  The decode step fetches a group once for all queries that
            # selected it, and 128 random selections cover nearly the whole pool at every ratio: its alpha is the
            # time to stream that union once
            "fit_vs_keys": {"query_prefill": affine_fit(mk, [r["query_prefill_ms"] for r in rows]),
                            "decode_step": affine_fit(mk, [r["decode_step_ms"] for r in rows]),
                            "query_stage": affine_fit(mk, [r["query_stage_ms"] for r in rows])},
            # at 100 % retrieval every one of the 128 queries scores the whole pool: a dense contraction
            "roofline_decode_many_queries": {
                "kernel": "attn_prefill64_kernel<4,2,false,true,true,false> (pool items as a contraction: 64 queries per wave, rows "
                          "gathered through the schedule's references) + decode_group_kernel (own caches) + "
                          "decode_group_merge_kernel, 100 % retrieval", "bound": "mfma", "achieved": full["decode_useful_tflops"],
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": full["decode_frac_of_mfma_peak"], "traffic": None,
                "algorithmic": {"useful_tflop_per_step": full["decode_useful_tflops"] * full["decode_step_ms"] / 1e3,
                                "step_ms": full["decode_step_ms"]}}}


def repositioned_stage(torch, B, pc, qc, k, v, qs, ks, vs, oq, dq, kc, vc, self_len, od, plain_query_ms,
                       plain_decode_ms, iters: int = 20):
    """Query prefill and one decode step of config 3 through the *_rope entry points (timing only:
    the tensors of the benchmark step stand in for un-rotated Q and encoding-rotated K)."""
    p = pc.pool
    d = pc.head_dim
    layq = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                               sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=QUERY_BLOCK_M, block_n=64)
    inv_freq = 500000.0 ** (-2.0 * np.arange(d // 2, dtype=np.float64) / d)      # Llama-3.1 rotary base
    n_pos = 2 * p.n_tokens + int(np.diff(qc.cu_qlens).max()) + qc.n_decode + 1
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    tab = B.dbsa_rope_table(inv_freq, n_pos)
    e1.record()
    torch.cuda.synchronize()
    table_ms = e0.elapsed_time(e1)
    e0.record()
    B.dbsa_rope_apply(k, tab, out=torch.empty_like(k))
    e1.record()
    torch.cuda.synchronize()
    rotate_pool_ms = e0.elapsed_time(e1)
    ws = torch.empty(max(16, layq.workspace_bytes(pc.n_q_heads, d)), dtype=torch.uint8, device="cuda")
    calls = (lambda: B.dbsa_query_attn_rope(layq, qs, ks, vs, k, v, tab, pc.scale, out=oq, workspace=ws),
             lambda: B.dbsa_decode_attn_rope(layq, dq[0], kc, vc, self_len, k, v, tab, pc.scale, out=od, workspace=ws))
    ms = []
    for fn, n in zip(calls, (iters, 5 * iters)):
        fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms.append(e0.elapsed_time(e1) / n)
    return {
        "workload": "config 3 query stage with re-positioning: Q rotated per segment inside the kernels, one shared "
                    "key tensor rotated at its encoding ids",
        "query_prefill_ms": ms[0], "query_prefill_ms_without": plain_query_ms,
        "decode_step_ms": ms[1], "decode_step_ms_without": plain_decode_ms,
        "rope_table_ms_once": table_ms, "rope_table_rows": n_pos, "rotate_pool_keys_ms_once": rotate_pool_ms,
    }


def cpu_baseline(pc, n_rows: int = 512):
    """The fp64 oracle, as it stands, on a bounded sample of pre-encode rows."""
    from oracle import dbsa_oracle as orc
    from paper_2503_08640_amd import synth
    p = pc.pool
    rng = np.random.default_rng(4242)
    rows = np.sort(rng.choice(p.n_tokens, size=n_rows, replace=False))
    q, k, v = synth.as_f64(pc.q), synth.as_f64(pc.k), synth.as_f64(pc.v)
    t0 = time.perf_counter()
    orc.preencode_attn(q, k, v, p.sink_len, p.demo_offsets, p.group_demo_offsets, pc.scale,
                       pc.prev_window, rows=rows)
    dt = time.perf_counter() - t0
    gb = p.group_token_bounds()
    g = np.searchsorted(gb, rows, side="right") - 1
    vis = np.where(rows < p.sink_len, rows + 1, p.sink_len + rows - gb[np.maximum(g, 0)] + 1)
    flops = 4.0 * pc.head_dim * float(vis.sum()) * pc.n_q_heads
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": f"pre-encode, {n_rows} seeded random rows x {pc.n_q_heads} heads, each scored densely in fp64 "
                      f"against all {p.n_tokens} keys ({dt:.1f} s); useful (visible-pair) flops counted",
            "rows_per_s": n_rows / dt}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-paper-setting", action="store_true",
                    help="skip the extra measurements (outside the timed step) of the paper's own pool structure and "
                         "of the 30k MHA setting")
    ap.add_argument("--only", choices=("mha30k", "config4", "paper"),
                    help="run ONE of the extra settings and nothing else (no benchmark step): what a profiler run of that "
                         "setting uses, so that its kernels are not mixed with the step's")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 256 MiB device copy, the known-size kernel the HBM counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (no multi-GPU path exists)", file=sys.stderr)
        return 2

    import torch
    from paper_2503_08640_amd import binding as B
    from paper_2503_08640_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.lib()  # fail loudly if the HIP library is not built

    def paper_extra():
        # the pool structure the paper itself runs (Sec. 3: blocks of 50 demonstrations, first block = sink,
        # two preceding blocks visible, 30 % of the blocks per query)
        pp = synth.paper_setting_pool()
        return extra_setting(
            torch, B, pp, synth.paper_setting_query(pp),
            "paper setting: 2400 demos / 90k tokens in 48 blocks of 50, sink = first block, window 2; "
            "16 queries x 64 tokens, 14 of 47 blocks each, first decode step", PRE_BLOCK_M, QUERY_BLOCK_M)

    def mha_extra():
        # the paper's other efficiency setting (Sec. 3: 30k pool, Llama-2-7B MHA shape) = config 1 + a query stage
        p1 = synth.config1_pool()
        return extra_setting(
            torch, B, p1, synth.mha30k_query(p1),
            "config 1 pool (32k tokens, 8 groups, sink 64, MHA) + query stage: 16 queries x 64 tokens, "
            "2 of 8 groups each, first decode step", 128, 64)

    if args.only in ("mha30k", "paper"):
        print(json.dumps({"only": args.only, "setting": mha_extra() if args.only == "mha30k" else paper_extra()}), flush=True)
        return 0

    # ---- seeded synthetic inputs, resident in HBM ----
    pc = synth.config2_pool()
    qc = synth.config3_query(pc)
    p = pc.pool

    def dev(x):
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)

    q, k, v = dev(pc.q), dev(pc.k), dev(pc.v)
    if args.only == "config4":
        print(json.dumps({"only": args.only, "setting": config4_sweep(torch, B, pc, k, v)}), flush=True)
        return 0
    o = torch.empty_like(q)
    qs, ks, vs = dev(qc.q), dev(qc.k), dev(qc.v)
    oq = torch.empty_like(qs)
    shp = qc.k_cache.shape
    kc, vc = dev(qc.k_cache.reshape(-1, shp[2], shp[3])).view(shp), dev(qc.v_cache.reshape(-1, shp[2], shp[3])).view(shp)
    dq = dev(qc.dec_q.reshape(-1, pc.n_q_heads, pc.head_dim)).view(qc.dec_q.shape)
    od = torch.empty_like(dq[0])
    lens = np.diff(qc.cu_qlens)
    self_lens = [torch.from_numpy((lens + s + 1).astype(np.int32)).cuda() for s in range(qc.n_decode)]
    hq, hkv, d = pc.n_q_heads, pc.n_kv_heads, pc.head_dim

    # ---- algorithmic work of one step ----
    pairs_pre = visible_pairs_pre(p)
    keys = selected_keys(p, qc)
    t_q = int(lens[0])
    flops_pre = 4.0 * d * pairs_pre * hq
    flops_query = 4.0 * d * hq * float((lens * keys).sum() + (lens * (lens + 1) // 2).sum())
    flops_decode = sum(4.0 * d * hq * float((keys + lens + s + 1).sum()) for s in range(qc.n_decode))
    bytes_decode_step = float((keys + lens + (qc.n_decode + 1) / 2.0).sum()) * hkv * d * 2 * 2
    flops_step = flops_pre + flops_query + flops_decode
    # bytes a decode step must move when a group selected by several queries is fetched once
    glens = np.diff(p.group_token_bounds()).astype(np.int64)
    union_keys = p.sink_len + int(glens[np.unique(qc.sel_idx)].sum())
    bytes_decode_unique = (union_keys + float((lens + (qc.n_decode + 1) / 2.0).sum())) * hkv * d * 2 * 2

    ws_holder = {}

    def step(ev=None):
        # a1 + a3: both layouts are built (host lists + one upload each) before any kernel is queued
        t0 = time.perf_counter()
        lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, block_m=PRE_BLOCK_M,
                                  block_n=64)
        layq = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                                   sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=QUERY_BLOCK_M,
                                   block_n=64)
        t1 = time.perf_counter()
        need = layq.workspace_bytes(hq, d)
        if ws_holder.get("n", 0) < need:
            ws_holder["t"] = torch.empty(need, dtype=torch.uint8, device="cuda")
            ws_holder["n"] = need
        if ev: ev[0].record()
        B.dbsa_preencode_attn(lay, q, k, v, pc.scale, out=o)                                        # a2
        if ev: ev[1].record()
        if ev: ev[2].record()
        B.dbsa_query_attn(layq, qs, ks, vs, k, v, pc.scale, out=oq, workspace=ws_holder["t"])     # a4
        if ev: ev[3].record()
        for s in range(qc.n_decode):                                                                # a5 + a6
            B.dbsa_decode_attn(layq, dq[s], kc, vc, self_lens[s], k, v, pc.scale, out=od, workspace=ws_holder["t"])
        if ev: ev[4].record()
        return t1 - t0

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calib_copy:
        src = torch.empty(256 * 1024 * 1024, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(args.steps)]
    layout_s = 0.0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        layout_s += step(evs[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    ms_step = elapsed * 1e3 / args.steps
    # per-launch durations from the events inside the timed region (mean = what the roofline rows use) ...
    pre_s = [e[0].elapsed_time(e[1]) for e in evs]
    query_s = [e[2].elapsed_time(e[3]) for e in evs]
    decode_s = [e[3].elapsed_time(e[4]) / qc.n_decode for e in evs]
    pre_ms, query_ms, decode_ms = float(np.mean(pre_s)), float(np.mean(query_s)), float(np.mean(decode_s))
    pre_tflops = flops_pre / pre_ms / 1e9
    dec_gbs = bytes_decode_step / decode_ms / 1e6
    # ... topped up, after the timed region, to at least MIN_STAGE_LAUNCHES single launches per stage for the
    # median / min figures (same layouts, tensors and entry points)
    extra = max(0, MIN_STAGE_LAUNCHES - args.steps)
    if extra:
        lay = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, block_m=PRE_BLOCK_M, block_n=64)
        layq = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                                   sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=QUERY_BLOCK_M, block_n=64)
        wsb = ws_holder["t"]
        pre_s += launch_samples(torch, lambda: B.dbsa_preencode_attn(lay, q, k, v, pc.scale, out=o), extra)
        query_s += launch_samples(torch, lambda: B.dbsa_query_attn(layq, qs, ks, vs, k, v, pc.scale, out=oq, workspace=wsb), extra)
        mid = qc.n_decode // 2
        decode_s += launch_samples(torch, lambda: B.dbsa_decode_attn(layq, dq[mid], kc, vc, self_lens[mid], k, v, pc.scale,
                                                                     out=od, workspace=wsb), extra)
        lay.destroy()
        layq.destroy()
    # host time of the two layout builds alone (lists only, no device block, no upload)
    t0 = time.perf_counter()
    for _ in range(5):
        B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, block_m=PRE_BLOCK_M, block_n=64,
                            host_only=True).destroy()
        B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens, sel_ptr=qc.sel_ptr,
                            sel_idx=qc.sel_idx, n_split=0, block_m=QUERY_BLOCK_M, block_n=64, host_only=True).destroy()
    layout_host_ms = (time.perf_counter() - t0) * 1e3 / 5
    # ... and of the two builds with their device blocks and uploads while the GPU is idle.  Inside the timed steps
    # the host runs ahead of the GPU; a build then waits for a list block of a destroyed layout to come free (the
    # library keeps 16), so layout_build_ms_per_step there mostly measures that wait, which overlaps kernels
    layout_idle = []
    for _ in range(5):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        la = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, 0, block_m=PRE_BLOCK_M, block_n=64)
        lb = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens, sel_ptr=qc.sel_ptr,
                                 sel_idx=qc.sel_idx, n_split=0, block_m=QUERY_BLOCK_M, block_n=64)
        layout_idle.append((time.perf_counter() - t0) * 1e3)
        la.destroy()
        lb.destroy()
    layout_idle_ms = float(np.median(layout_idle))
    traffic, traffic_at = load_traffic()

    out = {
        "metric": "useful attn TFLOP/s + query-stage ms @90k-token pool, 30% retrieval, 1 GPU",
        "value": flops_step / (ms_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": "config 2 pre-encode (90k pool, GQA 32/8 x 128, 22 groups, sink 64) + config 3 query stage "
                        "(16 queries x 64 tokens, 7 of 22 groups each, 32 decode steps)",
            "pool_tokens": int(p.n_tokens), "n_groups": int(p.n_groups), "n_queries": int(qc.n_queries),
            "query_len": t_q, "groups_per_query": int(qc.sel_ptr[1]), "decode_steps": int(qc.n_decode),
            "block_m_preencode": PRE_BLOCK_M, "block_m_query": QUERY_BLOCK_M, "block_n": 64,
        },
        "stages": {
            "preencode_ms": pre_ms, "preencode_useful_tflops": pre_tflops,
            "query_prefill_ms": query_ms, "query_prefill_useful_tflops": flops_query / query_ms / 1e9,
            "decode_step_ms": decode_ms, "query_stage_ms": query_ms + decode_ms * qc.n_decode,
            "layout_build_ms_per_step": layout_s * 1e3 / args.steps, "layout_build_host_lists_only_ms": layout_host_ms,
            "layout_build_idle_gpu_ms": layout_idle_ms,
            "useful_tflop_per_step": flops_step / 1e12,
            # mean over the timed region above; median / min over >= MIN_STAGE_LAUNCHES launches (timed region + top-up)
            "launch_stats": {"preencode": stats(pre_s), "query_prefill": stats(query_s), "decode_step": stats(decode_s)},
        },
        "roofline": {
            "kernel": "attn_prefill64_kernel<4,2,false,true,false,false> (pre-encode launch: persistent, four waves of 64 query rows "
                      "per workgroup, one workgroup per compute unit; the <4,2,true,*,false,*> instances serve the query prefill)",
            "bound": "mfma", "achieved": pre_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": pre_tflops / PEAK_BF16_TFLOPS, "traffic": traffic.get("preencode"),
            "traffic_measured_at": traffic_at,
            "algorithmic": {"useful_tflop_per_launch": flops_pre / 1e12, "launch_ms": pre_ms,
                            "launch_ms_median": stats(pre_s)["median_ms"], "launch_ms_min": stats(pre_s)["min_ms"],
                            "frac_at_median": flops_pre / stats(pre_s)["median_ms"] / 1e9 / PEAK_BF16_TFLOPS},
        },
        "roofline_query_prefill": {
            "kernel": "attn_prefill64_kernel<4,2,true,false,false,false> + prefill_merge_kernel (16 Q tiles x 8 head blocks, lists cut in two)",
            "bound": "mfma", "achieved": flops_query / query_ms / 1e9, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": flops_query / query_ms / 1e9 / PEAK_BF16_TFLOPS, "traffic": traffic.get("query_prefill"),
            "algorithmic": {"useful_tflop_per_launch": flops_query / 1e12, "launch_ms": query_ms,
                            "note": "the launch re-reads pool K/V across its Q tiles (mostly from L2): traffic above the "
                                    "unique bytes is expected while the kernel is matrix-bound"},
        },
        "roofline_decode": {
            "kernel": "decode_group_kernel + decode_group_merge_kernel (one decode step)", "bound": "hbm",
            # algorithmic bytes = the UNIQUE bytes of a step: the group-major schedule fetches a group once for all
            # the queries that selected it, so that is what has to cross the HBM interface
            "achieved": bytes_decode_unique / decode_ms / 1e6, "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": bytes_decode_unique / decode_ms / 1e6 / PEAK_HBM_GBS,
            "traffic": traffic.get("decode_step"),
            # bytes counted once per query that reads them (what a query-major schedule would move) over the same
            # time: a rate of work, not of memory traffic, and not bounded by the HBM peak
            "effective_gbs": dec_gbs,
            "algorithmic": {"unique_gb_per_step": bytes_decode_unique / 1e9, "per_query_gb_per_step": bytes_decode_step / 1e9,
                            "step_ms": decode_ms, "step_ms_median": stats(decode_s)["median_ms"],
                            "step_ms_min": stats(decode_s)["min_ms"]},
        },
    }
    if not args.no_paper_setting:
        # config 3 again, with the new in-order position ids of Sec. 2.2 applied inside the kernels
        out["repositioned_query_stage"] = repositioned_stage(torch, B, pc, qc, k, v, qs, ks, vs, oq, dq, kc, vc,
                                                             self_lens[0], od, query_ms, decode_ms)
        # config 3's decode step over the same pool stored as 8-bit floats (timing only: values are re-quantised
        # copies of the benchmark's pool, one scale per KV head)
        k8, v8 = k.to(torch.float8_e4m3fn), v.to(torch.float8_e4m3fn)
        ones = torch.ones(hkv, dtype=torch.float32, device="cuda")
        layq8 = B.dbsa_layout_build(p.sink_len, p.demo_offsets, p.group_demo_offsets, cu_qlens=qc.cu_qlens,
                                    sel_ptr=qc.sel_ptr, sel_idx=qc.sel_idx, n_split=0, block_m=QUERY_BLOCK_M, block_n=64)
        for _ in range(4):
            B.dbsa_decode_attn_kv8(layq8, dq[0], kc, vc, self_lens[0], k8, v8, ones, ones, pc.scale, out=od,
                                   workspace=ws_holder["t"])
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(100):
            B.dbsa_decode_attn_kv8(layq8, dq[0], kc, vc, self_lens[0], k8, v8, ones, ones, pc.scale, out=od,
                                   workspace=ws_holder["t"])
        e1.record()
        torch.cuda.synchronize()
        ms8 = e0.elapsed_time(e1) / 100
        out["fp8_kv_decode"] = {
            "workload": "config 3 decode step, pool K/V stored as e4m3 bytes with one scale per KV head (self caches "
                        "bf16)", "decode_step_ms": ms8, "decode_step_ms_bf16_pool": decode_ms,
            "unique_gb_per_step": (union_keys * hkv * d * 2 * 1 + float((lens + 1).sum()) * hkv * d * 2 * 2) / 1e9,
        }
        del k8, v8
        out["config4_sweep"] = config4_sweep(torch, B, pc, k, v)
        out["paper_setting"] = paper_extra()
        out["mha30k_setting"] = mha_extra()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(pc)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
