"""Seeded synthetic inputs for the DBSA attention path.

This module only draws random numbers and lays out index arrays; it holds none
of the method's arithmetic (no masks, no softmax, no tiling).  Both the CPU
oracle's tests and the HIP path's tests/bench take their inputs from here so
that the two are compared on identical data.

The shapes follow the paper's two efficiency settings (Sec. 3 "Models":
Llama-2-7B MHA at a ~30k pool, Llama-3.1-8B GQA at a ~90k pool; Sec. 3
"Configuration": demonstrations are packed into groups, a fixed fraction of
groups is retrieved per query).  The paper's datasets are not used: the
attention operator's cost depends on shapes and the mask only.

Conventions
-----------
* tokens ``[0, S)`` are the attention-sink prefix; pool tokens follow.
* ``demo_offsets[n_demos+1]``: token offsets, ``demo_offsets[0] == S``.
* ``group_demo_offsets[n_groups+1]``: demo indices, first 0, last n_demos.
* bf16 values are carried as ``uint16`` bit patterns (round-to-nearest-even).
* tensors are token-major ``[tokens, heads, D]``.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

# --------------------------------------------------------------------------
# dtype plumbing (representation only)
# --------------------------------------------------------------------------


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest-even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounding = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rounding) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def as_f64(x: np.ndarray) -> np.ndarray:
    """Up-cast a stored tensor (fp32 values or bf16 bit patterns) to fp64."""
    if x.dtype == np.uint16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return np.asarray(x, dtype=np.float64)


# --------------------------------------------------------------------------
# pool structure
# --------------------------------------------------------------------------


@dataclass
class Pool:
    sink_len: int
    demo_offsets: np.ndarray        # int32 [n_demos+1]
    group_demo_offsets: np.ndarray  # int32 [n_groups+1]

    @property
    def n_tokens(self) -> int:
        return int(self.demo_offsets[-1])

    @property
    def n_demos(self) -> int:
        return len(self.demo_offsets) - 1

    @property
    def n_groups(self) -> int:
        return len(self.group_demo_offsets) - 1

    def group_token_bounds(self) -> np.ndarray:
        """int32 [n_groups+1]: first token of each group, then N."""
        return self.demo_offsets[self.group_demo_offsets].astype(np.int32)


def draw_demo_lengths(rng: np.random.Generator, pool_tokens: int, lo: int, hi: int) -> np.ndarray:
    """Integer lengths U[lo, hi] until the sum reaches ``pool_tokens``; the last
    demo is cut to land exactly on it, and folded into its predecessor when the
    cut leaves it shorter than ``lo``."""
    lens: List[int] = []
    total = 0
    while total < pool_tokens:
        n = int(rng.integers(lo, hi + 1))
        lens.append(n)
        total += n
    lens[-1] -= total - pool_tokens
    if lens[-1] < lo and len(lens) > 1:
        tail = lens.pop()
        lens[-1] += tail
    return np.asarray(lens, dtype=np.int64)


def pack_groups(sink_len: int, demo_lens: np.ndarray, n_groups: int) -> Pool:
    """Close group g at the demo boundary nearest to ``S + (g+1)*P/G`` (ties to
    the lower boundary); the last group ends at the last demo."""
    offs = np.concatenate([[sink_len], sink_len + np.cumsum(demo_lens)]).astype(np.int64)
    pool_tokens = int(offs[-1]) - sink_len
    gdo = [0]
    for g in range(n_groups - 1):
        target = sink_len + (g + 1) * pool_tokens / n_groups
        dist = np.abs(offs - target)
        b = int(np.argmin(dist))  # argmin returns the first (lower) boundary on ties
        if b <= gdo[-1]:
            b = gdo[-1] + 1
        gdo.append(b)
    gdo.append(len(demo_lens))
    gdo_arr = np.asarray(gdo, dtype=np.int32)
    assert np.all(np.diff(gdo_arr) > 0), "pool too small for the requested group count"
    return Pool(sink_len, offs.astype(np.int32), gdo_arr)


def uniform_pool(sink_len: int, n_demos: int, demo_len: int, demos_per_group: int) -> Pool:
    offs = sink_len + demo_len * np.arange(n_demos + 1)
    gdo = np.arange(0, n_demos + 1, demos_per_group)
    assert gdo[-1] == n_demos
    return Pool(sink_len, offs.astype(np.int32), gdo.astype(np.int32))


# --------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------


def _normal(rng: np.random.Generator, shape, chunk_rows: int = 8192) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(shape[0], -1)
    for r0 in range(0, shape[0], chunk_rows):
        r1 = min(shape[0], r0 + chunk_rows)
        flat[r0:r1] = rng.standard_normal((r1 - r0, flat.shape[1]), dtype=np.float32)
    return out


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    assert dtype == "f32"
    return np.ascontiguousarray(x, dtype=np.float32)


def select_count(ratio: float, n_groups: int) -> int:
    return max(1, int(np.floor(ratio * n_groups + 0.5)))


def draw_selections(rng: np.random.Generator, n_queries: int, n_groups: int, m: int):
    """Per query: m distinct groups, uniform without replacement, ascending.
    Returned as CSR (sel_ptr, sel_idx), both int32."""
    idx = []
    for _ in range(n_queries):
        idx.append(np.sort(rng.choice(n_groups, size=m, replace=False)))
    sel_ptr = (m * np.arange(n_queries + 1)).astype(np.int32)
    sel_idx = np.concatenate(idx).astype(np.int32) if idx else np.zeros(0, np.int32)
    return sel_ptr, sel_idx


@dataclass
class PoolCase:
    """Stage-1 inputs: one pool and its post-RoPE Q/K/V."""
    name: str
    seed: int
    dtype: str          # "bf16" | "f32"
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    scale: float
    pool: Pool
    q: np.ndarray       # [N, Hq, D]
    k: np.ndarray       # [N, Hkv, D]
    v: np.ndarray       # [N, Hkv, D]
    prev_window: int = 0


@dataclass
class QueryCase:
    """Stage-2 inputs over a pool case's K/V."""
    name: str
    seed: int
    cu_qlens: np.ndarray    # int32 [B+1]
    sel_ptr: np.ndarray     # int32 [B+1]
    sel_idx: np.ndarray     # int32 [nnz]
    q: np.ndarray           # [sum T, Hq, D]
    k: np.ndarray           # [sum T, Hkv, D]
    v: np.ndarray           # [sum T, Hkv, D]
    # decode: step s (0-based) uses dec_q[s] and the self cache filled up to
    # self_len = T_u + s + 1; the cache already holds every token's K/V.
    n_decode: int = 0
    t_max: int = 0
    dec_q: Optional[np.ndarray] = None      # [n_decode, B, Hq, D]
    k_cache: Optional[np.ndarray] = None    # [B, t_max, Hkv, D]
    v_cache: Optional[np.ndarray] = None    # [B, t_max, Hkv, D]

    @property
    def n_queries(self) -> int:
        return len(self.cu_qlens) - 1


def make_pool_case(name: str, seed: int, *, dtype: str, n_q_heads: int, n_kv_heads: int, head_dim: int,
                   sink_len: int, pool_tokens: int, demo_len_range=None, n_groups: int = 1,
                   uniform_demo_len: Optional[int] = None, demos_per_group: Optional[int] = None,
                   k_channel_sigma: float = 0.0, prev_window: int = 0) -> PoolCase:
    """Draw order: demo lengths, Q, K, V, K channel scales."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if uniform_demo_len is not None:
        pool = uniform_pool(sink_len, pool_tokens // uniform_demo_len, uniform_demo_len, demos_per_group)
    else:
        lo, hi = demo_len_range
        pool = pack_groups(sink_len, draw_demo_lengths(rng, pool_tokens, lo, hi), n_groups)
    n = pool.n_tokens
    q = _normal(rng, (n, n_q_heads, head_dim))
    k = _normal(rng, (n, n_kv_heads, head_dim))
    v = _normal(rng, (n, n_kv_heads, head_dim))
    if k_channel_sigma > 0.0:
        z = rng.standard_normal((n_kv_heads, head_dim)).astype(np.float32)
        k *= np.exp(np.float32(k_channel_sigma) * z)[None, :, :]
    return PoolCase(name, seed, dtype, n_q_heads, n_kv_heads, head_dim, 1.0 / float(np.sqrt(head_dim)),
                    pool, _store(q, dtype), _store(k, dtype), _store(v, dtype), prev_window)


def make_query_case(name: str, seed: int, pc: PoolCase, *, n_queries: int, q_len, n_select: Optional[int] = None,
                    selections=None, n_decode: int = 0) -> QueryCase:
    """Draw order: selections, query Q/K/V, decode q, decode K/V.
    ``q_len`` is an int (uniform) or a list of per-query lengths."""
    rng = np.random.Generator(np.random.PCG64(seed))
    if selections is None:
        sel_ptr, sel_idx = draw_selections(rng, n_queries, pc.pool.n_groups, n_select)
    else:
        sel_ptr = np.concatenate([[0], np.cumsum([len(s) for s in selections])]).astype(np.int32)
        sel_idx = (np.concatenate([np.asarray(s, np.int32) for s in selections])
                   if sel_ptr[-1] > 0 else np.zeros(0, np.int32))
    lens = np.full(n_queries, q_len, dtype=np.int64) if np.isscalar(q_len) else np.asarray(q_len, np.int64)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    tot = int(cu[-1])
    hq, hkv, d = pc.n_q_heads, pc.n_kv_heads, pc.head_dim
    q = _store(_normal(rng, (tot, hq, d)), pc.dtype)
    k = _store(_normal(rng, (tot, hkv, d)), pc.dtype)
    v = _store(_normal(rng, (tot, hkv, d)), pc.dtype)
    qc = QueryCase(name, seed, cu, sel_ptr, sel_idx, q, k, v)
    if n_decode > 0:
        t_max = int(lens.max()) + n_decode
        dec_q = _store(_normal(rng, (n_decode * n_queries, hq, d)), pc.dtype).reshape(n_decode, n_queries, hq, d)
        dk = _store(_normal(rng, (n_decode * n_queries, hkv, d)), pc.dtype).reshape(n_decode, n_queries, hkv, d)
        dv = _store(_normal(rng, (n_decode * n_queries, hkv, d)), pc.dtype).reshape(n_decode, n_queries, hkv, d)
        kc = np.zeros((n_queries, t_max, hkv, d), dtype=k.dtype)
        vc = np.zeros((n_queries, t_max, hkv, d), dtype=v.dtype)
        for u in range(n_queries):
            t = int(lens[u])
            kc[u, :t] = k[cu[u]:cu[u + 1]]
            vc[u, :t] = v[cu[u]:cu[u + 1]]
            kc[u, t:t + n_decode] = dk[:, u]
            vc[u, t:t + n_decode] = dv[:, u]
        qc.n_decode, qc.t_max, qc.dec_q, qc.k_cache, qc.v_cache = n_decode, t_max, dec_q, kc, vc
    return qc


# --------------------------------------------------------------------------
# the five workload configurations
# --------------------------------------------------------------------------

RETRIEVAL_RATIOS = (0.10, 0.30, 0.50, 1.00)


def config0_pool() -> PoolCase:
    """Tiny fp32 case: 4-token sink, 8 demos x 32 tokens, 2 groups of 4."""
    return make_pool_case("cfg0", 1000, dtype="f32", n_q_heads=2, n_kv_heads=2, head_dim=64, sink_len=4,
                          pool_tokens=256, uniform_demo_len=32, demos_per_group=4)


def config0_query(pc: PoolCase) -> QueryCase:
    """One 16-token query selecting group index 1."""
    return make_query_case("cfg0q", 1000 + 500, pc, n_queries=1, q_len=16, selections=[[1]], n_decode=2)


def config1_pool(pool_tokens: int = 32768, n_groups: int = 8) -> PoolCase:
    """Llama-2-7B shape: MHA 32 x 128, 64-token sink, demos U[32,128]."""
    return make_pool_case("cfg1", 1001, dtype="bf16", n_q_heads=32, n_kv_heads=32, head_dim=128, sink_len=64,
                          pool_tokens=pool_tokens, demo_len_range=(32, 128), n_groups=n_groups)


def config2_pool(pool_tokens: int = 90112, n_groups: int = 22) -> PoolCase:
    """Llama-3.1-8B shape: GQA 32/8 x 128, 64-token sink, demos U[32,256],
    K scaled per channel by exp(0.5 z)."""
    return make_pool_case("cfg2", 1002, dtype="bf16", n_q_heads=32, n_kv_heads=8, head_dim=128, sink_len=64,
                          pool_tokens=pool_tokens, demo_len_range=(32, 256), n_groups=n_groups,
                          k_channel_sigma=0.5)


def config3_query(pc: PoolCase, n_queries: int = 16, q_len: int = 64, ratio: float = 0.30,
                  n_decode: int = 32) -> QueryCase:
    return make_query_case("cfg3", 1003, pc, n_queries=n_queries, q_len=q_len,
                           n_select=select_count(ratio, pc.pool.n_groups), n_decode=n_decode)


def mha30k_query(pc: PoolCase, n_queries: int = 16, q_len: int = 64, ratio: float = 0.30,
                 n_decode: int = 32) -> QueryCase:
    """Query stage over the config-1 pool (the paper's 30k / Llama-2-7B MHA setting, Sec. 3):
    30 % of 8 groups = 2 groups per query."""
    return make_query_case("mha30k", 1007, pc, n_queries=n_queries, q_len=q_len,
                           n_select=select_count(ratio, pc.pool.n_groups), n_decode=n_decode)


def config4_query(pc: PoolCase, ratio: float, n_queries: int = 128, q_len: int = 32) -> QueryCase:
    # one seed per ratio so that the four sweeps are independent draws
    seed = 1004 + 10 * RETRIEVAL_RATIOS.index(ratio) if ratio in RETRIEVAL_RATIOS else 1004
    return make_query_case(f"cfg4_r{int(round(ratio * 100))}", seed, pc, n_queries=n_queries, q_len=q_len,
                           n_select=select_count(ratio, pc.pool.n_groups), n_decode=1)


# --------------------------------------------------------------------------
# the paper's own pool structure (Sec. 3 implementation details; Sec. 5.2 patterns)
# --------------------------------------------------------------------------


def block_pool(demo_lens: np.ndarray, demos_per_block: int, sink_is_first_block: bool = True) -> Pool:
    """Blocks of ``demos_per_block`` consecutive demos (the last block takes the remainder).
    With ``sink_is_first_block`` the first block becomes the sink prefix and the remaining
    blocks the groups; otherwise there is no sink and every block is a group."""
    lens = np.asarray(demo_lens, dtype=np.int64)
    n_sink = min(demos_per_block, len(lens) - 1) if sink_is_first_block else 0
    sink_len = int(lens[:n_sink].sum())
    rest = lens[n_sink:]
    offs = np.concatenate([[sink_len], sink_len + np.cumsum(rest)])
    gdo = list(range(0, len(rest), demos_per_block))
    if len(rest) - gdo[-1] < max(1, demos_per_block // 2) and len(gdo) > 1:
        gdo.pop()                      # a short remainder joins the block before it
    gdo.append(len(rest))
    return Pool(sink_len, offs.astype(np.int32), np.asarray(gdo, dtype=np.int32))


def make_block_pool_case(name: str, seed: int, *, n_demos: int, demos_per_block: int, demo_len_range,
                         prev_window: int, sink_is_first_block: bool = True, dtype: str = "bf16",
                         n_q_heads: int = 32, n_kv_heads: int = 8, head_dim: int = 128,
                         k_channel_sigma: float = 0.5) -> PoolCase:
    """Draw order: demo lengths, Q, K, V, K channel scales (as make_pool_case)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    lo, hi = demo_len_range
    pool = block_pool(rng.integers(lo, hi + 1, size=n_demos), demos_per_block, sink_is_first_block)
    n = pool.n_tokens
    q = _normal(rng, (n, n_q_heads, head_dim))
    k = _normal(rng, (n, n_kv_heads, head_dim))
    v = _normal(rng, (n, n_kv_heads, head_dim))
    if k_channel_sigma > 0.0:
        z = rng.standard_normal((n_kv_heads, head_dim)).astype(np.float32)
        k *= np.exp(np.float32(k_channel_sigma) * z)[None, :, :]
    return PoolCase(name, seed, dtype, n_q_heads, n_kv_heads, head_dim, 1.0 / float(np.sqrt(head_dim)),
                    pool, _store(q, dtype), _store(k, dtype), _store(v, dtype), prev_window)


def paper_setting_pool(n_demos: int = 2400, demos_per_block: int = 50) -> PoolCase:
    """The 90k setting as the paper runs it (Sec. 3): 2400 demonstrations of ~37 tokens in
    blocks of 50, the first block is the attention sink, every block also sees the two
    blocks before it.  Llama-3.1-8B head shape, synthetic values as in config 2."""
    return make_block_pool_case("paper90k", 1005, n_demos=n_demos, demos_per_block=demos_per_block,
                                demo_len_range=(28, 47), prev_window=2)


def paper_setting_query(pc: PoolCase, n_queries: int = 16, q_len: int = 64, ratio: float = 0.30,
                        n_decode: int = 32) -> QueryCase:
    """30 % of the blocks per query (the sink block is always present), then decode."""
    return make_query_case("paper90k_q", 1006, pc, n_queries=n_queries, q_len=q_len,
                           n_select=select_count(ratio, pc.pool.n_groups), n_decode=n_decode)
