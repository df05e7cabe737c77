"""CPU oracle for the query stage WITH re-positioning -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module.  It shares no code with the HIP library and never calls it.

What the paper states (Sec. 2.1, last paragraphs; Sec. 2.2): the pool is encoded with
sequential position ids and its keys are cached BEFORE the rotary transformation; for a
test query the caches of the anchor and of the selected groups are concatenated in order,
rotary position encoding is re-applied with new in-order position ids 0 .. |D'|-1, the
query is encoded with full attention to that cache (and causally to itself), and the
answer is generated token by token.

This module takes those steps literally, in fp64: gather the un-rotated keys of
[sink ; selected groups in the caller's order], rotate them at ids 0 .. |D'|-1, rotate the
query's own keys and its queries at ids |D'| + a, then one dense softmax.  No masks are
needed on the pool part (everything gathered is visible); the query's own part is causal.
numpy's matmul is the only library primitive.

Rotary convention: the one of the Llama models the paper runs (Sec. 3): channel i pairs
with channel i + D/2, angle = position * inv_freq[i]; ``inv_freq`` is an argument so that
any base or frequency scaling can be used.

Pins (tests/test_rope_oracle_pins.py): the 2x2 rotation matrix for D = 2, position 0 is the
identity, norms are kept, scores depend on position differences only, the rotation equals
multiplication by e^{i p w} on the complex pairs, the whole function equals dense causal
attention (a library routine) over the explicitly concatenated sequence, and with every
group selected in pool order it equals the already-pinned query oracle on keys rotated at
their encoding positions.  Nothing here is "parity unpinned".
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np


def inv_freq(base: float, head_dim: int) -> np.ndarray:
    """inv_freq[i] = base^(-2i/D), i = 0 .. D/2-1 (fp64)."""
    i = np.arange(head_dim // 2, dtype=np.float64)
    return np.float64(base) ** (-2.0 * i / head_dim)


def rope(x: np.ndarray, positions, freqs: np.ndarray) -> np.ndarray:
    """x [T, H, D] rotated at integer ``positions`` [T]: for every pair (i, i + D/2)
    (x_i, x_{i+D/2}) -> (x_i cos - x_{i+D/2} sin, x_{i+D/2} cos + x_i sin), angle = pos * freqs[i]."""
    x = np.asarray(x, dtype=np.float64)
    half = x.shape[-1] // 2
    ang = np.asarray(positions, dtype=np.float64)[:, None] * np.asarray(freqs, dtype=np.float64)[None, :]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def selected_token_ids(sink_len: int, demo_offsets, group_demo_offsets, selection) -> np.ndarray:
    """Pool token indices of [sink ; selected groups in the given order]: the concatenated
    cache D' of Sec. 2.2.  Its i-th entry gets the new position id i."""
    demo_offsets = np.asarray(demo_offsets, dtype=np.int64)
    group_demo_offsets = np.asarray(group_demo_offsets, dtype=np.int64)
    parts = [np.arange(sink_len, dtype=np.int64)]
    for g in selection:
        lo = demo_offsets[group_demo_offsets[int(g)]]
        hi = demo_offsets[group_demo_offsets[int(g) + 1]]
        parts.append(np.arange(lo, hi, dtype=np.int64))
    return np.concatenate(parts)


def _softmax_attend(q: np.ndarray, k: np.ndarray, v: np.ndarray, mask: Optional[np.ndarray], scale: float):
    s = scale * (q @ k.T)
    if mask is not None:
        s = np.where(mask, s, -np.inf)
    p = np.exp(s - s.max(axis=1, keepdims=True))
    return (p / p.sum(axis=1, keepdims=True)) @ v


def query_attn_repositioned(q_raw: np.ndarray, k_self_raw: np.ndarray, v_self: np.ndarray, k_pool_raw: np.ndarray,
                            v_pool: np.ndarray, sink_len: int, demo_offsets, group_demo_offsets, cu_qlens, sel_ptr,
                            sel_idx, freqs: np.ndarray, scale: float,
                            queries: Optional[Sequence[int]] = None) -> np.ndarray:
    """Prefill of the test queries against re-positioned caches.  All q/k inputs are
    UN-rotated.  Returns O [sum T, Hq, D]; rows of queries not in ``queries`` are NaN."""
    tot, hq, d = q_raw.shape
    hkv = k_pool_raw.shape[1]
    r = hq // hkv
    out = np.full((tot, hq, d), np.nan, dtype=np.float64)
    for u in (range(len(cu_qlens) - 1) if queries is None else queries):
        t0, t1 = int(cu_qlens[u]), int(cu_qlens[u + 1])
        t = t1 - t0
        ids = selected_token_ids(sink_len, demo_offsets, group_demo_offsets,
                                 sel_idx[int(sel_ptr[u]):int(sel_ptr[u + 1])])
        n_sel = len(ids)
        k_cat = rope(k_pool_raw[ids], np.arange(n_sel), freqs)              # new in-order ids 0 .. |D'|-1
        k_own = rope(k_self_raw[t0:t1], n_sel + np.arange(t), freqs)        # the query follows the cache
        q_rot = rope(q_raw[t0:t1], n_sel + np.arange(t), freqs)
        a = np.arange(t)
        mask = np.concatenate([np.ones((t, n_sel), dtype=bool), a[None, :] <= a[:, None]], axis=1)
        for h in range(hq):
            kk = np.concatenate([k_cat[:, h // r, :], k_own[:, h // r, :]], axis=0)
            vv = np.concatenate([v_pool[ids, h // r, :], v_self[t0:t1, h // r, :]], axis=0)
            out[t0:t1, h, :] = _softmax_attend(q_rot[:, h, :], kk, vv, mask, scale)
    return out


def decode_attn_repositioned(q_step_raw: np.ndarray, k_cache_raw: np.ndarray, v_cache: np.ndarray, self_len,
                             k_pool_raw: np.ndarray, v_pool: np.ndarray, sink_len: int, demo_offsets,
                             group_demo_offsets, sel_ptr, sel_idx, freqs: np.ndarray, scale: float,
                             queries: Optional[Sequence[int]] = None) -> np.ndarray:
    """One generated token per query.  q_step_raw [B, Hq, D]; caches [B, Tmax, Hkv, D]
    un-rotated; self_len[u] counts the query's own keys including the new token, which sits
    at position |D'| + self_len[u] - 1 and attends the whole re-positioned cache and all of
    its own keys."""
    b, hq, d = q_step_raw.shape
    hkv = k_pool_raw.shape[1]
    r = hq // hkv
    out = np.full((b, hq, d), np.nan, dtype=np.float64)
    for u in (range(b) if queries is None else queries):
        ids = selected_token_ids(sink_len, demo_offsets, group_demo_offsets,
                                 sel_idx[int(sel_ptr[u]):int(sel_ptr[u + 1])])
        n_sel, n_own = len(ids), int(self_len[u])
        k_cat = rope(k_pool_raw[ids], np.arange(n_sel), freqs)
        k_own = rope(k_cache_raw[u, :n_own], n_sel + np.arange(n_own), freqs)
        q_rot = rope(q_step_raw[u][None], [n_sel + n_own - 1], freqs)[0]    # [Hq, D]
        for h in range(hq):
            kk = np.concatenate([k_cat[:, h // r, :], k_own[:, h // r, :]], axis=0)
            vv = np.concatenate([v_pool[ids, h // r, :], v_cache[u, :n_own, h // r, :]], axis=0)
            out[u, h, :] = _softmax_attend(q_rot[h][None, :], kk, vv, None, scale)[0]
    return out
