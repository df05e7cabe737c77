"""Pins for oracle/rope_oracle.py: each check reaches the expected value by a route that does
not go through the oracle's own formula (rotation matrices, complex arithmetic, a library
attention routine over an explicitly built sequence, the already-pinned query oracle)."""
import numpy as np
import pytest
import torch

from oracle import dbsa_oracle as orc
from oracle import rope_oracle as ro
from paper_2503_08640_amd import synth


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def test_two_channels_is_the_plane_rotation_matrix():
    rng = np.random.default_rng(0)
    x = _rand(rng, 5, 3, 2)
    pos = np.array([0, 1, 2, 7, 100])
    w = np.array([0.3])
    got = ro.rope(x, pos, w)
    for t, p in enumerate(pos):
        c, s = np.cos(p * 0.3), np.sin(p * 0.3)
        rot = np.array([[c, -s], [s, c]])
        assert np.allclose(got[t], x[t] @ rot.T, atol=1e-14)


def test_position_zero_is_identity_norms_are_kept_and_frequencies_fall_geometrically():
    rng = np.random.default_rng(1)
    x = _rand(rng, 4, 2, 16)
    f = ro.inv_freq(10000.0, 16)
    assert f[0] == 1.0 and np.allclose(f[1:] / f[:-1], 10000.0 ** (-2.0 / 16)) and np.isclose(f[-1], 10000.0 ** (-14 / 16))
    assert np.array_equal(ro.rope(x, np.zeros(4, dtype=int), f), x)
    y = ro.rope(x, np.array([3, 50, 1000, 90000]), f)
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)


def test_rotation_is_complex_multiplication_on_the_channel_pairs():
    """(x_i, x_{i+D/2}) as the complex number x_i + j x_{i+D/2}, times e^{j p w_i}."""
    rng = np.random.default_rng(2)
    d = 12
    x = _rand(rng, 6, 2, d)
    pos = rng.integers(0, 5000, size=6)
    f = ro.inv_freq(500000.0, d)
    z = (x[..., : d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * pos[:, None, None] * f[None, None, :])
    want = np.concatenate([z.real, z.imag], axis=-1)
    assert np.allclose(ro.rope(x, pos, f), want, atol=1e-12)
    # pairing neighbouring channels (2i, 2i+1) instead is a different function
    zi = (x[..., 0::2] + 1j * x[..., 1::2]) * np.exp(1j * pos[:, None, None] * f[None, None, :])
    inter = np.empty_like(x)
    inter[..., 0::2], inter[..., 1::2] = zi.real, zi.imag
    assert np.abs(inter - want).max() > 0.1


def test_scores_depend_on_position_differences_only():
    rng = np.random.default_rng(3)
    d = 8
    q, k = _rand(rng, 1, 1, d), _rand(rng, 1, 1, d)
    f = ro.inv_freq(10000.0, d)
    s = [float(ro.rope(q, [m], f)[0, 0] @ ro.rope(k, [n], f)[0, 0]) for m, n in ((9, 4), (105, 100), (5, 0))]
    assert np.allclose(s, s[0], atol=1e-12)
    assert not np.isclose(float(ro.rope(q, [9], f)[0, 0] @ ro.rope(k, [5], f)[0, 0]), s[0])


def _tiny_case(seed, hq=4, hkv=2, d=8):
    rng = np.random.default_rng(seed)
    pool = synth.uniform_pool(sink_len=3, n_demos=8, demo_len=5, demos_per_group=2)   # 4 groups of 10 tokens
    n = pool.n_tokens
    k_pool, v_pool = _rand(rng, n, hkv, d), _rand(rng, n, hkv, d)
    cu = np.array([0, 6, 7, 11])
    q, ks, vs = _rand(rng, 11, hq, d), _rand(rng, 11, hkv, d), _rand(rng, 11, hkv, d)
    return pool, k_pool, v_pool, cu, q, ks, vs


def test_query_stage_equals_dense_causal_attention_over_the_concatenated_sequence():
    """Sec. 2.2 read literally: [sink ; selected groups ; query] is an ordinary prompt with
    position ids 0, 1, 2, ...; the query rows of dense causal attention over it (library
    routine, complex-number rotary) are the answer."""
    pool, k_pool, v_pool, cu, q, ks, vs = _tiny_case(10)
    hq, hkv, d = q.shape[1], k_pool.shape[1], q.shape[2]
    f = ro.inv_freq(10000.0, d)
    sels = [[2, 0], [], [3, 1, 2]]
    sel_ptr = np.concatenate([[0], np.cumsum([len(s) for s in sels])])
    sel_idx = np.concatenate([np.asarray(s, dtype=np.int64) for s in sels])
    got = ro.query_attn_repositioned(q, ks, vs, k_pool, v_pool, pool.sink_len, pool.demo_offsets,
                                     pool.group_demo_offsets, cu, sel_ptr, sel_idx, f, 0.37)
    gb = pool.group_token_bounds()

    def crope(x, pos):
        z = (x[..., : d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * np.asarray(pos)[:, None, None] * f[None, None, :])
        return np.concatenate([z.real, z.imag], axis=-1)

    for u, sel in enumerate(sels):
        t0, t1 = cu[u], cu[u + 1]
        idx = list(range(pool.sink_len)) + [j for g in sel for j in range(gb[g], gb[g + 1])]
        k_seq = np.concatenate([k_pool[idx], ks[t0:t1]])
        v_seq = np.concatenate([v_pool[idx], vs[t0:t1]])
        n_seq = len(k_seq)
        q_seq = np.zeros((n_seq, hq, d))
        q_seq[len(idx):] = q[t0:t1]
        pos = np.arange(n_seq)
        qt = torch.from_numpy(crope(q_seq, pos)).permute(1, 0, 2)
        kt = torch.from_numpy(crope(k_seq, pos)).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)
        vt = torch.from_numpy(v_seq).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)
        dense = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, is_causal=True, scale=0.37)
        assert np.allclose(got[t0:t1], dense.permute(1, 0, 2).numpy()[len(idx):], atol=1e-12), u


def test_all_groups_in_pool_order_keeps_the_encoding_positions():
    """Selecting every group in pool order gives each key the id it was encoded with, so the
    result must equal the position-free query oracle on tensors rotated at those ids."""
    pool, k_pool, v_pool, cu, q, ks, vs = _tiny_case(11)
    d = q.shape[2]
    f = ro.inv_freq(10000.0, d)
    g = pool.n_groups
    sel_ptr = np.arange(0, 3 * g + 1, g)
    sel_idx = np.tile(np.arange(g), 3)
    got = ro.query_attn_repositioned(q, ks, vs, k_pool, v_pool, pool.sink_len, pool.demo_offsets,
                                     pool.group_demo_offsets, cu, sel_ptr, sel_idx, f, 0.5)
    n = pool.n_tokens
    local = np.concatenate([np.arange(cu[u + 1] - cu[u]) for u in range(3)])
    want = orc.query_attn(ro.rope(q, n + local, f), ro.rope(ks, n + local, f), vs, ro.rope(k_pool, np.arange(n), f),
                          v_pool, pool.sink_len, pool.demo_offsets, pool.group_demo_offsets, cu, sel_ptr, sel_idx, 0.5)
    assert np.allclose(got, want, atol=1e-12)
    # and the order of the selection now matters (positions move), unlike the position-free stage
    sel_rev = np.tile(np.arange(g)[::-1], 3)
    other = ro.query_attn_repositioned(q, ks, vs, k_pool, v_pool, pool.sink_len, pool.demo_offsets,
                                       pool.group_demo_offsets, cu, sel_ptr, sel_rev, f, 0.5)
    assert np.abs(other - got).max() > 1e-3


def test_decode_step_is_the_last_row_of_a_prefill_over_the_same_tokens():
    pool, k_pool, v_pool, cu, q, ks, vs = _tiny_case(12)
    d = q.shape[2]
    f = ro.inv_freq(10000.0, d)
    sels = [[1, 3], [0], [2, 1]]
    sel_ptr = np.concatenate([[0], np.cumsum([len(s) for s in sels])])
    sel_idx = np.concatenate([np.asarray(s, dtype=np.int64) for s in sels])
    pre = ro.query_attn_repositioned(q, ks, vs, k_pool, v_pool, pool.sink_len, pool.demo_offsets,
                                     pool.group_demo_offsets, cu, sel_ptr, sel_idx, f, 0.4)
    lens = np.diff(cu)
    t_max = int(lens.max())
    kc = np.zeros((3, t_max) + ks.shape[1:])
    vc = np.zeros_like(kc)
    for u in range(3):
        kc[u, : lens[u]] = ks[cu[u]:cu[u + 1]]
        vc[u, : lens[u]] = vs[cu[u]:cu[u + 1]]
    q_last = q[cu[1:] - 1]
    dec = ro.decode_attn_repositioned(q_last, kc, vc, lens, k_pool, v_pool, pool.sink_len, pool.demo_offsets,
                                      pool.group_demo_offsets, sel_ptr, sel_idx, f, 0.4)
    assert np.allclose(dec, pre[cu[1:] - 1], atol=1e-12)


@pytest.mark.parametrize("shift", [1, 17])
def test_rotating_the_query_back_instead_of_the_keys_forward(shift):
    """The identity the GPU path rests on: <R(m) q, R(n + s) k> = <R(m - s) q, R(n) k>."""
    rng = np.random.default_rng(20 + shift)
    d = 16
    f = ro.inv_freq(500000.0, d)
    q, k = _rand(rng, 1, 1, d), _rand(rng, 7, 1, d)
    n = np.arange(7) + 40
    lhs = ro.rope(k, n + shift, f)[:, 0] @ ro.rope(q, [300], f)[0, 0]
    rhs = ro.rope(k, n, f)[:, 0] @ ro.rope(q, [300 - shift], f)[0, 0]
    assert np.allclose(lhs, rhs, atol=1e-12)
