"""Pins for the oracle's RoPE variant (full equation of Sec. 3.2): rotated ReLU
features in the numerator, un-rotated ones in the denominator."""
import os

import numpy as np
import pytest

import sv_workloads as wl
from oracle import linattn_oracle as orc
from tests.brute import kernel_score_attention_rope, rotate_pairs
from tests.test_oracle_pins import _golden, _rand, _relerr


def _table(N, d, seed):
    """Arbitrary angles: nothing in the equation needs them to come from positions."""
    ang = np.random.default_rng(seed).uniform(-np.pi, np.pi, size=(N, d // 2))
    return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)


@pytest.mark.parametrize("N,d", [(1, 32), (5, 32), (33, 64), (130, 64)])
def test_rope_bidirectional_equals_two_matrix_bruteforce(N, d):
    Q, K, V = _rand(300 + N, 1, 2, N, d)
    T = _table(N, d, N)
    O, S, z = orc.bidirectional(Q, K, V, 1e-6, rope=T)
    for h in range(2):
        ref = kernel_score_attention_rope(Q[0, h], K[0, h], V[0, h], T, 1e-6)
        assert _relerr(O[0, h], ref) <= 1e-10
    # matrix-product form of the state: rotated keys for S, plain keys for z
    for h in range(2):
        pK = np.maximum(K[0, h].astype(np.float64), 0)
        assert _relerr(S[0, h], rotate_pairs(pK, T).T @ V[0, h].astype(np.float64)) <= 1e-12
        assert _relerr(z[0, h], pK.sum(axis=0)) <= 1e-12


def test_rope_block_stream_equals_masked_bruteforce():
    sizes = [3, 1, 6, 4]
    N, d = sum(sizes), 32
    Q, K, V = _rand(310, 1, 2, N, d)
    T = _table(N, d, 7)
    edges = np.concatenate([[0], np.cumsum(sizes)])
    blocks = [(Q[:, :, a:b], K[:, :, a:b], V[:, :, a:b]) for a, b in zip(edges[:-1], edges[1:])]
    ropes = [T[a:b] for a, b in zip(edges[:-1], edges[1:])]
    O = np.concatenate([o for o, _, _ in orc.block_stream(blocks, 1e-6, ropes=ropes)], axis=2)
    block_of = np.repeat(np.arange(len(sizes)), sizes)
    for h in range(2):
        ref = kernel_score_attention_rope(Q[0, h], K[0, h], V[0, h], T, 1e-6, block_of=block_of)
        assert _relerr(O[0, h], ref) <= 1e-10


def test_rope_hand_example():
    g = _golden("hand_example_rope.txt")
    eps = 1e-6
    Q = np.array([[1, 2], [3, -1]], np.float32).reshape(1, 1, 2, 2)
    K = np.array([[2, 0], [1, 1]], np.float32).reshape(1, 1, 2, 2)
    V = np.array([[1, 0], [0, 2]], np.float32).reshape(1, 1, 2, 2)
    T = np.array([[[1, 0]], [[0, 1]]], np.float32)          # angles 0 and 90 degrees
    O, S, z = orc.bidirectional(Q, K, V, eps, rope=T)
    np.testing.assert_array_equal(S.ravel(), g["S"])
    np.testing.assert_array_equal(z.ravel(), g["z"])
    np.testing.assert_allclose(O[0, 0, 0], g["num0"] / (g["den0"][0] + eps), rtol=1e-15)
    np.testing.assert_allclose(O[0, 0, 1], g["num1"] / (g["den1"][0] + eps), rtol=1e-15)


def test_zero_angles_reduce_to_the_plain_path_bitwise():
    Q, K, V = _rand(320, 2, 2, 40, 64)
    T = np.zeros((40, 32, 2), np.float32)
    T[..., 0] = 1.0
    a = orc.bidirectional(Q, K, V, 1e-6, rope=T)
    b = orc.bidirectional(Q, K, V, 1e-6)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))


def test_key_sum_and_denominator_ignore_the_rotation():
    Q, K, V = _rand(330, 1, 2, 25, 32)
    T = _table(25, 32, 3)
    O_r, S_r, z_r = orc.bidirectional(Q, K, V, 1e-6, rope=T)
    O_p, S_p, z_p = orc.bidirectional(Q, K, V, 1e-6)
    assert np.array_equal(z_r, z_p) and not np.array_equal(S_r, S_p)
    # same denominators: O_r * den == rotated numerators, O_p * den == plain numerators
    den = np.einsum("bhik,bhk->bhi", np.maximum(Q.astype(np.float64), 0), z_p)[..., None] + 1e-6
    num_r = np.einsum("bhik,bhkv->bhiv", np.stack([[rotate_pairs(np.maximum(Q[0, h].astype(np.float64), 0), T)
                                                    for h in range(2)]]), S_r)
    assert _relerr(O_r * den, num_r) <= 1e-12


def test_scores_depend_on_relative_position_only():
    """With angles = position * frequency, shifting every position by a constant leaves the
    numerator scores, hence O, unchanged (the defining property of a rotary embedding)."""
    N, d = 30, 32
    Q, K, V = _rand(340, 1, 1, N, d)
    freq = 10000.0 ** (-np.arange(d // 2) / (d // 2))
    pos = np.random.default_rng(1).integers(0, 50, size=N).astype(np.float64)

    def table(p):
        ang = p[:, None] * freq[None, :]
        return np.stack([np.cos(ang), np.sin(ang)], axis=-1)        # float64 here: exact shift test

    O1, _, _ = orc.bidirectional(Q, K, V, 1e-6, rope=table(pos).astype(np.float32))
    O2, _, _ = orc.bidirectional(Q, K, V, 1e-6, rope=table(pos + 17.0).astype(np.float32))
    assert _relerr(O2, O1) <= 1e-5          # tables are rounded to fp32: angles agree to ~1e-7


def test_rope_apply_range_and_state_ranges():
    Q, K, V = _rand(350, 1, 2, 50, 32)
    T = _table(50, 32, 5)
    O, S, z = orc.bidirectional(Q, K, V, 1e-6, rope=T)
    assert np.array_equal(orc.apply(Q, S, z, 1e-6, 7, 31, rope=T), O[:, :, 7:31])
    S1, z1 = orc.state(K, V, 0, 20, rope=T)
    S2, z2 = orc.state(K, V, 20, 50, S1, z1, rope=T)
    assert _relerr(S2, S) <= 1e-12 and _relerr(z2, z) <= 1e-12


def test_3d_table_generator():
    T = wl.rope_table_3d(3, 4, 5, 64)
    assert T.shape == (60, 32, 2) and T.dtype == np.float32
    np.testing.assert_allclose(T[..., 0] ** 2 + T[..., 1] ** 2, 1.0, atol=1e-6)
    assert (T[0, :, 0] == 1).all() and (T[0, :, 1] == 0).all()          # position (0,0,0): no rotation
    # token (t=1,r=0,c=0) rotates only the time pairs; (0,1,0) only the row pairs
    n_hw = (3 * 32) // 8
    n_t = 32 - 2 * n_hw
    t1, r1 = T[20], T[5]
    assert (t1[n_t:, 1] == 0).all() and (t1[:n_t, 1] != 0).all()
    assert (r1[:n_t, 1] == 0).all() and (r1[n_t:n_t + n_hw, 1] != 0).all() and (r1[n_t + n_hw:, 1] == 0).all()
    # blocks of a stream continue the time axis
    assert np.array_equal(wl.rope_table_3d(2, 4, 5, 64, t0=1), T[20:])


def test_factored_tables_expand_to_the_full_table():
    """The per-axis tables and the full table come from two separate generators; expanding the
    former by pure indexing must reproduce the latter bit for bit (this is what lets the GPU's
    factored-table entry points be checked against the oracle's full-table form)."""
    for (fr, ro, co, d, t0) in [(3, 5, 7, 64, 0), (2, 4, 3, 32, 5), (3, 6, 9, 112, 3), (1, 1, 1, 64, 0)]:
        cs_t, cs_h, cs_w = wl.rope_tables_3d_factored(fr, ro, co, d, t0=t0)
        assert cs_t.shape[1] + cs_h.shape[1] + cs_w.shape[1] == d // 2
        full = wl.expand_rope_tables(cs_t, cs_h, cs_w)
        ref = wl.rope_table_3d(fr, ro, co, d, t0=t0)
        assert full.shape == ref.shape and full.dtype == np.float32
        assert np.array_equal(full, ref)
