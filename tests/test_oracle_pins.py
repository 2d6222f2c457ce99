"""Pins for the CPU oracle: what the paper and the mathematics fix, checked
without a GPU.  A plausible mistake anywhere in the oracle (dropped term, wrong
sign or index, transposed operand, exclusive instead of inclusive block sum,
eps in the wrong place) fails at least one of these.
"""
import os

import numpy as np
import pytest

import sv_workloads as wl
from oracle import linattn_oracle as orc
from tests.brute import kernel_score_attention, kernel_score_attention_dense

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(seed, B, H, N, d, scale=1.0):
    rng = np.random.default_rng(seed)
    return [(rng.standard_normal((B, H, N, d)) * scale).astype(np.float32) for _ in range(3)]


def _relerr(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.max(np.abs(a - b)) / max(1e-300, np.max(np.abs(b))))


# ---- P1: brute-force O(N^2) kernel-score attention --------------------------------------

@pytest.mark.parametrize("N,d", [(1, 32), (2, 32), (7, 64), (64, 32), (65, 64), (40, 112), (33, 128)])
def test_bidirectional_equals_bruteforce_small(N, d):
    Q, K, V = _rand(10 + N, 1, 2, N, d)
    O, _, _ = orc.bidirectional(Q, K, V, 1e-6)
    for h in range(2):
        ref = kernel_score_attention(Q[0, h], K[0, h], V[0, h], 1e-6)
        assert _relerr(O[0, h], ref) <= 1e-10


def test_bidirectional_equals_bruteforce_tiny_workload():
    """The fp32 validation workload itself (N=1024, d=32, 2 heads)."""
    w = wl.workload("tiny_f32")
    Q, K, V = wl.draw_qkv(w)
    O, _, _ = orc.bidirectional(Q, K, V, w.eps)
    for h in range(w.H):
        ref = kernel_score_attention_dense(Q[0, h], K[0, h], V[0, h], w.eps)
        assert _relerr(O[0, h], ref) <= 1e-10


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_block_stream_equals_masked_bruteforce(seed):
    """Random block partitions: block i sees blocks 0..i entirely (inclusive)."""
    rng = np.random.default_rng(100 + seed)
    d = [32, 64, 32][seed]
    sizes = rng.integers(1, 9, size=rng.integers(2, 6)).tolist()
    N = int(sum(sizes))
    Q, K, V = _rand(200 + seed, 1, 2, N, d)
    block_of = np.repeat(np.arange(len(sizes)), sizes)
    edges = np.concatenate([[0], np.cumsum(sizes)])
    blocks = [(Q[:, :, a:b], K[:, :, a:b], V[:, :, a:b]) for a, b in zip(edges[:-1], edges[1:])]
    outs = [o for o, _, _ in orc.block_stream(blocks, 1e-6)]
    O = np.concatenate(outs, axis=2)
    for h in range(2):
        ref = kernel_score_attention(Q[0, h], K[0, h], V[0, h], 1e-6, block_of=block_of)
        assert _relerr(O[0, h], ref) <= 1e-10
        # the loop and the dense brute force agree with each other too
        ref2 = kernel_score_attention_dense(Q[0, h], K[0, h], V[0, h], 1e-6, block_of=block_of)
        assert _relerr(ref2, ref) <= 1e-12


def test_block_causal_differs_from_bidirectional():
    """Guards against a block path that silently ignores the mask."""
    Q, K, V = _rand(5, 1, 1, 12, 32)
    blocks = [(Q[:, :, a:a + 4], K[:, :, a:a + 4], V[:, :, a:a + 4]) for a in (0, 4, 8)]
    O_blk = np.concatenate([o for o, _, _ in orc.block_stream(blocks, 1e-6)], axis=2)
    O_bi, _, _ = orc.bidirectional(Q, K, V, 1e-6)
    assert _relerr(O_blk[:, :, :8], O_bi[:, :, :8]) > 1e-3      # early blocks see less
    assert _relerr(O_blk[:, :, 8:], O_bi[:, :, 8:]) <= 1e-12    # last block sees everything


# ---- P2: hand-computed example -------------------------------------------------------------

def _golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            parts = line.split()
            vals[parts[0]] = np.array([float(x) for x in parts[1:]])
    return vals


def test_hand_example():
    g = _golden("hand_example_2tok.txt")
    eps = 1e-6
    Q = np.array([[1, -1], [2, 3]], np.float32).reshape(1, 1, 2, 2)
    K = np.array([[1, 0], [-1, 2]], np.float32).reshape(1, 1, 2, 2)
    V = np.array([[1, 2], [3, 4]], np.float32).reshape(1, 1, 2, 2)
    O, S, z = orc.bidirectional(Q, K, V, eps)
    np.testing.assert_array_equal(S.ravel(), g["S"])
    np.testing.assert_array_equal(z.ravel(), g["z"])
    np.testing.assert_allclose(O[0, 0, 0], g["num0"] / (g["den0"][0] + eps), rtol=1e-15)
    np.testing.assert_allclose(O[0, 0, 1], g["num1"] / (g["den1"][0] + eps), rtol=1e-15)
    # two one-token blocks
    S0, z0 = orc.zero_state(1, 1, 2)
    O0, S1, z1 = orc.block_step(Q[:, :, :1], K[:, :, :1], V[:, :, :1], S0, z0, eps)
    np.testing.assert_array_equal(S1.ravel(), g["S_after_block0"])
    np.testing.assert_array_equal(z1.ravel(), g["z_after_block0"])
    np.testing.assert_allclose(O0[0, 0, 0], g["num0"] / (g["den0"][0] + eps), rtol=1e-15)
    O1, S2, z2 = orc.block_step(Q[:, :, 1:], K[:, :, 1:], V[:, :, 1:], S1, z1, eps)
    np.testing.assert_array_equal(S2.ravel(), g["S"])
    np.testing.assert_array_equal(z2.ravel(), g["z"])
    np.testing.assert_allclose(O1[0, 0, 0], g["num1"] / (g["den1"][0] + eps), rtol=1e-15)


def test_eps_is_added_to_the_denominator_after_the_dot_product():
    """Large eps makes its placement visible: O = num / (den + eps) exactly."""
    Q, K, V = _rand(7, 1, 1, 5, 32)
    O0, S, z = orc.bidirectional(Q, K, V, 0.0)
    O1, _, _ = orc.bidirectional(Q, K, V, 3.0)
    den = np.einsum("bhik,bhk->bhi", np.maximum(Q.astype(np.float64), 0), z)[..., None]
    np.testing.assert_allclose(O1, O0 * den / (den + 3.0), rtol=1e-12)


# ---- P3: one block run block-causally equals the bidirectional layer ------------------------

def test_single_block_equals_bidirectional_bitwise():
    Q, K, V = _rand(11, 2, 3, 50, 64)
    O, S, z = orc.bidirectional(Q, K, V, 1e-6)
    S0, z0 = orc.zero_state(2, 3, 64)
    Ob, S1, z1 = orc.block_step(Q, K, V, S0, z0, 1e-6)
    assert np.array_equal(O, Ob) and np.array_equal(S, S1) and np.array_equal(z, z1)


def test_non_committing_step_leaves_state_unchanged():
    """Alg. 1 reads the cache without updating it during the noisy passes."""
    Q, K, V = _rand(12, 1, 2, 9, 32)
    S0, z0 = orc.state(K, V)                       # some non-trivial carried state
    Q2, K2, V2 = _rand(13, 1, 2, 6, 32)
    O_c, S_c, z_c = orc.block_step(Q2, K2, V2, S0, z0, 1e-6, commit=True)
    O_n, S_n, z_n = orc.block_step(Q2, K2, V2, S0, z0, 1e-6, commit=False)
    assert np.array_equal(O_c, O_n)
    assert np.array_equal(S_n, S0) and np.array_equal(z_n, z0)
    assert not np.array_equal(S_c, S0)


# ---- P4: chunked state sums equal the one-shot sum ------------------------------------------

@pytest.mark.parametrize("splits", [[17], [1, 2, 40], [5, 5, 5, 5, 5, 30]])
def test_chunk_additivity(splits):
    N = 64
    _, K, V = _rand(21, 1, 2, N, 64)
    S_all, z_all = orc.state(K, V)
    edges = [0] + list(np.cumsum(splits)) + [N]
    S, z = None, None
    for a, b in zip(edges[:-1], edges[1:]):
        S, z = orc.state(K, V, a, b, S, z)
    assert _relerr(S, S_all) <= 1e-12 and _relerr(z, z_all) <= 1e-12


def test_empty_range_is_a_noop_or_zero():
    _, K, V = _rand(22, 1, 1, 8, 32)
    S, z = orc.state(K, V, 3, 3)
    assert not S.any() and not z.any()
    S1, z1 = orc.state(K, V)
    S2, z2 = orc.state(K, V, 5, 5, S1, z1)
    assert np.array_equal(S1, S2) and np.array_equal(z1, z2)


def test_apply_range_matches_full_apply():
    Q, K, V = _rand(23, 1, 2, 20, 32)
    O, S, z = orc.bidirectional(Q, K, V, 1e-6)
    part = orc.apply(Q, S, z, 1e-6, 4, 13)
    assert np.array_equal(part, O[:, :, 4:13])


# ---- P5: carried state size does not depend on the video length -----------------------------

def test_state_size_is_independent_of_length():
    sizes = set()
    for n_blocks, nb in [(1, 5), (10, 5), (80, 3), (3, 40)]:
        Q, K, V = _rand(31, 1, 2, n_blocks * nb, 32)
        blocks = [(Q[:, :, a:a + nb], K[:, :, a:a + nb], V[:, :, a:a + nb])
                  for a in range(0, n_blocks * nb, nb)]
        for _, S, z in orc.block_stream(blocks, 1e-6):
            sizes.add((S.nbytes, z.nbytes))
    assert sizes == {(2 * 32 * 32 * 8, 2 * 32 * 8)}


# ---- P6: convexity, scale invariance, linearity, permutation invariance ---------------------

def test_outputs_are_convex_combinations_of_values():
    Q, K, V = _rand(41, 1, 2, 33, 32)
    O, _, _ = orc.bidirectional(Q, K, V, 0.0)
    live = (np.maximum(Q, 0) @ np.maximum(K, 0).transpose(0, 1, 3, 2)).sum(-1) > 0
    lo = V.min(axis=2, keepdims=True) - 1e-12
    hi = V.max(axis=2, keepdims=True) + 1e-12
    ok = (O >= lo) & (O <= hi)
    assert ok[live].all()


def test_constant_values_give_den_over_den_plus_eps():
    Q, K, _ = _rand(42, 1, 1, 16, 32)
    V = np.full_like(Q, 2.5)
    eps = 0.125
    O, _, z = orc.bidirectional(Q, K, V, eps)
    den = np.einsum("bhik,bhk->bhi", np.maximum(Q.astype(np.float64), 0), z)[..., None]
    np.testing.assert_allclose(O, 2.5 * den / (den + eps) * np.ones_like(O), rtol=1e-12)


def test_positive_rescaling_of_q_or_k_cancels_without_eps():
    Q, K, V = _rand(43, 1, 2, 24, 64)
    O, _, _ = orc.bidirectional(Q, K, V, 0.0)
    O_q, _, _ = orc.bidirectional(Q * np.float32(4.0), K, V, 0.0)
    O_k, _, _ = orc.bidirectional(Q, K * np.float32(0.25), V, 0.0)
    ok = np.isfinite(O)
    assert _relerr(O_q[ok], O[ok]) <= 1e-12 and _relerr(O_k[ok], O[ok]) <= 1e-12


def test_linear_in_values():
    Q, K, V = _rand(44, 1, 1, 24, 32)
    _, _, V2 = _rand(45, 1, 1, 24, 32)
    a, b = np.float32(2.0), np.float32(-0.5)        # exact in fp32
    O1, _, _ = orc.bidirectional(Q, K, V, 1e-6)
    O2, _, _ = orc.bidirectional(Q, K, V2, 1e-6)
    O12, _, _ = orc.bidirectional(Q, K, a * V + b * V2, 1e-6)
    lhs, rhs = O12, float(a) * O1 + float(b) * O2
    assert np.max(np.abs(lhs - rhs)) <= 1e-6 * np.max(np.abs(rhs))   # fp32 rounding of a*V+b*V2


def test_token_permutation_of_keys_and_values():
    Q, K, V = _rand(46, 1, 2, 40, 32)
    perm = np.random.default_rng(0).permutation(40)
    O, _, _ = orc.bidirectional(Q, K, V, 1e-6)
    Op, _, _ = orc.bidirectional(Q, K[:, :, perm], V[:, :, perm], 1e-6)
    assert _relerr(Op, O) <= 1e-12
    # permuting K alone must change the result (K_j stays paired with V_j)
    Ox, _, _ = orc.bidirectional(Q, K[:, :, perm], V, 1e-6)
    assert _relerr(Ox, O) > 1e-3


def test_heads_and_batches_are_independent():
    Q, K, V = _rand(47, 2, 3, 10, 32)
    O, S, z = orc.bidirectional(Q, K, V, 1e-6)
    for b in range(2):
        for h in range(3):
            o1, s1, z1 = orc.bidirectional(Q[b:b + 1, h:h + 1], K[b:b + 1, h:h + 1],
                                           V[b:b + 1, h:h + 1], 1e-6)
            assert np.array_equal(o1[0, 0], O[b, h])
            assert np.array_equal(s1[0, 0], S[b, h]) and np.array_equal(z1[0, 0], z[b, h])


# ---- P7: degenerate rows ---------------------------------------------------------------------

def test_all_negative_query_row_gives_exact_zero():
    Q, K, V = _rand(51, 1, 1, 6, 32)
    Q[0, 0, 2] = -np.abs(Q[0, 0, 2]) - 1
    O, _, _ = orc.bidirectional(Q, K, V, 1e-6)
    assert not O[0, 0, 2].any() and np.isfinite(O).all()


def test_all_negative_keys_give_zero_state_and_output():
    Q, K, V = _rand(52, 1, 1, 6, 32)
    K = -np.abs(K) - 1
    O, S, z = orc.bidirectional(Q, K, V, 1e-6)
    assert not S.any() and not z.any() and not O.any()


def test_relu_is_on_q_and_k_but_not_on_v():
    Q, K, V = _rand(53, 1, 1, 8, 32)
    O, S, z = orc.bidirectional(Q, K, V, 1e-6)
    On, Sn, zn = orc.bidirectional(Q, K, -V, 1e-6)
    assert np.array_equal(Sn, -S) and np.array_equal(zn, z) and np.array_equal(On, -O)
    # negative parts of Q and K are invisible
    Oc, Sc, zc = orc.bidirectional(np.maximum(Q, 0), np.maximum(K, 0), V, 1e-6)
    assert np.array_equal(Oc, O) and np.array_equal(Sc, S)


# ---- P8: the sums as library matrix products ---------------------------------------------------

@pytest.mark.parametrize("d", [32, 64])
def test_state_and_apply_as_matrix_products(d):
    Q, K, V = _rand(61, 2, 2, 100, d)
    O, S, z = orc.bidirectional(Q, K, V, 1e-6)
    Kd, Vd, Qd = (np.asarray(t, np.float64) for t in (K, V, Q))
    pK, pQ = np.maximum(Kd, 0), np.maximum(Qd, 0)
    S_ref = pK.transpose(0, 1, 3, 2) @ Vd          # [k][v] = sum_j phiK[j][k] V[j][v]
    z_ref = pK.sum(axis=2)
    O_ref = (pQ @ S_ref) / ((pQ @ z_ref[..., None]) + 1e-6)
    assert _relerr(S, S_ref) <= 1e-12 and _relerr(z, z_ref) <= 1e-12 and _relerr(O, O_ref) <= 1e-11
    # orientation: S is [key feature][value feature], not its transpose
    assert _relerr(S, S_ref.transpose(0, 1, 3, 2)) > 1e-2


def test_bf16_inputs_are_widened_exactly():
    x = np.random.default_rng(3).standard_normal((1, 1, 9, 32)).astype(np.float32)
    bits = wl.f32_to_bf16_bits(x)
    xf = wl.bf16_bits_to_f32(bits)
    S1, z1 = orc.state(bits, bits)
    S2, z2 = orc.state(xf, xf)
    assert np.array_equal(S1, S2) and np.array_equal(z1, z2)


# ---- P9: closed-form statistics of the synthetic workloads -------------------------------------

def test_closed_form_statistics_of_gaussian_inputs():
    """For K, V ~ sigma*N(0,1): E z_k = N sigma / sqrt(2 pi), Var S_kv = N (sigma^2/2) sigma^2.
    Rounding the draws to bf16 perturbs both by far less than the sampling tolerance."""
    sigma, N, d, H = 0.5, 4096, 64, 4
    _, K, V = wl.draw_tensors(77, (1, H, N, d), sigma, "bf16")
    S, z = orc.state(K, V)
    ez = N * sigma / np.sqrt(2 * np.pi)
    # std of z_k is sigma*sqrt(N*(1/2 - 1/(2 pi))) ~ 18.7; mean over 256 values ~ 1.2
    assert abs(z.mean() - ez) < 6.0
    assert np.all(np.abs(z - ez) < 6 * sigma * np.sqrt(N * (0.5 - 1 / (2 * np.pi))))
    var_s = N * (sigma ** 2 / 2) * sigma ** 2
    assert abs(S.var() / var_s - 1.0) < 0.05
    # entries of S sharing a value column are correlated through sum_j V[j][v]:
    # Var(mean S) = N * E[(sum_k phiK)^2] * Var(sum_v V) / d^4
    e_sum_sq = d * sigma ** 2 * (0.5 - 1 / (2 * np.pi)) + (d * sigma / np.sqrt(2 * np.pi)) ** 2
    std_mean = np.sqrt(N * e_sum_sq * d * sigma ** 2 / d ** 4)
    assert abs(S[0, 0].mean()) < 5 * std_mean


# ---- input generator ---------------------------------------------------------------------------

def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.00390625, 1.01171875, -2.0, 3.0e-39], np.float32)
    # 1 + 2^-8 is a tie between 1.0 and 1+2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up
    bits = wl.f32_to_bf16_bits(f)
    back = wl.bf16_bits_to_f32(bits)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == np.float32(1.015625)
    assert back[3] == -2.0
    x = np.random.default_rng(1).standard_normal(10000).astype(np.float32)
    err = np.abs(wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(x)) - x)
    assert np.all(err <= np.abs(x) * 2.0 ** -8)


def test_generators_are_seeded_and_shaped():
    w = wl.workload("tiny_f32")
    a = wl.draw_qkv(w)
    b = wl.draw_qkv(w)
    assert all(np.array_equal(x, y) for x, y in zip(a, b))
    assert a[0].shape == (1, 2, 1024, 32) and a[0].dtype == np.float32
    assert not np.array_equal(a[0], a[1])
    ws = wl.workload("stream_720p")
    assert (ws.B, ws.H, ws.N, ws.d, ws.n_blocks) == (1, 32, 10800, 64, 80)
    assert wl.workload("bidir_480p").N == 32760 and wl.workload("bidir_720p").N == 75600
    assert wl.workload("block_480p").N == 4680
    assert wl.workload("bidir_480p").algorithmic_bytes == 536739840
