"""Pins of the temporal-convolution oracle against things other than itself: a hand-worked
example, closed forms for shift kernels, the library convolution for the cache-free case,
brute-force loops, and the relation between block-wise and whole-clip processing
(Sec. 3.3.1, "Block Causal Mix-FFN")."""
import os

import numpy as np
import pytest
import torch

from oracle import tconv_oracle as orc
from sv_workloads import TCONV_WORKLOADS, bf16_bits_to_f32, draw_tconv

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_example_tconv.txt")


def _rand(seed, *shape):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def test_hand_example():
    vals = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            key, *nums = line.split()
            vals[key] = np.array([float(v) for v in nums])
    W = vals["w"].reshape(3, 1, 1)
    y0, c0 = orc.tconv_block(vals["x0"].reshape(1, 2, 1, 1), W, None)
    assert np.array_equal(y0.ravel(), vals["y0"]) and np.array_equal(c0.ravel(), vals["c0"])
    y1, c1 = orc.tconv_block(vals["x1"].reshape(1, 2, 1, 1), W, c0)
    assert np.array_equal(y1.ravel(), vals["y1"]) and np.array_equal(c1.ravel(), vals["c1"])


@pytest.mark.parametrize("tap", [0, 1, 2])
def test_shift_kernels_closed_form(tap):
    B, T, HW, D = 2, 4, 3, 5
    x, cache = _rand(1, B, T, HW, D), _rand(2, B, HW, D)
    W = np.zeros((3, D, D))
    W[tap] = np.eye(D)
    y, new_cache = orc.tconv_block(x, W, cache)
    if tap == 0:      # every frame gets the frame before it; the first one gets the cache
        want = x + np.concatenate([cache[:, None], x[:, :-1]], axis=1)
    elif tap == 1:
        want = 2 * x
    else:             # every frame gets the frame after it; the last one gets nothing
        want = x + np.concatenate([x[:, 1:], np.zeros((B, 1, HW, D))], axis=1)
    assert np.array_equal(y, want)
    assert np.array_equal(new_cache, x[:, -1])


def test_channel_orientation():
    """W[tap][out][in]: a single non-zero weight moves channel `i` of the earlier frame to channel `o`."""
    D, o, i = 4, 3, 1
    x, cache = _rand(3, 1, 2, 1, D), _rand(4, 1, 1, D)
    W = np.zeros((3, D, D))
    W[0, o, i] = 2.0
    y, _ = orc.tconv_block(x, W, cache)
    want = x.copy()
    want[0, 0, 0, o] += 2.0 * cache[0, 0, i]
    want[0, 1, 0, o] += 2.0 * x[0, 0, 0, i]
    assert np.allclose(y, want, rtol=0, atol=1e-15)


def test_cache_free_block_is_library_conv():
    """No cache, zero frame behind: the ordinary zero-padded convolution of a deep-learning library."""
    B, T, HW, D = 2, 6, 7, 9
    x, W = _rand(5, B, T, HW, D), _rand(6, 3, D, D)
    y, _ = orc.tconv_block(x, W, None)
    xt = torch.from_numpy(x).permute(0, 3, 1, 2)                       # [B][D][T][HW]
    wt = torch.from_numpy(W).permute(1, 2, 0)[..., None].contiguous()  # [out][in][3][1]
    ref = xt + torch.nn.functional.conv2d(xt, wt, padding=(1, 0))
    assert np.allclose(y, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-12, atol=1e-12)


def test_brute_force_loops():
    B, T, HW, D = 2, 3, 2, 4
    x, W, cache = _rand(7, B, T, HW, D), _rand(8, 3, D, D), _rand(9, B, HW, D)
    y, _ = orc.tconv_block(x, W, cache)
    for b in range(B):
        for t in range(T):
            for p in range(HW):
                for o in range(D):
                    acc = x[b, t, p, o]
                    for tap in range(3):
                        src = t + tap - 1
                        for i in range(D):
                            if src < 0:
                                v = cache[b, p, i]
                            elif src >= T:
                                v = 0.0
                            else:
                                v = x[b, src, p, i]
                            acc += W[tap, o, i] * v
                    assert abs(acc - y[b, t, p, o]) < 1e-12


def test_blocks_versus_whole_clip():
    """Processing block by block with the cache differs from one pass over the whole clip only
    in the last frame of each block but the final one, and there by exactly tap 2 applied to
    the next block's first frame (the information that must not leak)."""
    B, T, HW, D, nb = 1, 3, 4, 6, 3
    x, W = _rand(10, B, nb * T, HW, D), _rand(11, 3, D, D)
    whole, _ = orc.tconv_block(x, W, None)
    blocks = [x[:, m * T:(m + 1) * T] for m in range(nb)]
    ys = [y for y, _ in orc.tconv_stream(blocks, W)]
    for m, y in enumerate(ys):
        want = whole[:, m * T:(m + 1) * T].copy()
        if m + 1 < nb:
            want[:, -1] -= x[:, (m + 1) * T] @ W[2].T
        assert np.allclose(y, want, rtol=1e-12, atol=1e-12)


def test_rows_form_agrees_and_bf16_inputs_widen_exactly():
    w = TCONV_WORKLOADS["tconv_tiny"]
    xb, Wb = draw_tconv(w)
    blk = xb[:, w.T:2 * w.T]
    cache = xb[:, w.T - 1]
    y, new_cache = orc.tconv_block(blk, Wb, cache)
    y_f, _ = orc.tconv_block(bf16_bits_to_f32(blk), bf16_bits_to_f32(Wb), bf16_bits_to_f32(cache))
    assert np.array_equal(y, y_f)
    assert np.array_equal(new_cache, bf16_bits_to_f32(blk[:, -1]).astype(np.float64))
    rows = [(0, 0, 0), (1, w.T - 1, w.HW - 1), (0, 2, 17), (1, 0, 52)]
    got = orc.tconv_rows(blk, Wb, cache, rows)
    for g, (b, t, p) in zip(got, rows):
        assert np.allclose(g, y[b, t, p], rtol=1e-12, atol=1e-12)
    no_cache = orc.tconv_rows(blk, Wb, None, rows[:1])
    y0, _ = orc.tconv_block(blk, Wb, None)
    assert np.allclose(no_cache[0], y0[0, 0, 0], rtol=1e-12, atol=1e-12)
