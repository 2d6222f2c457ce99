"""Float64 CPU oracle of the block-causal temporal convolution of the Mix-FFN.

Test infrastructure only: tests, the smoke check and the benchmark's
CPU-baseline leg call this; the GPU library never does.

What it computes (Sec. 3.3.1, "Block Causal Mix-FFN", and the Mix-FFN paragraph
of Sec. 3.2): a block of T latent frames of HW tokens with D channels each goes
through a 1-D convolution of kernel size 3 along the frame axis, every spatial
position on its own, and the result is added to the input (the shortcut).  The
frame before the block is the cached last frame of the previous block
(`Token_-1`; nothing cached = zeros, the empty cache Alg. 1 starts from); the
frame after the block is all zeros, so nothing of a later block leaks in.  The
new cache is the block's own last frame.

Readings where the paper is silent: the convolution mixes channels (dense
D x D per tap, no bias), taps are applied as a cross-correlation (tap 0 meets
the earlier frame), and the cache holds the module's input frame.

All arithmetic is numpy float64; the one library step is the matrix product of
each tap.
"""
from __future__ import annotations

import numpy as np


def _widen(a: np.ndarray) -> np.ndarray:
    """Stored values (bf16 bit patterns as uint16, or floats) -> float64, exactly."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        a = (a.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return a.astype(np.float64)


def tconv_block(x, W, cache=None):
    """One block through the temporal convolution with shortcut.

    x      [B][T][HW][D]   input frames of the block
    W      [3][D][D]       W[tap][out][in]; tap 0 multiplies frame t-1, tap 1 frame t, tap 2 frame t+1
    cache  [B][HW][D]      last input frame of the previous block, or None (zeros)

    Returns (y [B][T][HW][D] float64, new_cache [B][HW][D] float64 = x[:, T-1]).
    """
    x, W = _widen(x), _widen(W)
    if x.ndim != 4 or W.shape != (3, x.shape[3], x.shape[3]):
        raise ValueError("x must be [B][T][HW][D] and W [3][D][D]")
    B, T, HW, D = x.shape
    if T < 1:
        raise ValueError("a block has at least one frame")
    before = np.zeros((B, 1, HW, D)) if cache is None else _widen(cache).reshape(B, 1, HW, D)
    after = np.zeros((B, 1, HW, D))
    padded = np.concatenate([before, x, after], axis=1)          # frames -1 .. T
    y = x.copy()                                                 # the shortcut
    for tap in range(3):
        frames = padded[:, tap:tap + T]                          # frame t + tap - 1 for every t
        y += frames @ W[tap].T                                   # sum over input channels
    return y, x[:, T - 1].copy()


def tconv_stream(blocks, W, cache=None):
    """Runs tconv_block over consecutive blocks, handing each block's last frame to
    the next; yields (y, cache) after each block."""
    for xb in blocks:
        y, cache = tconv_block(xb, W, cache)
        yield y, cache


def tconv_rows(x, W, cache, rows):
    """The outputs of chosen tokens only: `rows` is a sequence of (b, t, hw); returns
    [len(rows)][D] float64.  Same definition as tconv_block, token by token."""
    xs, W = np.asarray(x), _widen(W)
    B, T, HW, D = xs.shape
    out = np.empty((len(rows), D))
    for i, (b, t, hw) in enumerate(rows):
        cur = _widen(xs[b, t, hw])
        if t > 0:
            prev = _widen(xs[b, t - 1, hw])
        elif cache is not None:
            prev = _widen(np.asarray(cache)[b, hw])
        else:
            prev = np.zeros(D)
        nxt = _widen(xs[b, t + 1, hw]) if t + 1 < T else np.zeros(D)
        out[i] = cur + W[0] @ prev + W[1] @ cur + W[2] @ nxt
    return out
