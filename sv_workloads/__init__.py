"""Seeded synthetic inputs for ReLU linear attention (and the Mix-FFN's temporal
convolution) over video token sequences.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmarks.  It holds no arithmetic of the method itself: only the workload
shapes, the random draw, and the storage format of the drawn values (bf16 bit
patterns or fp32).

The workloads stand in for the paper's video resolutions (Sec. 4.1 and the
latency tables): 480x832x81 and 720x1280x81 clips tokenised to 21x30x52 and
21x45x80 latent tokens, and the one-minute block-autoregressive stream of
Sec. 3.3.3.  Real activations are not available, so every tensor is i.i.d.
Gaussian, drawn as documented in `draw_qkv`.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

__all__ = [
    "Workload", "WORKLOADS", "workload", "draw_qkv", "draw_block",
    "draw_tensors", "f32_to_bf16_bits", "bf16_bits_to_f32", "as_f32", "rope_table_3d", "rope_tables_3d_factored",
    "expand_rope_tables", "TconvWorkload", "TCONV_WORKLOADS", "draw_tconv",
]


@dataclass(frozen=True)
class Workload:
    """Shape of one benchmark/parity configuration.

    `n_blocks == 0` means a bidirectional layer over N tokens; otherwise the
    sequence is `n_blocks` consecutive blocks of `N` tokens each, attended
    block-causally with a carried state.
    """
    name: str
    B: int
    H: int
    N: int          # tokens per head (per block when n_blocks > 0)
    d: int
    dtype: str      # "bf16" or "f32"
    scale: float    # values are scale * N(0, 1)
    seed: int
    n_blocks: int = 0
    per_block_seed: bool = False
    eps: float = 1e-6
    grid: tuple = ()    # (latent frames, rows, cols) of the N tokens, when they form a video volume

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def head_tokens(self) -> int:
        """Head-tokens in one pass (one block for block workloads)."""
        return self.B * self.H * self.N

    @property
    def algorithmic_bytes(self) -> int:
        """Q, K, V read once and O written once (per block for block workloads)."""
        return 4 * self.head_tokens * self.d * self.elem_bytes

    @property
    def algorithmic_flops(self) -> int:
        """(4 d^2 + 4 d) per head-token: two d x d contractions, key sum,
        denominator dot product and the final scale."""
        return self.head_tokens * (4 * self.d * self.d + 4 * self.d)


WORKLOADS = {
    # 4 latent frames x 16 x 16 tokens, fp32 validation mode
    "tiny_f32": Workload("tiny_f32", B=1, H=2, N=4 * 16 * 16, d=32, dtype="f32",
                         scale=1.0, seed=1001, grid=(4, 16, 16)),
    # 480p-like bidirectional layer
    "bidir_480p": Workload("bidir_480p", B=1, H=32, N=21 * 30 * 52, d=64,
                           dtype="bf16", scale=0.5, seed=1002, grid=(21, 30, 52)),
    # 720p-like bidirectional layer, conditional + unconditional pair
    "bidir_720p": Workload("bidir_720p", B=2, H=32, N=21 * 45 * 80, d=64,
                           dtype="bf16", scale=0.5, seed=1003, grid=(21, 45, 80)),
    # the same layer in the geometry of the paper's 2B model: 20 heads of 112 features
    "bidir_480p_h20d112": Workload("bidir_480p_h20d112", B=1, H=20, N=21 * 30 * 52, d=112,
                                   dtype="bf16", scale=0.5, seed=1012, grid=(21, 30, 52)),
    "block_480p_h20d112": Workload("block_480p_h20d112", B=1, H=20, N=3 * 30 * 52, d=112,
                                   dtype="bf16", scale=0.5, seed=1014, n_blocks=10, grid=(3, 30, 52)),
    # block-causal, 10 blocks of 3 latent frames x 30 x 52
    "block_480p": Workload("block_480p", B=1, H=32, N=3 * 30 * 52, d=64,
                           dtype="bf16", scale=0.5, seed=1004, n_blocks=10, grid=(3, 30, 52)),
    # minute-length stream, 80 blocks of 3 latent frames x 45 x 80
    "stream_720p": Workload("stream_720p", B=1, H=32, N=3 * 45 * 80, d=64,
                            dtype="bf16", scale=0.5, seed=5000, n_blocks=80,
                            per_block_seed=True, grid=(3, 45, 80)),
}


def workload(name: str) -> Workload:
    return WORKLOADS[name]


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest, ties to even); returns the uint16 patterns.

    Finite inputs only (the generators never produce NaN or Inf).
    """
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32)
            << np.uint32(16)).view(np.float32)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    raise ValueError(f"unknown dtype {dtype!r}")


def draw_tensors(seed: int, shape, scale: float, dtype: str, count: int = 3):
    """`count` tensors of `shape`, drawn one after another from one
    `numpy.random.Generator(PCG64(seed))` as float32 standard normals in C
    order, multiplied by `scale` in fp32, then stored as `dtype`
    ("bf16": uint16 bit patterns, "f32": float32)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    out = []
    for _ in range(count):
        x = rng.standard_normal(size=shape, dtype=np.float32)
        if scale != 1.0:
            x *= np.float32(scale)
        out.append(_store(x, dtype))
    return out


def draw_qkv(w: Workload):
    """Q, K, V for a bidirectional workload, or for the WHOLE sequence of a
    block workload whose blocks share one seed (shape [B][H][n_blocks*N][d];
    block m is tokens [m*N, (m+1)*N)).  Drawn in the order Q, K, V."""
    if w.per_block_seed:
        raise ValueError("per-block-seed workloads are drawn with draw_block")
    n = w.N * max(1, w.n_blocks)
    return draw_tensors(w.seed, (w.B, w.H, n, w.d), w.scale, w.dtype)


def draw_block(w: Workload, m: int):
    """Q, K, V of block m ([B][H][N][d]) of a block workload."""
    if w.n_blocks <= 0 or not 0 <= m < w.n_blocks:
        raise ValueError("block index out of range")
    if w.per_block_seed:
        return draw_tensors(w.seed + m, (w.B, w.H, w.N, w.d), w.scale, w.dtype)
    q, k, v = draw_qkv(w)
    sl = slice(m * w.N, (m + 1) * w.N)
    return [np.ascontiguousarray(t[:, :, sl, :]) for t in (q, k, v)]


def as_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    """The stored values as fp32, exactly (bf16 bits are widened)."""
    return bf16_bits_to_f32(x) if dtype == "bf16" else np.asarray(x, np.float32)


def rope_table_3d(frames: int, rows: int, cols: int, d: int, base: float = 10000.0,
                  t0: int = 0) -> np.ndarray:
    """Rotation table [frames*rows*cols][d/2][2] (cos, sin) in fp32 for tokens laid
    out frame-major, then row, then column: a 3-D rotary embedding.

    The paper says "3D RoPE" without frequencies; this generator (a proposal, used
    for test and benchmark inputs only) gives the d/2 feature pairs to the three
    axes in the proportion 2:3:3 (time gets what is left after rows and columns
    take floor(3/8 * d/2) each) and uses angle = position * base^(-i/n_axis) for
    the i-th pair of an axis with n_axis pairs.  `t0` is the index of the first
    frame (blocks of a stream continue the time axis).  The library itself only
    sees the table."""
    half = d // 2
    n_hw = (3 * half) // 8
    n_t = half - 2 * n_hw
    t = np.arange(t0, t0 + frames, dtype=np.float64)[:, None, None]
    r = np.arange(rows, dtype=np.float64)[None, :, None]
    c = np.arange(cols, dtype=np.float64)[None, None, :]
    ang = np.empty((frames, rows, cols, half), np.float64)
    for i in range(n_t):
        ang[..., i] = t * base ** (-i / n_t)
    for i in range(n_hw):
        ang[..., n_t + i] = r * base ** (-i / n_hw)
        ang[..., n_t + n_hw + i] = c * base ** (-i / n_hw)
    ang = ang.reshape(frames * rows * cols, half)
    return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)


def rope_tables_3d_factored(frames: int, rows: int, cols: int, d: int, base: float = 10000.0, t0: int = 0):
    """The same 3-D rotary embedding as `rope_table_3d`, as the three per-axis tables it
    is made of: (cs_t [frames][n_t][2], cs_h [rows][n_h][2], cs_w [cols][n_w][2]) in fp32,
    pairs ordered frame, row, column."""
    half = d // 2
    n_hw = (3 * half) // 8
    n_t = half - 2 * n_hw

    def axis(pos, n):
        ang = pos[:, None].astype(np.float64) * base ** (-np.arange(n, dtype=np.float64) / max(n, 1))[None, :]
        return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)

    return (axis(np.arange(t0, t0 + frames), n_t), axis(np.arange(rows), n_hw), axis(np.arange(cols), n_hw))


def expand_rope_tables(cs_t: np.ndarray, cs_h: np.ndarray, cs_w: np.ndarray) -> np.ndarray:
    """Full table [frames*rows*cols][n_t+n_h+n_w][2] of factored tables (tokens frame-major, then
    row, then column): pure indexing, no arithmetic."""
    frames, rows, cols = cs_t.shape[0], cs_h.shape[0], cs_w.shape[0]
    f, r, c = np.meshgrid(np.arange(frames), np.arange(rows), np.arange(cols), indexing="ij")
    full = np.concatenate([cs_t[f.ravel()], cs_h[r.ravel()], cs_w[c.ravel()]], axis=1)
    return np.ascontiguousarray(full, dtype=np.float32)


@dataclass(frozen=True)
class TconvWorkload:
    """Shape of one temporal-convolution configuration (Mix-FFN, Sec. 3.2 and 3.3.1):
    `n_blocks` consecutive blocks of T latent frames of HW tokens with D channels
    (`n_blocks == 1`: the whole clip at once, as in the bidirectional model)."""
    name: str
    B: int
    T: int          # latent frames per block
    HW: int         # tokens per frame
    D: int          # channels (hidden size of the model)
    seed: int
    n_blocks: int = 1

    @property
    def tokens(self) -> int:
        return self.B * self.T * self.HW

    @property
    def algorithmic_flops(self) -> int:
        """Three D x D taps per token, multiply and add (per block)."""
        return 2 * 3 * self.D * self.D * self.tokens

    @property
    def algorithmic_bytes(self) -> int:
        """Input read once, output written once, weights read once, cache in and out (per block)."""
        return 2 * (2 * self.tokens * self.D + 3 * self.D * self.D + 2 * self.B * self.HW * self.D)


TCONV_WORKLOADS = {
    # several tiles with ragged tails in tokens, channels and frames
    "tconv_tiny": TconvWorkload("tconv_tiny", B=2, T=5, HW=53, D=328, seed=2001, n_blocks=3),
    # the 2B model's hidden size (20 heads x 112) on the 480p token grid, whole clip
    "tconv_480p": TconvWorkload("tconv_480p", B=1, T=21, HW=30 * 52, D=2240, seed=2002),
    # the same in blocks of 3 latent frames
    "tconv_block_480p": TconvWorkload("tconv_block_480p", B=1, T=3, HW=30 * 52, D=2240, seed=2003, n_blocks=7),
}


def draw_tconv(w: TconvWorkload):
    """x [B][n_blocks*T][HW][D] and W [3][D][D] (tap, out, in) as bf16 bit patterns: x ~ N(0, 1)
    from PCG64(seed), W ~ N(0, 1 / (3 D)) from PCG64(seed + 7919), so that the convolution output
    has about the input's variance (block m is frames [m*T, (m+1)*T))."""
    x, = draw_tensors(w.seed, (w.B, w.n_blocks * w.T, w.HW, w.D), 1.0, "bf16", count=1)
    rng = np.random.Generator(np.random.PCG64(w.seed + 7919))
    wt = rng.standard_normal(size=(3, w.D, w.D), dtype=np.float32) * np.float32(1.0 / np.sqrt(3.0 * w.D))
    return x, f32_to_bf16_bits(wt)
