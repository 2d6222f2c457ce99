"""GPU parity of the temporal convolution (sv_tconv_block_step) against the float64 oracle.

Tolerance: products of bf16 values are exact in fp32, the 3*D-term sum is accumulated in fp32
(relative error of order sqrt(3 D) * 2^-24 of the sum of magnitudes, far below bf16 resolution),
and the result is rounded to bf16 once (relative error 2^-9).  The bar is the one used for the
attention outputs: max |diff| / max |ref| <= 2e-2 and relative L2 error <= 5e-3; in addition
every element must lie within one bf16 step (2^-8 of its magnitude) plus 1e-3 of the oracle.
"""
import numpy as np
import pytest

import paper_2509_24695_amd as sv
from oracle import tconv_oracle as orc
from sv_workloads import TCONV_WORKLOADS, TconvWorkload, draw_tconv
from tests.gpu_util import say, to_dev, to_host

pytestmark = pytest.mark.gpu


def _check(got, ref, what):
    diff = np.abs(got - ref)
    scale = np.abs(ref).max()
    assert diff.max() <= 2e-2 * scale, f"{what}: max diff {diff.max()} vs scale {scale}"
    rel_l2 = np.sqrt((diff ** 2).sum() / (ref ** 2).sum())
    assert rel_l2 <= 5e-3, f"{what}: rel l2 {rel_l2}"
    bound = np.abs(ref) * 2.0 ** -8 + 1e-3
    bad = diff > bound
    assert not bad.any(), f"{what}: {bad.sum()} elements off by more than a bf16 step, worst {diff[bad].max()}"


def _run_block(xd, Wd, cache_d, B, T, HW, D, commit=True):
    import torch
    y = torch.full((B, T, HW, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    cache_out = torch.full((B, HW, D), float("nan"), dtype=torch.bfloat16, device="cuda") if commit else None
    sv.sv_tconv_block_step(xd, Wd, cache_d, y, cache_out, B, T, HW, D)
    torch.cuda.synchronize()
    return y, cache_out


CASES = [
    TCONV_WORKLOADS["tconv_tiny"],
    # one frame per block: both neighbours come from outside the block
    TconvWorkload("one_frame", B=1, T=1, HW=300, D=64, seed=2101, n_blocks=3),
    # channel count below one tile and not a multiple of the K-step; token rows below one tile
    TconvWorkload("narrow", B=3, T=2, HW=7, D=40, seed=2102, n_blocks=2),
    # several channel tiles with a ragged last one, token tiles straddling frames and batches
    TconvWorkload("wide", B=2, T=3, HW=211, D=584, seed=2103, n_blocks=2),
    # more token-tile groups than XCDs take in one round
    TconvWorkload("many_tiles", B=1, T=4, HW=2400, D=64, seed=2104, n_blocks=1),
    # more tiles than compute units (several rounds), ragged in tokens, channels and the K-step
    TconvWorkload("rounds", B=1, T=2, HW=8900, D=760, seed=2105, n_blocks=1),
]


@pytest.mark.parametrize("w", CASES, ids=lambda w: w.name)
def test_block_stream_matches_oracle(w):
    xb, Wb = draw_tconv(w)
    Wd = to_dev(Wb)
    cache_ref, cache_d = None, None
    for m in range(w.n_blocks):
        say(f"tconv {w.name} block {m}: B={w.B} T={w.T} HW={w.HW} D={w.D}")
        blk = np.ascontiguousarray(xb[:, m * w.T:(m + 1) * w.T])
        y_ref, cache_ref = orc.tconv_block(blk, Wb, cache_ref)
        xd = to_dev(blk)
        y, cache_new = _run_block(xd, Wd, cache_d, w.B, w.T, w.HW, w.D)
        _check(to_host(y).astype(np.float64), y_ref, f"{w.name} block {m}")
        assert np.array_equal(to_host(cache_new).astype(np.float64), cache_ref)     # a copy: bit-exact
        cache_d = cache_new


def test_without_commit_and_in_place_cache():
    import torch
    w = TCONV_WORKLOADS["tconv_tiny"]
    xb, Wb = draw_tconv(w)
    Wd = to_dev(Wb)
    blk0, blk1 = (np.ascontiguousarray(xb[:, m * w.T:(m + 1) * w.T]) for m in (0, 1))
    say("tconv: non-committing call leaves no cache; in-place cache update")
    cache = to_dev(np.ascontiguousarray(blk0[:, -1]))
    before = cache.clone()
    y_a, none = _run_block(to_dev(blk1), Wd, cache, w.B, w.T, w.HW, w.D, commit=False)
    assert none is None and torch.equal(cache.view(torch.int16), before.view(torch.int16))
    # committing into the buffer that is also read as cache_in gives the same y and the new cache
    y_b = torch.empty_like(y_a)
    sv.sv_tconv_block_step(to_dev(blk1), Wd, cache, y_b, cache, w.B, w.T, w.HW, w.D)
    torch.cuda.synchronize()
    assert torch.equal(y_a.view(torch.int16), y_b.view(torch.int16))
    y_ref, cache_ref = orc.tconv_block(blk1, Wb, blk0[:, -1])
    _check(to_host(y_b).astype(np.float64), y_ref, "in-place")
    assert np.array_equal(to_host(cache).astype(np.float64), cache_ref)


def test_repeatable_bits():
    import torch
    w = CASES[3]
    xb, Wb = draw_tconv(w)
    xd, Wd = to_dev(np.ascontiguousarray(xb[:, :w.T])), to_dev(Wb)
    say("tconv: two identical calls give identical bits")
    y1, _ = _run_block(xd, Wd, None, w.B, w.T, w.HW, w.D)
    y2, _ = _run_block(xd, Wd, None, w.B, w.T, w.HW, w.D)
    assert torch.equal(y1.view(torch.int16), y2.view(torch.int16))


@pytest.mark.parametrize("name", ["tconv_480p", "tconv_block_480p"])
def test_full_size(name):
    """The benchmark's shapes in the benchmark's launch configuration, every element of y against the oracle
    (for the block workload: every block of the stream, the cache carried on the device), y pre-filled with
    NaN; the new cache must be the block's last input frame bit for bit."""
    import torch
    w = TCONV_WORKLOADS[name]
    xb, Wb = draw_tconv(w)
    Wd = to_dev(Wb)
    say(f"tconv full size {name}: B={w.B} T={w.T} HW={w.HW} D={w.D}, {w.n_blocks} block(s)")
    cache_d, cache_ref = None, None
    for m in range(max(1, w.n_blocks)):
        blk = np.ascontiguousarray(xb[:, m * w.T:(m + 1) * w.T])
        y = torch.full((w.B, w.T, w.HW, w.D), float("nan"), dtype=torch.bfloat16, device="cuda")
        new_cache = torch.empty((w.B, w.HW, w.D), dtype=torch.bfloat16, device="cuda")
        sv.sv_tconv_block_step(to_dev(blk), Wd, cache_d, y, new_cache, w.B, w.T, w.HW, w.D)
        torch.cuda.synchronize()
        y_ref, cache_ref = orc.tconv_block(blk, Wb, cache_ref)
        _check(to_host(y).astype(np.float64), y_ref, f"{name} block {m}")
        assert np.array_equal(to_host(new_cache).astype(np.float64), cache_ref)
        cache_d = new_cache


def test_measurement_variants_write_all_of_y_and_variant_0_is_the_library_kernel():
    """sv_measure_tconv_variant: variant 0 is sv_tconv_block_step's kernel bit for bit; variants 1-3 (parts of
    the tile loop left out, for timing) touch nothing but y and leave no element of it unwritten."""
    import torch
    B, T, HW, D = 1, 3, 300, 320                       # two token tiles, two channel tiles, ten K-steps per tap
    rng = np.random.default_rng(77)
    x = (rng.standard_normal((B, T, HW, D)) * 0.5).astype(np.float32)
    Wt = (rng.standard_normal((3, D, D)) * 0.05).astype(np.float32)
    cache = (rng.standard_normal((B, HW, D)) * 0.5).astype(np.float32)
    xd, Wd, cd = (torch.from_numpy(t).to(torch.bfloat16).cuda() for t in (x, Wt, cache))
    keep = [t.clone() for t in (xd, Wd, cd)]
    y_lib = torch.empty_like(xd)
    sv.sv_tconv_block_step(xd, Wd, cd, y_lib, None, B, T, HW, D)
    say("tconv measurement variants")
    for variant in range(4):
        y = torch.full_like(xd, float("nan"))
        sv.sv_measure_tconv_variant(variant, xd, Wd, cd, y, B, T, HW, D)
        torch.cuda.synchronize()
        assert bool(torch.isfinite(y.float()).all()), variant
        if variant == 0:
            assert torch.equal(y.view(torch.int16), y_lib.view(torch.int16))
        for t, k in zip((xd, Wd, cd), keep):
            assert torch.equal(t.view(torch.int16), k.view(torch.int16))
