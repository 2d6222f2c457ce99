"""GPU parity: the HIP library, called through its C ABI, against the float64
CPU oracle on the same seeded inputs, element by element.

Tolerances (written out in sv_workloads.metrics.TOL): bf16 tokens -- max
relative error 2e-2 and relative L2 error 5e-3 on O; fp32 validation mode --
1e-5 on both.  S and z are fp32 sums of exactly representable products in both
modes and are held to the 1e-5 class everywhere.
"""
import numpy as np
import pytest

import paper_2509_24695_amd as sv
import sv_workloads as wl
from oracle import linattn_oracle as orc
from sv_workloads import metrics
from tests.gpu_util import gpu_bidirectional, new_state, new_workspace, say, to_dev, to_host

pytestmark = pytest.mark.gpu

STATE_TOL = 1e-5


def _draw(seed, B, H, N, d, dtype, scale=0.5):
    return wl.draw_tensors(seed, (B, H, N, d), scale, dtype)


def _check_state(S, z, S_ref, z_ref, what):
    for name, g, r in (("S", S, S_ref), ("z", z, z_ref)):
        g = to_host(g)
        assert np.isfinite(g).all(), f"{what}: non-finite {name}"
        assert metrics.rel_l2(g, r) <= STATE_TOL, f"{what}: {name} rel_l2 {metrics.rel_l2(g, r)}"
        assert metrics.max_rel(g, r) <= STATE_TOL, f"{what}: {name} max_rel {metrics.max_rel(g, r)}"


# ---- configuration 1: fp32 validation mode ---------------------------------------------------

def test_tiny_f32_bidirectional():
    w = wl.workload("tiny_f32")
    say(f"{w.name} B={w.B} H={w.H} N={w.N} d={w.d} f32")
    Q, K, V = wl.draw_qkv(w)
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, w.eps)
    O, S, z = gpu_bidirectional(to_dev(Q), to_dev(K), to_dev(V), w.eps)
    _check_state(S, z, S_ref, z_ref, w.name)
    metrics.check(to_host(O), O_ref, "f32", w.name)


# ---- small shapes: several tiles, ragged tails, both dtypes and head dims ----------------------

@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("bf16", 32), ("f32", 64), ("f32", 32),
                                     ("bf16", 112), ("bf16", 128), ("f32", 112), ("f32", 128)])
@pytest.mark.parametrize("B,H,N", [(1, 1, 1), (1, 2, 7), (2, 3, 33), (1, 2, 100), (1, 4, 1000), (2, 2, 4681)])
def test_bidirectional_small(dtype, d, B, H, N):
    say(f"bidirectional_small dtype={dtype} d={d} B={B} H={H} N={N}")
    Q, K, V = _draw(7000 + N, B, H, N, d, dtype)
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6)
    O, S, z = gpu_bidirectional(to_dev(Q), to_dev(K), to_dev(V), 1e-6)
    _check_state(S, z, S_ref, z_ref, "state")
    metrics.check(to_host(O), O_ref, dtype, "O")


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("f32", 32), ("bf16", 112), ("bf16", 128), ("f32", 112)])
def test_state_range_and_accumulate(dtype, d):
    """Token ranges and accumulate semantics; chunked sums equal the one-shot sum."""
    import torch
    B, H, N = 2, 3, 3000
    say(f"state_range_and_accumulate dtype={dtype} d={d}")
    _, K, V = _draw(7100, B, H, N, d, dtype)
    Kd, Vd = to_dev(K), to_dev(V)
    dsc = sv.desc_of(Kd)
    ws = new_workspace(B, H, N, d)
    S, z = new_state(B, H, d)
    edges = [0, 1, 18, 18, 1500, 2999, 3000]          # includes an empty range
    for a, b in zip(edges[:-1], edges[1:]):
        sv.sv_linattn_state(Kd, Vd, dsc, a, b, 1, S, z, ws)
    torch.cuda.synchronize()
    S_ref, z_ref = orc.state(K, V)
    _check_state(S, z, S_ref, z_ref, "accumulated")
    # a strict sub-range, overwrite mode
    sv.sv_linattn_state(Kd, Vd, dsc, 37, 2050, 0, S, z, ws)
    torch.cuda.synchronize()
    S_ref, z_ref = orc.state(K, V, 37, 2050)
    _check_state(S, z, S_ref, z_ref, "sub-range")
    # empty range, overwrite mode: zero fill
    sv.sv_linattn_state(Kd, Vd, dsc, 5, 5, 0, S, z, ws)
    torch.cuda.synchronize()
    assert not to_host(S).any() and not to_host(z).any()


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("f32", 32), ("bf16", 112), ("bf16", 128), ("f32", 112)])
def test_apply_range_leaves_other_rows_untouched(dtype, d):
    import torch
    B, H, N = 1, 2, 500
    say(f"apply_range dtype={dtype} d={d}")
    Q, K, V = _draw(7200, B, H, N, d, dtype)
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6)
    Qd = to_dev(Q)
    Sd = torch.from_numpy(S_ref.astype(np.float32)).cuda()
    zd = torch.from_numpy(z_ref.astype(np.float32)).cuda()
    O = torch.full_like(Qd, 7.0)
    sv.sv_linattn_apply(Qd, sv.desc_of(Qd), 33, 401, Sd, zd, 1e-6, O)
    torch.cuda.synchronize()
    Oh = to_host(O)
    assert (Oh[:, :, :33] == 7.0).all() and (Oh[:, :, 401:] == 7.0).all()
    metrics.check(Oh[:, :, 33:401], O_ref[:, :, 33:401], dtype, "O range")


def test_strided_token_layout():
    """[B][N][H][d] memory (a projection's natural output) through the strides."""
    import torch
    B, H, N, d = 2, 4, 300, 64
    say("strided_token_layout")
    Q, K, V = _draw(7300, B, H, N, d, "bf16")
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6)

    def bnhd(x):          # same logical tensor, physical layout [B][N][H][d]
        return to_dev(x).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)

    Qd, Kd, Vd = bnhd(Q), bnhd(K), bnhd(V)
    assert Qd.stride() == (N * H * d, d, H * d, 1)
    S, z = new_state(B, H, d)
    ws = new_workspace(B, H, N, d)
    O = torch.zeros_like(Qd)               # preserves the permuted strides
    assert O.stride() == Qd.stride()
    sv.sv_linattn_state(Kd, Vd, sv.desc_of(Kd), 0, N, 0, S, z, ws)
    sv.sv_linattn_apply(Qd, sv.desc_of(Qd), 0, N, S, z, 1e-6, O)
    torch.cuda.synchronize()
    _check_state(S, z, S_ref, z_ref, "strided")
    metrics.check(to_host(O), O_ref, "bf16", "strided O")


@pytest.mark.parametrize("log2_stride,path", [(19, "MFMA kernels, offsets near 1 GiB"),
                                              (20, "head spans more than 2 GiB: generic kernels")])
def test_far_apart_token_rows(log2_stride, path):
    """Token rows 1-2 MiB apart: the bf16 d=64 kernels address a head with 32-bit byte offsets and
    the library must route heads that do not fit to kernels that do not."""
    import torch
    B, H, N, d = 1, 1, 1100, 64
    stride_n = 1 << log2_stride
    say(f"far_apart_token_rows stride_n=2^{log2_stride} ({path})")
    Q, K, V = _draw(7400, B, H, N, d, "bf16")
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6)

    def spread(x):
        base = torch.zeros(N * stride_n, dtype=torch.bfloat16, device="cuda")
        view = base.as_strided((B, H, N, d), (N * stride_n, N * stride_n, stride_n, 1))
        if x is not None:
            view.copy_(to_dev(x))
        return view

    Qd, Kd, Vd, O = spread(Q), spread(K), spread(V), spread(None)
    dsc = sv.desc_of(Qd)
    assert dsc.stride_n == stride_n
    S, z = new_state(B, H, d)
    ws = new_workspace(B, H, N, d)
    sv.sv_linattn_state(Kd, Vd, dsc, 0, N, 0, S, z, ws)
    sv.sv_linattn_apply(Qd, dsc, 0, N, S, z, 1e-6, O)
    torch.cuda.synchronize()
    _check_state(S, z, S_ref, z_ref, "far apart")
    metrics.check(to_host(O), O_ref, "bf16", "far apart O")
    # the block step over the same rows, from a zero state, must agree with the two calls
    S2, z2 = new_state(B, H, d)
    O2 = spread(None)
    sv.sv_block_linattn_step(Qd, Kd, Vd, dsc, S2, z2, 1e-6, O2, ws)
    torch.cuda.synchronize()
    _check_state(S2, z2, S_ref, z_ref, "far apart block step")
    metrics.check(to_host(O2), O_ref, "bf16", "far apart block step O")


# ---- degenerate rows -------------------------------------------------------------------------

@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("f32", 32), ("bf16", 112), ("bf16", 128), ("f32", 112)])
def test_degenerate_rows(dtype, d):
    say(f"degenerate_rows dtype={dtype} d={d}")
    B, H, N = 1, 2, 70
    Q, K, V = (wl.as_f32(t, dtype) for t in _draw(7400, B, H, N, d, dtype))
    Q[0, 0, 3] = -np.abs(Q[0, 0, 3]) - 0.5          # a query with phi(Q) = 0
    Q[0, 1, 69] = -np.abs(Q[0, 1, 69]) - 0.5
    K[0, 1] = -np.abs(K[0, 1]) - 0.5                # a head whose keys are all negative
    store = (lambda x: wl.f32_to_bf16_bits(x)) if dtype == "bf16" else (lambda x: x)
    Q, K, V = store(Q), store(K), store(V)
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6)
    O, S, z = gpu_bidirectional(to_dev(Q), to_dev(K), to_dev(V), 1e-6)
    Oh, Sh, zh = to_host(O), to_host(S), to_host(z)
    assert np.isfinite(Oh).all()
    assert not Oh[0, 0, 3].any() and not Oh[0, 1].any()
    assert not Sh[0, 1].any() and not zh[0, 1].any()
    metrics.check(Oh, O_ref, dtype, "degenerate O")


# ---- block-causal stream -----------------------------------------------------------------------

def _gpu_stream(blocks, eps, B, H, d):
    """Runs sv_block_linattn_step over host blocks; returns per-block O (host), final S, z."""
    import torch
    S, z = new_state(B, H, d)
    ws = new_workspace(B, H, max(b[0].shape[2] for b in blocks), d)
    outs = []
    for (Q, K, V) in blocks:
        Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
        O = torch.empty_like(Qd)
        sv.sv_block_linattn_step(Qd, Kd, Vd, sv.desc_of(Qd), S, z, eps, O, ws)
        torch.cuda.synchronize()
        outs.append(to_host(O))
    return outs, S, z


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("f32", 32), ("bf16", 112), ("bf16", 128), ("f32", 112)])
def test_block_stream_small(dtype, d):
    B, H = 1, 3
    sizes = [130, 1, 64, 333, 17]
    say(f"block_stream_small dtype={dtype} d={d} sizes={sizes}")
    blocks = [_draw(7500 + i, B, H, n, d, dtype) for i, n in enumerate(sizes)]
    outs, S, z = _gpu_stream(blocks, 1e-6, B, H, d)
    S_ref = z_ref = None
    for i, (O_ref, S_ref, z_ref) in enumerate(orc.block_stream(blocks, 1e-6)):
        metrics.check(outs[i], O_ref, dtype, f"block {i}")
    _check_state(S, z, S_ref, z_ref, "final state")


def test_block_stream_few_heads_many_chunks():
    """Two heads only: each head's tokens go to the largest number of workgroups the library uses (32),
    so the fold of the carried state runs over several groups of partials."""
    B, H, d = 1, 2, 64
    sizes = [6000, 4500, 4100]
    say(f"block_stream_few_heads sizes={sizes}")
    blocks = [_draw(7550 + i, B, H, n, d, "bf16") for i, n in enumerate(sizes)]
    outs, S, z = _gpu_stream(blocks, 1e-6, B, H, d)
    S_ref = z_ref = None
    for i, (O_ref, S_ref, z_ref) in enumerate(orc.block_stream(blocks, 1e-6)):
        metrics.check(outs[i], O_ref, "bf16", f"block {i}")
    _check_state(S, z, S_ref, z_ref, "final state")


def test_single_block_equals_bidirectional_bitwise():
    """One block from the empty cache is the bidirectional layer (same kernels, same order)."""
    import torch
    B, H, N, d = 1, 4, 2000, 64
    say("single_block_equals_bidirectional")
    Q, K, V = _draw(7600, B, H, N, d, "bf16")
    Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
    O1, S1, z1 = gpu_bidirectional(Qd, Kd, Vd, 1e-6)
    S2, z2 = new_state(B, H, d)
    O2 = torch.empty_like(Qd)
    sv.sv_block_linattn_step(Qd, Kd, Vd, sv.desc_of(Qd), S2, z2, 1e-6, O2, new_workspace(B, H, N, d))
    torch.cuda.synchronize()
    assert torch.equal(S1, S2) and torch.equal(z1, z2)
    assert torch.equal(O1.view(torch.int16), O2.view(torch.int16))


def test_determinism_and_resume():
    """Two runs are bit-identical; stopping, saving (S, z) to the host and resuming in fresh
    buffers continues bit-identically (the carried state is the whole context)."""
    import torch
    B, H, d = 1, 8, 64
    sizes = [700, 700, 700, 700]
    say("determinism_and_resume")
    blocks = [_draw(7700 + i, B, H, n, d, "bf16") for i, n in enumerate(sizes)]
    outs1, S1, z1 = _gpu_stream(blocks, 1e-6, B, H, d)
    outs2, S2, z2 = _gpu_stream(blocks, 1e-6, B, H, d)
    assert torch.equal(S1, S2) and torch.equal(z1, z2)
    assert all(np.array_equal(a, b) for a, b in zip(outs1, outs2))
    # resume after two blocks
    _, Sa, za = _gpu_stream(blocks[:2], 1e-6, B, H, d)
    Sh, zh = Sa.cpu(), za.cpu()
    del Sa, za
    S, z = Sh.cuda(), zh.cuda()
    ws = new_workspace(B, H, 700, d)
    for i in (2, 3):
        Qd, Kd, Vd = (to_dev(t) for t in blocks[i])
        O = torch.empty_like(Qd)
        sv.sv_block_linattn_step(Qd, Kd, Vd, sv.desc_of(Qd), S, z, 1e-6, O, ws)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(O), outs1[i])
    assert torch.equal(S, S1) and torch.equal(z, z1)


def test_workspace_and_state_bytes_do_not_depend_on_length():
    sizes = {sv.sv_linattn_workspace_bytes(1, 32, n, 64) for n in (1, 4680, 10800, 864000)}
    assert len(sizes) == 1


# ---- error paths reach the caller before any launch ----------------------------------------------

def test_errors_leave_outputs_untouched():
    import torch
    B, H, N, d = 1, 2, 64, 64
    say("error paths")
    Q, K, V = (to_dev(t) for t in _draw(7800, B, H, N, d, "bf16"))
    S, z = new_state(B, H, d)
    S.fill_(3.0)
    ws = new_workspace(B, H, N, d)
    dsc = sv.desc_of(K)
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_state(K, V, dsc, 10, 65, 0, S, z, ws)
    assert e.value.status == 5
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_state(K, V, dsc, 0, N, 0, S, z, ws, workspace_bytes=16)
    assert e.value.status == 6
    torch.cuda.synchronize()
    assert (S == 3.0).all()


# ---- launch shapes beyond the resident grid, and the timeout word ---------------------------------

@pytest.mark.parametrize("BH,d", [(130, 64), (300, 64), (130, 112), (300, 112), (300, 128)])
def test_many_heads_bidirectional_and_block(BH, d):
    """More heads than compute units: one chunk per head; at 300 heads the grid is not resident, so
    the state call takes the two-launch route and the block step the state + apply route."""
    import torch
    B, H, N = 1, BH, 150
    say(f"many_heads BH={BH} N={N} d={d}")
    Q, K, V = _draw(7900 + BH, B, H, N, d, "bf16")
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6)
    Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
    O, S, z = gpu_bidirectional(Qd, Kd, Vd, 1e-6)
    _check_state(S, z, S_ref, z_ref, "state")
    metrics.check(to_host(O), O_ref, "bf16", "O")
    # the same tokens as two blocks through the block step
    S2, z2 = new_state(B, H, d)
    ws = new_workspace(B, H, N, d)
    O2 = torch.empty_like(Qd)
    for a, b in ((0, 70), (70, 150)):
        q, k, v, o = (t[:, :, a:b] for t in (Qd, Kd, Vd, O2))
        sv.sv_block_linattn_step(q, k, v, sv.desc_of(q), S2, z2, 1e-6, o, ws)
    torch.cuda.synchronize()
    blocks = [tuple(np.ascontiguousarray(t[:, :, a:b]) for t in (Q, K, V)) for a, b in ((0, 70), (70, 150))]
    outs = list(orc.block_stream(blocks, 1e-6))
    metrics.check(to_host(O2)[:, :, :70], outs[0][0], "bf16", "block 0")
    metrics.check(to_host(O2)[:, :, 70:], outs[1][0], "bf16", "block 1")
    _check_state(S2, z2, outs[1][1], outs[1][2], "carried state")


@pytest.mark.parametrize("H,d", [(32, 64), (20, 112)])
def test_bounded_waits_never_time_out(H, d):
    """The workspace records a timed-out wait; after many calls on a workspace that was never
    initialised (undefined contents) the library's query must still say that none has."""
    import torch
    B, N = 1, 4680
    say("bounded_waits_never_time_out")
    Q, K, V = (to_dev(t) for t in _draw(7950, B, H, N, d, "bf16"))
    ws = new_workspace(B, H, N, d)
    ws.fill_(0xA5)
    S, z = new_state(B, H, d)
    O = torch.empty_like(Q)
    dsc = sv.desc_of(Q)
    for _ in range(20):
        sv.sv_linattn_state(K, V, dsc, 0, N, 0, S, z, ws)
        sv.sv_block_linattn_step(Q, K, V, dsc, S, z, 1e-6, O, ws)
    assert sv.sv_linattn_workspace_status(ws, B, H, d) == 0
    # the word the query reads is where the header says it is
    off = sv.sv_linattn_workspace_status_offset(B, H, d)
    assert int(ws[off:off + 8].view(torch.int64)[0]) != 0x54494d454f555421


@pytest.mark.parametrize("H,d", [(8, 64), (20, 112)])
def test_timed_out_wait_stores_nothing_and_is_reported(H, d):
    """With the wait bound set to zero polls every in-kernel wait fails at once (the kernels still run to
    their end): the carried S, z and the rows of O must keep their contents, the workspace must report the
    timeout, initialising the workspace must clear the report, and the next call must be right again."""
    import torch
    B, N = 1, 2000
    say(f"timed_out_wait H={H} d={d}")
    Q, K, V = _draw(7960, B, H, N, d, "bf16")
    Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
    dsc = sv.desc_of(Qd)
    ws = new_workspace(B, H, N, d)
    sv.sv_linattn_workspace_init(ws, B, H, d)
    S, z = new_state(B, H, d)
    S.fill_(3.0)
    z.fill_(5.0)
    O = torch.full_like(Qd, float("nan"))
    try:
        sv.sv_linattn_set_wait_limit(0)
        sv.sv_linattn_state(Kd, Vd, dsc, 0, N, 1, S, z, ws)
        sv.sv_block_linattn_step(Qd, Kd, Vd, dsc, S, z, 1e-6, O, ws)
        torch.cuda.synchronize()
    finally:
        sv.sv_linattn_set_wait_limit(-1)
    assert sv.sv_linattn_workspace_status(ws, B, H, d) == 1
    assert bool((S == 3.0).all()) and bool((z == 5.0).all()), "a timed-out call changed the carried state"
    if d == 64:                       # one launch: the apply phase is skipped too
        assert bool(torch.isnan(O.float()).all()), "a timed-out block step wrote rows of O"
    sv.sv_linattn_workspace_init(ws, B, H, d)
    assert sv.sv_linattn_workspace_status(ws, B, H, d) == 0
    S.zero_()
    z.zero_()
    sv.sv_block_linattn_step(Qd, Kd, Vd, dsc, S, z, 1e-6, O, ws)
    torch.cuda.synchronize()
    assert sv.sv_linattn_workspace_status(ws, B, H, d) == 0
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6)
    _check_state(S, z, S_ref, z_ref, "after the timeout")
    metrics.check(to_host(O), O_ref, "bf16", "O after the timeout")


def test_head_spread_over_dies_gives_up_and_is_reported():
    """The die-local block step checks where its workgroups really run.  Told to place heads as if the device
    had four dies, every head ends up on two: the step must store nothing (S, z, O as they were), set the
    mark that the status query reads, and work again once the real die count is back."""
    import torch
    B, H, N, d = 1, 32, 4680, 64
    say("head spread over dies")
    Q, K, V = _draw(7980, B, H, N, d, "bf16")
    Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
    dsc = sv.desc_of(Qd)
    ws = new_workspace(B, H, N, d)
    sv.sv_linattn_workspace_init(ws, B, H, d)
    S, z = new_state(B, H, d)
    S.fill_(3.0)
    z.fill_(5.0)
    O = torch.full_like(Qd, float("nan"))
    try:
        sv.sv_measure_assume_dies(4)
        sv.sv_block_linattn_step(Qd, Kd, Vd, dsc, S, z, 1e-6, O, ws)
        torch.cuda.synchronize()
    finally:
        sv.sv_measure_assume_dies(8)
    if sv.sv_linattn_workspace_status(ws, B, H, d) == 0:
        pytest.skip("this device did not take the die-local form (not the 8 x 32 compute-unit part)")
    assert bool((S == 3.0).all()) and bool((z == 5.0).all()) and bool(torch.isnan(O.float()).all())
    sv.sv_linattn_workspace_init(ws, B, H, d)
    S.zero_()
    z.zero_()
    sv.sv_block_linattn_step(Qd, Kd, Vd, dsc, S, z, 1e-6, O, ws)
    torch.cuda.synchronize()
    assert sv.sv_linattn_workspace_status(ws, B, H, d) == 0
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6)
    _check_state(S, z, S_ref, z_ref, "after the refused step")
    metrics.check(to_host(O), O_ref, "bf16", "O after the refused step")


@pytest.mark.parametrize("H,d", [(32, 64), (20, 112)])
def test_workspace_reinitialised_between_uses(H, d):
    """Device-side epochs restart when a workspace is initialised again, so a flag left by the single
    launch of its earlier life equals the first epoch of the new one: initialisation must clear the flags,
    or the second call below folds partials that are not there yet."""
    import torch
    B, N = 1, 4680
    say(f"workspace_reinitialised H={H} d={d}")
    _, K0, V0 = _draw(7970, B, H, N, d, "bf16")
    _, K1, V1 = _draw(7971, B, H, N, d, "bf16")
    ws = new_workspace(B, H, N, d)
    S, z = new_state(B, H, d)
    for K, V in ((K0, V0), (K1, V1)):
        Kd, Vd = to_dev(K), to_dev(V)
        sv.sv_linattn_workspace_init(ws, B, H, d)
        sv.sv_linattn_state(Kd, Vd, sv.desc_of(Kd), 0, N, 0, S, z, ws)
        torch.cuda.synchronize()
        S_ref, z_ref = orc.state(K, V)
        _check_state(S, z, S_ref, z_ref, "state after (re)initialisation")
    assert sv.sv_linattn_workspace_status(ws, B, H, d) == 0


# ---- look-ahead step: the cache is used but not updated (noisy passes of Alg. 1) -------------------

@pytest.mark.parametrize("dtype,d,H", [("bf16", 64, 8), ("f32", 32, 2), ("bf16", 64, 300), ("bf16", 112, 20),
                                       ("bf16", 128, 7), ("f32", 128, 2)])
def test_lookahead_leaves_state_untouched(dtype, d, H):
    import torch
    B, N0, N1 = 1, 900, 333
    say(f"lookahead dtype={dtype} d={d} H={H}")
    Q0, K0, V0 = _draw(8000, B, H, N0, d, dtype)
    Q1, K1, V1 = _draw(8001, B, H, N1, d, dtype)
    S, z = new_state(B, H, d)
    ws = new_workspace(B, H, max(N0, N1), d)
    d0 = [to_dev(t) for t in (Q0, K0, V0)]
    d1 = [to_dev(t) for t in (Q1, K1, V1)]
    O0 = torch.empty_like(d0[0])
    sv.sv_block_linattn_step(*d0, sv.desc_of(d0[0]), S, z, 1e-6, O0, ws)        # some carried state
    torch.cuda.synchronize()
    S_before, z_before = S.clone(), z.clone()
    O_look = torch.empty_like(d1[0])
    sv.sv_block_linattn_lookahead(*d1, sv.desc_of(d1[0]), S, z, 1e-6, O_look, ws)
    torch.cuda.synchronize()
    assert torch.equal(S, S_before) and torch.equal(z, z_before)
    O_commit = torch.empty_like(d1[0])
    sv.sv_block_linattn_step(*d1, sv.desc_of(d1[0]), S, z, 1e-6, O_commit, ws)
    torch.cuda.synchronize()
    assert not torch.equal(S, S_before)
    # both passes see the same updated state, so their outputs are bit-identical
    view = torch.int16 if dtype == "bf16" else torch.int32
    assert torch.equal(O_look.view(view), O_commit.view(view))
    S0r, z0r = orc.state(K0, V0)
    O_ref, S_same, z_same = orc.block_step(Q1, K1, V1, S0r, z0r, 1e-6, commit=False)
    assert np.array_equal(S_same, S0r)
    metrics.check(to_host(O_look), O_ref, dtype, "lookahead O")
    _, S1r, z1r = orc.block_step(Q1, K1, V1, S0r, z0r, 1e-6, commit=True)
    _check_state(S, z, S1r, z1r, "state after the committing pass")


# ---- guard words: nothing outside the buffers a call is given may change -------------------------------

def _guarded(nbytes, dtype, pattern=0xC3):
    """A device buffer of `nbytes` with 4 KiB of a byte pattern in front of it and behind it.
    Returns (whole allocation, view of the payload reinterpreted as `dtype`)."""
    import torch
    pad = 4096
    whole = torch.full((pad + nbytes + pad,), pattern, dtype=torch.uint8, device="cuda")
    return whole, whole[pad:pad + nbytes].view(dtype)


def _guards_intact(whole, nbytes, pattern=0xC3):
    pad = 4096
    return bool((whole[:pad] == pattern).all()) and bool((whole[pad + nbytes:] == pattern).all())


@pytest.mark.parametrize("dtype,d,H,N", [("bf16", 64, 32, 4681), ("bf16", 64, 3, 333), ("bf16", 112, 20, 4680),
                                         ("bf16", 128, 5, 1000), ("f32", 32, 2, 1024), ("bf16", 32, 4, 777)])
def test_nothing_is_written_outside_the_buffers(dtype, d, H, N):
    """S, z, O and the workspace each sit between guard areas; after a state + apply pair, a committing step
    and a look-ahead step (on ragged lengths: the kernels' last tiles reach past the token range and rely on
    the buffer resources' range checks) every guard byte must be as it was, and the results must be right."""
    import torch
    B = 1
    say(f"guard words dtype={dtype} d={d} H={H} N={N}")
    Q, K, V = _draw(8100 + N, B, H, N, d, dtype)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    esz = 2 if dtype == "bf16" else 4
    tok_bytes = B * H * N * d * esz
    bufs = {}
    for name, src in (("Q", Q), ("K", K), ("V", V)):
        whole, view = _guarded(tok_bytes, tdt)
        view.view(B, H, N, d).copy_(to_dev(src))
        bufs[name] = (whole, view.view(B, H, N, d))
    O_w, O = _guarded(tok_bytes, tdt)
    O = O.view(B, H, N, d)
    S_w, S = _guarded(B * H * d * d * 4, torch.float32)
    z_w, z = _guarded(B * H * d * 4, torch.float32)
    ws_bytes = sv.sv_linattn_workspace_bytes(B, H, N, d)
    ws_w, ws = _guarded(ws_bytes, torch.uint8)
    S, z = S.view(B, H, d, d), z.view(B, H, d)
    Qd, Kd, Vd = bufs["Q"][1], bufs["K"][1], bufs["V"][1]
    dsc = sv.desc_of(Qd)
    sv.sv_linattn_state(Kd, Vd, dsc, 0, N, 0, S, z, ws, workspace_bytes=ws_bytes)
    sv.sv_linattn_apply(Qd, dsc, 0, N, S, z, 1e-6, O)
    torch.cuda.synchronize()
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6)
    _check_state(S, z, S_ref, z_ref, "guarded state")
    metrics.check(to_host(O), O_ref, dtype, "guarded O")
    sv.sv_block_linattn_lookahead(Qd, Kd, Vd, dsc, S, z, 1e-6, O, ws, workspace_bytes=ws_bytes)
    sv.sv_block_linattn_step(Qd, Kd, Vd, dsc, S, z, 1e-6, O, ws, workspace_bytes=ws_bytes)
    torch.cuda.synchronize()
    O2_ref, S2_ref, z2_ref = orc.block_step(Q, K, V, S_ref, z_ref, 1e-6)
    _check_state(S, z, S2_ref, z2_ref, "guarded state after the step")
    metrics.check(to_host(O), O2_ref, dtype, "guarded O of the step")
    for name, (whole, _) in bufs.items():
        assert _guards_intact(whole, tok_bytes), f"guard of {name} changed"
    assert _guards_intact(O_w, tok_bytes), "a kernel wrote outside O"
    assert _guards_intact(S_w, B * H * d * d * 4), "a kernel wrote outside S"
    assert _guards_intact(z_w, B * H * d * 4), "a kernel wrote outside z"
    assert _guards_intact(ws_w, ws_bytes), "a kernel wrote outside the workspace"


def test_long_stream_resumes_bit_identically():
    """80 blocks with the state carried; the stream is cut after every 16th block (state copied to the host,
    device buffers freed, a fresh workspace) and must continue bit for bit like the uncut run."""
    import torch
    B, H, d, N, n_blocks = 1, 8, 64, 300, 80
    say("long stream resume")
    blocks = [_draw(8200 + i, B, H, N, d, "bf16") for i in range(n_blocks)]
    outs1, S1, z1 = _gpu_stream(blocks, 1e-6, B, H, d)
    S, z = new_state(B, H, d)
    ws = new_workspace(B, H, N, d)
    for i, blk in enumerate(blocks):
        if i and i % 16 == 0:
            Sh, zh = S.cpu(), z.cpu()
            del S, z, ws
            torch.cuda.empty_cache()
            S, z, ws = Sh.cuda(), zh.cuda(), new_workspace(B, H, N, d)
        Qd, Kd, Vd = (to_dev(t) for t in blk)
        O = torch.empty_like(Qd)
        sv.sv_block_linattn_step(Qd, Kd, Vd, sv.desc_of(Qd), S, z, 1e-6, O, ws)
        torch.cuda.synchronize()
        assert np.array_equal(to_host(O), outs1[i]), f"block {i}"
    assert torch.equal(S, S1) and torch.equal(z, z1)
