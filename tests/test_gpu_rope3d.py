"""GPU parity of the factored 3-D RoPE entry points (*_rope3d).

The factored tables are expanded on the host by pure indexing
(sv_workloads.expand_rope_tables; pinned against the full-table generator on the
CPU) and the results are checked (a) against the float64 oracle's full-table
form, to the tolerances of tests/test_gpu_rope.py, and (b) against the
library's own full-table entry points, with which they must agree bit for bit:
both rotate with the same fp32 (cos, sin) values in the same arithmetic.
"""
import numpy as np
import pytest

import paper_2509_24695_amd as sv
import sv_workloads as wl
from oracle import linattn_oracle as orc
from sv_workloads import metrics
from tests.gpu_util import new_state, new_workspace, say, to_dev, to_host

pytestmark = pytest.mark.gpu

S_TOL = {"bf16": 3e-3, "f32": 1e-5}


def _dev(x):
    import torch
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def _tables(frames, rows, cols, d, t0=0):
    cs = wl.rope_tables_3d_factored(frames, rows, cols, d, t0=t0)
    return cs, sv.Rope3D.from_tensors(*(_dev(t) for t in cs)), wl.expand_rope_tables(*cs)


def _same_bits(a, b):
    import torch
    view = torch.int16 if a.dtype == torch.bfloat16 else torch.int32
    return torch.equal(a.view(view), b.view(view))


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("bf16", 112), ("bf16", 128), ("f32", 32), ("bf16", 32), ("f32", 112)])
@pytest.mark.parametrize("B,H,grid", [(1, 1, (1, 1, 1)), (2, 3, (3, 5, 7)), (1, 4, (4, 16, 20)), (1, 2, (5, 30, 31))])
def test_rope3d_bidirectional(dtype, d, B, H, grid):
    import torch
    N = grid[0] * grid[1] * grid[2]
    say(f"rope3d_bidirectional dtype={dtype} d={d} B={B} H={H} grid={grid}")
    Q, K, V = wl.draw_tensors(9500 + N, (B, H, N, d), 0.5, dtype)
    _, R, T = _tables(*grid, d)
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6, rope=T)
    Qd, Kd, Vd, Td = to_dev(Q), to_dev(K), to_dev(V), _dev(T)
    dsc = sv.desc_of(Qd)
    ws = new_workspace(B, H, N, d)
    S, z = new_state(B, H, d)
    S.fill_(float("nan"))
    O = torch.empty_like(Qd)
    sv.sv_linattn_state_rope3d(Kd, Vd, dsc, R, 0, N, 0, S, z, ws)
    sv.sv_linattn_apply_rope3d(Qd, dsc, R, 0, N, S, z, 1e-6, O)
    torch.cuda.synchronize()
    assert metrics.rel_l2(to_host(S), S_ref) <= S_TOL[dtype]
    assert metrics.rel_l2(to_host(z), z_ref) <= 1e-5 and metrics.max_rel(to_host(z), z_ref) <= 1e-5
    metrics.check(to_host(O), O_ref, dtype, "O")
    # the full-table entry points on the expanded table
    S2, z2 = new_state(B, H, d)
    O2 = torch.empty_like(Qd)
    sv.sv_linattn_state_rope(Kd, Vd, dsc, Td, 0, N, 0, S2, z2, ws)
    sv.sv_linattn_apply_rope(Qd, dsc, Td, 0, N, S2, z2, 1e-6, O2)
    torch.cuda.synchronize()
    if dtype == "bf16" and d >= 112:
        # these two forms run different state kernels here (wave-private tiles with the factored
        # tables, one shared tile with the full table): same products, another summation order
        assert metrics.rel_l2(to_host(S), to_host(S2)) <= 1e-6 and metrics.rel_l2(to_host(z), to_host(z2)) <= 1e-6
        assert metrics.rel_l2(to_host(O), to_host(O2)) <= 1e-4
    else:
        assert torch.equal(S, S2) and torch.equal(z, z2) and _same_bits(O, O2)


def test_rope3d_token_ranges():
    import torch
    B, H, d, grid = 1, 3, 64, (3, 9, 11)
    N = grid[0] * grid[1] * grid[2]
    say("rope3d token ranges")
    Q, K, V = wl.draw_tensors(9600, (B, H, N, d), 0.5, "bf16")
    _, R, T = _tables(*grid, d)
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6, rope=T)
    Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
    dsc = sv.desc_of(Qd)
    ws = new_workspace(B, H, N, d)
    S, z = new_state(B, H, d)
    sv.sv_linattn_state_rope3d(Kd, Vd, dsc, R, 0, 100, 0, S, z, ws)
    sv.sv_linattn_state_rope3d(Kd, Vd, dsc, R, 100, N, 1, S, z, ws)
    O = torch.full_like(Qd, 3.0)
    sv.sv_linattn_apply_rope3d(Qd, dsc, R, 37, 250, S, z, 1e-6, O)
    torch.cuda.synchronize()
    assert metrics.rel_l2(to_host(S), S_ref) <= S_TOL["bf16"]
    Oh = to_host(O)
    assert (Oh[:, :, :37] == 3.0).all() and (Oh[:, :, 250:] == 3.0).all()
    metrics.check(Oh[:, :, 37:250], O_ref[:, :, 37:250], "bf16", "O range")


@pytest.mark.parametrize("dtype,d,H", [("bf16", 64, 32), ("bf16", 112, 20), ("bf16", 128, 5), ("f32", 32, 2),
                                       ("bf16", 64, 300)])
def test_rope3d_block_stream(dtype, d, H):
    """Blocks of two latent frames; the frame table of each block continues the time axis; the last
    block is also run as a look-ahead first.  Every block must equal the full-table step (bit for bit
    where both forms run the same kernels)."""
    import torch
    B, frames, rows, cols = 1, 2, 6, 9
    nb = frames * rows * cols
    say(f"rope3d_block_stream dtype={dtype} d={d} H={H}")
    blocks = [wl.draw_tensors(9700 + m, (B, H, nb, d), 0.5, dtype) for m in range(3)]
    per_block = [_tables(frames, rows, cols, d, t0=m * frames) for m in range(3)]
    refs = list(orc.block_stream(blocks, 1e-6, ropes=[t[2] for t in per_block]))
    S, z = new_state(B, H, d)
    S2, z2 = new_state(B, H, d)
    ws = new_workspace(B, H, nb, d)
    for m, (Q, K, V) in enumerate(blocks):
        Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
        R, Td = per_block[m][1], _dev(per_block[m][2])
        dsc = sv.desc_of(Qd)
        O, O2 = torch.empty_like(Qd), torch.empty_like(Qd)
        if m == 2:
            keep = S.clone()
            Ol = torch.empty_like(Qd)
            sv.sv_block_linattn_lookahead_rope3d(Qd, Kd, Vd, dsc, R, S, z, 1e-6, Ol, ws)
            torch.cuda.synchronize()
            assert torch.equal(S, keep)
        sv.sv_block_linattn_step_rope3d(Qd, Kd, Vd, dsc, R, S, z, 1e-6, O, ws)
        sv.sv_block_linattn_step_rope(Qd, Kd, Vd, dsc, Td, S2, z2, 1e-6, O2, ws)
        torch.cuda.synchronize()
        metrics.check(to_host(O), refs[m][0], dtype, f"block {m}")
        if dtype == "bf16" and d >= 112:     # different state kernels for the two forms: another summation order
            assert metrics.rel_l2(to_host(S), to_host(S2)) <= 1e-6 and metrics.rel_l2(to_host(z), to_host(z2)) <= 1e-6
            assert metrics.rel_l2(to_host(O), to_host(O2)) <= 1e-4, f"block {m} vs full table"
        else:
            assert _same_bits(O, O2) and torch.equal(S, S2) and torch.equal(z, z2), f"block {m} vs full table"
        if m == 2:
            assert _same_bits(O, Ol)


def test_rope3d_tables_too_large_for_lds():
    """A long single row of tokens whose column table exceeds the on-chip budget: the call
    still works (plain-FMA kernels read the tables from memory)."""
    import torch
    B, H, d, grid = 1, 2, 64, (1, 1, 1500)
    N = grid[2]
    say("rope3d tables too large for LDS")
    Q, K, V = wl.draw_tensors(9800, (B, H, N, d), 0.5, "bf16")
    ang = np.random.default_rng(3).uniform(-np.pi, np.pi, size=(N, d // 2))
    cs_w = np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)      # 1500 x 32 entries = 384 KB
    R = sv.Rope3D(1, 1, N, 0, 0, d // 2, None, None, _dev(cs_w))
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6, rope=cs_w)
    Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
    dsc = sv.desc_of(Qd)
    ws = new_workspace(B, H, N, d)
    S, z = new_state(B, H, d)
    O = torch.empty_like(Qd)
    sv.sv_linattn_state_rope3d(Kd, Vd, dsc, R, 0, N, 0, S, z, ws)
    sv.sv_linattn_apply_rope3d(Qd, dsc, R, 0, N, S, z, 1e-6, O)
    torch.cuda.synchronize()
    assert metrics.rel_l2(to_host(S), S_ref) <= 1e-5      # the plain-FMA path keeps rotated keys in fp32
    metrics.check(to_host(O), O_ref, "bf16", "O")
