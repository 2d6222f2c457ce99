"""GPU parity of the RoPE variants (full equation of Sec. 3.2: rotated ReLU features in the numerator,
plain ones in the denominator) against the float64 oracle.

Tolerances: O as everywhere (bf16: max_rel 2e-2, rel_l2 5e-3; fp32 mode: 1e-5).  z is never rotated and
stays in the 1e-5 class.  In bf16 mode the rotated keys are rounded to bf16 before the MFMA, so S (the
state of rotated keys) carries that rounding: one bf16 rounding per term of a zero-mean sum gives a
relative L2 error of about 2^-9/sqrt(3) ~ 1.1e-3; the test allows 3e-3.  In fp32 mode S is held to 1e-5.
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


def _draw(seed, B, H, N, d, dtype):
    return wl.draw_tensors(seed, (B, H, N, d), 0.5, dtype)


def _random_table(N, d, seed):
    ang = np.random.default_rng(seed).uniform(-np.pi, np.pi, size=(N, d // 2))
    return np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)


def _dev_table(T):
    import torch
    return torch.from_numpy(np.ascontiguousarray(T)).cuda()


def _check_state(S, z, S_ref, z_ref, dtype, what):
    Sg, zg = to_host(S), to_host(z)
    assert np.isfinite(Sg).all() and np.isfinite(zg).all()
    assert metrics.rel_l2(Sg, S_ref) <= S_TOL[dtype], f"{what}: S rel_l2 {metrics.rel_l2(Sg, S_ref):.2e}"
    assert metrics.rel_l2(zg, z_ref) <= 1e-5 and metrics.max_rel(zg, z_ref) <= 1e-5, f"{what}: z"


@pytest.mark.parametrize("dtype,d", [("bf16", 64), ("f32", 32), ("bf16", 32), ("f32", 64), ("bf16", 112), ("bf16", 128),
                                     ("f32", 112)])
@pytest.mark.parametrize("B,H,N", [(1, 1, 1), (2, 3, 33), (1, 4, 1000), (1, 2, 4681)])
def test_rope_bidirectional(dtype, d, B, H, N):
    import torch
    say(f"rope_bidirectional dtype={dtype} d={d} B={B} H={H} N={N}")
    Q, K, V = _draw(9000 + N, B, H, N, d, dtype)
    T = _random_table(N, d, N)
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6, rope=T)
    Qd, Kd, Vd, Td = to_dev(Q), to_dev(K), to_dev(V), _dev_table(T)
    S, z = new_state(B, H, d)
    S.fill_(float("nan"))
    ws = new_workspace(B, H, N, d)
    O = torch.empty_like(Qd)
    dsc = sv.desc_of(Qd)
    sv.sv_linattn_state_rope(Kd, Vd, dsc, Td, 0, N, 0, S, z, ws)
    sv.sv_linattn_apply_rope(Qd, dsc, Td, 0, N, S, z, 1e-6, O)
    torch.cuda.synchronize()
    _check_state(S, z, S_ref, z_ref, dtype, "state")
    metrics.check(to_host(O), O_ref, dtype, "O")


def test_rope_apply_from_exact_state_and_ranges():
    """Apply alone, fed the oracle's state: isolates the query-side rotation; token sub-range."""
    import torch
    B, H, N, d = 1, 3, 777, 64
    say("rope_apply_from_exact_state")
    Q, K, V = _draw(9100, B, H, N, d, "bf16")
    T = _random_table(N, d, 11)
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6, rope=T)
    Qd, Td = to_dev(Q), _dev_table(T)
    Sd = torch.from_numpy(S_ref.astype(np.float32)).cuda()
    zd = torch.from_numpy(z_ref.astype(np.float32)).cuda()
    O = torch.full_like(Qd, 3.0)
    sv.sv_linattn_apply_rope(Qd, sv.desc_of(Qd), Td, 100, 701, Sd, zd, 1e-6, O)
    torch.cuda.synchronize()
    Oh = to_host(O)
    assert (Oh[:, :, :100] == 3.0).all() and (Oh[:, :, 701:] == 3.0).all()
    metrics.check(Oh[:, :, 100:701], O_ref[:, :, 100:701], "bf16", "O range")
    # state over two ranges with accumulate
    Kd, Vd = to_dev(K), to_dev(V)
    S, z = new_state(B, H, d)
    ws = new_workspace(B, H, N, d)
    sv.sv_linattn_state_rope(Kd, Vd, sv.desc_of(Kd), Td, 0, 300, 0, S, z, ws)
    sv.sv_linattn_state_rope(Kd, Vd, sv.desc_of(Kd), Td, 300, N, 1, S, z, ws)
    torch.cuda.synchronize()
    _check_state(S, z, S_ref, z_ref, "bf16", "two ranges")


def test_zero_angles_equal_the_plain_kernels_bitwise():
    import torch
    B, H, N, d = 1, 4, 1500, 64
    say("rope zero angles")
    Q, K, V = (to_dev(t) for t in _draw(9200, B, H, N, d, "bf16"))
    T = np.zeros((N, d // 2, 2), np.float32)
    T[..., 0] = 1.0
    Td = _dev_table(T)
    dsc = sv.desc_of(Q)
    ws = new_workspace(B, H, N, d)
    S1, z1 = new_state(B, H, d)
    S2, z2 = new_state(B, H, d)
    O1, O2 = torch.empty_like(Q), torch.empty_like(Q)
    sv.sv_linattn_state(K, V, dsc, 0, N, 0, S1, z1, ws)
    sv.sv_linattn_apply(Q, dsc, 0, N, S1, z1, 1e-6, O1)
    sv.sv_linattn_state_rope(K, V, dsc, Td, 0, N, 0, S2, z2, ws)
    sv.sv_linattn_apply_rope(Q, dsc, Td, 0, N, S2, z2, 1e-6, O2)
    torch.cuda.synchronize()
    assert torch.equal(S1, S2) and torch.equal(z1, z2) and torch.equal(O1.view(torch.int16), O2.view(torch.int16))


@pytest.mark.parametrize("dtype,d,H", [("bf16", 64, 32), ("f32", 32, 2), ("bf16", 64, 300), ("bf16", 112, 20),
                                       ("bf16", 128, 5)])
def test_rope_block_stream_with_3d_table(dtype, d, H):
    """Blocks of latent frames with a 3-D table whose time axis continues across blocks; the last
    block is also run as a look-ahead first."""
    import torch
    B, frames, rows, cols = 1, 2, 6, 9
    nb = frames * rows * cols
    say(f"rope_block_stream dtype={dtype} d={d} H={H} block={nb}")
    blocks = [_draw(9300 + m, B, H, nb, d, dtype) for m in range(3)]
    tables = [wl.rope_table_3d(frames, rows, cols, d, t0=m * frames) for m in range(3)]
    S, z = new_state(B, H, d)
    ws = new_workspace(B, H, nb, d)
    refs = list(orc.block_stream(blocks, 1e-6, ropes=tables))
    for m, (Q, K, V) in enumerate(blocks):
        Qd, Kd, Vd, Td = to_dev(Q), to_dev(K), to_dev(V), _dev_table(tables[m])
        O = torch.empty_like(Qd)
        if m == 2:
            S_keep, z_keep = S.clone(), z.clone()
            Ol = torch.empty_like(Qd)
            sv.sv_block_linattn_lookahead_rope(Qd, Kd, Vd, sv.desc_of(Qd), Td, S, z, 1e-6, Ol, ws)
            torch.cuda.synchronize()
            assert torch.equal(S, S_keep) and torch.equal(z, z_keep)
        sv.sv_block_linattn_step_rope(Qd, Kd, Vd, sv.desc_of(Qd), Td, S, z, 1e-6, O, ws)
        torch.cuda.synchronize()
        metrics.check(to_host(O), refs[m][0], dtype, f"block {m}")
        if m == 2:
            view = torch.int16 if dtype == "bf16" else torch.int32
            assert torch.equal(O.view(view), Ol.view(view))
    _check_state(S, z, refs[-1][1], refs[-1][2], dtype, "final state")


def test_rope_480p_full_size():
    """The 480p-like layer with its 21x30x52 3-D table: S, z and every element of O."""
    import torch
    w = wl.workload("bidir_480p")
    say(f"rope {w.name} full size")
    Q, K, V = wl.draw_qkv(w)
    T = wl.rope_table_3d(21, 30, 52, w.d)
    Qd, Kd, Vd, Td = to_dev(Q), to_dev(K), to_dev(V), _dev_table(T)
    S, z = new_state(w.B, w.H, w.d)
    ws = new_workspace(w.B, w.H, w.N, w.d)
    O = torch.full_like(Qd, float("nan"))
    dsc = sv.desc_of(Qd)
    sv.sv_linattn_state_rope(Kd, Vd, dsc, Td, 0, w.N, 0, S, z, ws)
    sv.sv_linattn_apply_rope(Qd, dsc, Td, 0, w.N, S, z, w.eps, O)
    torch.cuda.synchronize()
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, w.eps, rope=T)
    _check_state(S, z, S_ref, z_ref, "bf16", w.name)
    metrics.check(to_host(O), O_ref, "bf16", f"rope {w.name}")
