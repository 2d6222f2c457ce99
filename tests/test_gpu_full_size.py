"""GPU parity at the full sizes of the workloads, in the launch
configuration bench.py times.  Every element of S, z and O is compared with the
float64 oracle's: a tile skipped or visited twice anywhere in a head's walk shows
up, whatever the sequence length, head count or chunk count.  O tensors are
filled with NaN before the call, so a row that no kernel wrote cannot pass.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import paper_2509_24695_amd as sv
import sv_workloads as wl
from oracle import linattn_oracle as orc
from sv_workloads import metrics
from tests.gpu_util import gpu_bidirectional, new_state, new_workspace, say, to_dev, to_host

pytestmark = pytest.mark.gpu

STATE_TOL = 1e-5


def _check_state(S, z, S_ref, z_ref, what):
    for name, g, r in (("S", S, S_ref), ("z", z, z_ref)):
        g = to_host(g)
        assert np.isfinite(g).all(), f"{what}: non-finite {name}"
        assert metrics.rel_l2(g, r) <= STATE_TOL and metrics.max_rel(g, r) <= STATE_TOL, \
            f"{what}: {name} rel_l2 {metrics.rel_l2(g, r):.2e} max_rel {metrics.max_rel(g, r):.2e}"


@pytest.mark.parametrize("name", ["bidir_480p", "bidir_480p_h20d112"])
def test_bidir_480p_full(name):
    w = wl.workload(name)
    say(f"{w.name} full size B={w.B} H={w.H} N={w.N}")
    Q, K, V = wl.draw_qkv(w)
    O, S, z = gpu_bidirectional(to_dev(Q), to_dev(K), to_dev(V), w.eps)
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, w.eps)
    _check_state(S, z, S_ref, z_ref, w.name)
    m = metrics.check(to_host(O), O_ref, "bf16", w.name)
    print(f"{w.name}: {m}")
    # closed-form magnitude of the key sum for these inputs: N * sigma / sqrt(2 pi)
    assert abs(to_host(z).mean() / (w.N * 0.5 / np.sqrt(2 * np.pi)) - 1) < 5e-3


def test_bidir_720p_full():
    """The largest single-GPU workload (conditional + unconditional pair, 64 heads of 75 600 tokens):
    S, z and every element of O."""
    w = wl.workload("bidir_720p")
    say(f"{w.name} full size B={w.B} H={w.H} N={w.N}")
    Q, K, V = wl.draw_qkv(w)
    O, S, z = gpu_bidirectional(to_dev(Q), to_dev(K), to_dev(V), w.eps)
    O_host = to_host(O)
    del O
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, w.eps)
    _check_state(S, z, S_ref, z_ref, w.name)
    m = metrics.check(O_host, O_ref, "bf16", w.name)
    print(f"{w.name}: {m}")


@pytest.mark.parametrize("name", ["block_480p", "block_480p_h20d112"])
def test_block_480p_full(name):
    import torch
    w = wl.workload(name)
    say(f"{w.name} full size: {w.n_blocks} blocks of {w.N} tokens")
    Q, K, V = wl.draw_qkv(w)
    Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
    S, z = new_state(w.B, w.H, w.d)
    ws = new_workspace(w.B, w.H, w.N, w.d)
    Od = torch.full_like(Qd, float("nan"))
    for m in range(w.n_blocks):              # blocks are token slices of one tensor: strides do the slicing
        sl = slice(m * w.N, (m + 1) * w.N)
        q, k, v, o = (t[:, :, sl] for t in (Qd, Kd, Vd, Od))
        sv.sv_block_linattn_step(q, k, v, sv.desc_of(q), S, z, w.eps, o, ws)
    torch.cuda.synchronize()
    O_host = to_host(Od)
    blocks = [tuple(np.ascontiguousarray(t[:, :, m * w.N:(m + 1) * w.N]) for t in (Q, K, V))
              for m in range(w.n_blocks)]
    S_ref = z_ref = None
    for m, (O_ref, S_ref, z_ref) in enumerate(orc.block_stream(blocks, w.eps)):
        metrics.check(O_host[:, :, m * w.N:(m + 1) * w.N], O_ref, "bf16", f"{w.name} block {m}")
    _check_state(S, z, S_ref, z_ref, f"{w.name} final state")


def test_stream_720p_full():
    """80 blocks, state carried on the device; per-block inputs from per-block seeds; every element of
    every block's O, and S, z at the end."""
    import torch
    w = wl.workload("stream_720p")
    say(f"{w.name} full size: {w.n_blocks} blocks of {w.N} tokens ")
    S, z = new_state(w.B, w.H, w.d)
    ws = new_workspace(w.B, w.H, w.N, w.d)
    lib_bytes = S.numel() * 4 + z.numel() * 4 + ws.numel()
    S_ref, z_ref = orc.zero_state(w.B, w.H, w.d)
    group = 8
    worst = {"max_rel": 0.0, "rel_l2": 0.0}
    with ThreadPoolExecutor(max_workers=group) as pool:
        for g0 in range(0, w.n_blocks, group):
            drawn = list(pool.map(lambda m: wl.draw_block(w, m), range(g0, min(w.n_blocks, g0 + group))))
            for i, (Q, K, V) in enumerate(drawn):
                m = g0 + i
                Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
                O = torch.full_like(Qd, float("nan"))
                sv.sv_block_linattn_step(Qd, Kd, Vd, sv.desc_of(Qd), S, z, w.eps, O, ws)
                torch.cuda.synchronize()
                O_ref, S_ref, z_ref = orc.block_step(Q, K, V, S_ref, z_ref, w.eps)
                mm = metrics.check(to_host(O), O_ref, "bf16", f"{w.name} block {m}")
                worst = {k: max(worst[k], mm[k]) for k in worst}
                # constant memory: nothing but S, z and the workspace belongs to the stream
                assert S.numel() * 4 + z.numel() * 4 + ws.numel() == lib_bytes
            print(f"{w.name}: blocks {g0}..{g0 + len(drawn) - 1} ok, worst so far {worst}", flush=True)
    _check_state(S, z, S_ref, z_ref, f"{w.name} final state after {w.n_blocks} blocks")
    # carried key sum after 864 000 tokens: closed form N sigma / sqrt(2 pi) = 172 342
    total = w.N * w.n_blocks
    assert abs(to_host(z).mean() / (total * 0.5 / np.sqrt(2 * np.pi)) - 1) < 2e-3


def test_rope_h20d112_full_size():
    """The paper's head geometry with the 3-D rotation table: S, z and every element of O; then the
    first blocks of the block-causal stream."""
    import torch
    w = wl.workload("bidir_480p_h20d112")
    say(f"rope {w.name} full size")
    Q, K, V = wl.draw_qkv(w)
    T = wl.rope_table_3d(*w.grid, w.d)
    Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
    Td = torch.from_numpy(T).cuda()
    S, z = new_state(w.B, w.H, w.d)
    ws = new_workspace(w.B, w.H, w.N, w.d)
    O = torch.full_like(Qd, float("nan"))
    dsc = sv.desc_of(Qd)
    sv.sv_linattn_state_rope(Kd, Vd, dsc, Td, 0, w.N, 0, S, z, ws)
    sv.sv_linattn_apply_rope(Qd, dsc, Td, 0, w.N, S, z, w.eps, O)
    torch.cuda.synchronize()
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, w.eps, rope=T)
    assert metrics.rel_l2(to_host(S), S_ref) <= 3e-3          # rotated keys are rounded to bf16 once more
    assert metrics.rel_l2(to_host(z), z_ref) <= STATE_TOL and metrics.max_rel(to_host(z), z_ref) <= STATE_TOL
    print(f"rope {w.name}: {metrics.check(to_host(O), O_ref, 'bf16', 'rope ' + w.name)}")
    # block stream: three blocks of three latent frames each, time axis continuing
    wb = wl.workload("block_480p_h20d112")
    S, z = new_state(wb.B, wb.H, wb.d)
    blocks = [tuple(np.ascontiguousarray(t[:, :, m * wb.N:(m + 1) * wb.N]) for t in (Q, K, V)) for m in range(3)]
    tables = [wl.rope_table_3d(*wb.grid, wb.d, t0=m * wb.grid[0]) for m in range(3)]
    refs = list(orc.block_stream(blocks, wb.eps, ropes=tables))
    for m, (q, k, v) in enumerate(blocks):
        qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
        o = torch.full_like(qd, float("nan"))
        sv.sv_block_linattn_step_rope(qd, kd, vd, sv.desc_of(qd), torch.from_numpy(tables[m]).cuda(), S, z, wb.eps, o, ws)
        torch.cuda.synchronize()
        metrics.check(to_host(o), refs[m][0], "bf16", f"rope block {m}")


@pytest.mark.parametrize("name", ["bidir_480p", "bidir_480p_h20d112"])
def test_rope3d_full_size(name):
    """The factored-table entry points at the size and in the launch configuration bench.py times:
    long tile walks (many strides per wave, staggered starts, the cyclic wrap); S, z and every element of
    O against the oracle on the expanded table; then three blocks of the block-causal stream with the
    time axis continuing."""
    import torch
    w = wl.workload(name)
    say(f"rope3d {w.name} full size B={w.B} H={w.H} N={w.N} d={w.d}")
    Q, K, V = wl.draw_qkv(w)
    T = wl.rope_table_3d(*w.grid, w.d)
    R = sv.Rope3D.from_tensors(*(torch.from_numpy(t).cuda() for t in wl.rope_tables_3d_factored(*w.grid, w.d)))
    Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
    S, z = new_state(w.B, w.H, w.d)
    ws = new_workspace(w.B, w.H, w.N, w.d)
    O = torch.full_like(Qd, float("nan"))
    dsc = sv.desc_of(Qd)
    sv.sv_linattn_state_rope3d(Kd, Vd, dsc, R, 0, w.N, 0, S, z, ws)
    sv.sv_linattn_apply_rope3d(Qd, dsc, R, 0, w.N, S, z, w.eps, O)
    torch.cuda.synchronize()
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, w.eps, rope=T)
    assert metrics.rel_l2(to_host(S), S_ref) <= 3e-3          # rotated keys are rounded to bf16 once more
    assert metrics.rel_l2(to_host(z), z_ref) <= STATE_TOL and metrics.max_rel(to_host(z), z_ref) <= STATE_TOL
    print(f"rope3d {w.name}: {metrics.check(to_host(O), O_ref, 'bf16', 'rope3d ' + w.name)}")
    # an apply over a range that starts and ends inside tiles: other rows stay untouched
    O2 = torch.full_like(Qd, 7.0)
    a, b = 4681, 23457
    sv.sv_linattn_apply_rope3d(Qd, dsc, R, a, b, S, z, w.eps, O2)
    torch.cuda.synchronize()
    assert torch.equal(O2[:, :, a:b], O[:, :, a:b])
    assert bool((O2[:, :, :a] == 7.0).all()) and bool((O2[:, :, b:] == 7.0).all())
    # block stream
    wb = wl.workload("block_480p" if w.d == 64 else "block_480p_h20d112")
    S, z = new_state(wb.B, wb.H, wb.d)
    blocks = [tuple(np.ascontiguousarray(t[:, :, m * wb.N:(m + 1) * wb.N]) for t in (Q, K, V)) for m in range(3)]
    tables = [wl.rope_table_3d(*wb.grid, wb.d, t0=m * wb.grid[0]) for m in range(3)]
    refs = list(orc.block_stream(blocks, wb.eps, ropes=tables))
    for m, (q, k, v) in enumerate(blocks):
        qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
        o = torch.full_like(qd, float("nan"))
        Rm = sv.Rope3D.from_tensors(*(torch.from_numpy(t).cuda()
                                      for t in wl.rope_tables_3d_factored(*wb.grid, wb.d, t0=m * wb.grid[0])))
        sv.sv_block_linattn_step_rope3d(qd, kd, vd, sv.desc_of(qd), Rm, S, z, wb.eps, o, ws)
        torch.cuda.synchronize()
        metrics.check(to_host(o), refs[m][0], "bf16", f"rope3d block {m}")
