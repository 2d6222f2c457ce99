"""HIP graph capture of the calls that synchronise workgroups inside a kernel.

A workspace prepared with sv_linattn_workspace_init takes its flag epochs from a
counter in device memory, so a captured launch sequence can be replayed.  The
graph is replayed several times, with eager calls and synchronisations in
between, and every replay is compared with the eager result (which itself is
checked against the oracle).
"""
import numpy as np
import pytest

import paper_2509_24695_amd as sv
import sv_workloads as wl
from oracle import linattn_oracle as orc
from sv_workloads import metrics
from tests.gpu_util import new_state, new_workspace, say, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("H,d,nb", [(32, 64, 1200), (20, 112, 700)])
def test_block_stream_graph_replays(H, d, nb):
    import torch
    B, n_blocks = 1, 4
    say(f"graph replay H={H} d={d} blocks of {nb}")
    blocks = [wl.draw_tensors(8800 + m, (B, H, nb, d), 0.5, "bf16") for m in range(n_blocks)]
    refs = list(orc.block_stream(blocks, 1e-6))
    dev = [tuple(to_dev(t) for t in blk) for blk in blocks]
    outs = [torch.empty_like(q) for (q, _, _) in dev]
    S, z = new_state(B, H, d)
    ws = new_workspace(B, H, nb, d)
    dsc = sv.desc_of(dev[0][0])

    def enqueue(stream=None):
        for (q, k, v), o in zip(dev, outs):
            sv.sv_block_linattn_step(q, k, v, dsc, S, z, 1e-6, o, ws, stream=stream)

    def zero_state():
        S.zero_()
        z.zero_()

    # eager, with host epochs (workspace not initialised) and again with device epochs
    for initialise in (False, True):
        if initialise:
            sv.sv_linattn_workspace_init(ws, B, H, d)
        zero_state()
        enqueue()
        torch.cuda.synchronize()
        for m in range(n_blocks):
            metrics.check(to_host(outs[m]), refs[m][0], "bf16", f"eager block {m} (init={initialise})")
    eager = [o.clone() for o in outs]
    S_eager, z_eager = S.clone(), z.clone()

    # capture the four steps once (S and z are zeroed by a fill kernel inside the graph)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        zero_state()
        enqueue(stream=side)                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph, stream=side):
        zero_state()
        enqueue(stream=torch.cuda.current_stream())
    for rep in range(4):
        for o in outs:
            o.fill_(7.0)
        S.fill_(3.0)
        graph.replay()
        torch.cuda.synchronize()
        for m in range(n_blocks):
            assert torch.equal(outs[m].view(torch.int16), eager[m].view(torch.int16)), f"replay {rep} block {m}"
        assert torch.equal(S, S_eager) and torch.equal(z, z_eager), f"replay {rep} state"
        # eager work between the replays, on the same workspace
        zero_state()
        sv.sv_block_linattn_step(dev[0][0], dev[0][1], dev[0][2], dsc, S, z, 1e-6, outs[0], ws)
        torch.cuda.synchronize()
        assert torch.equal(outs[0].view(torch.int16), eager[0].view(torch.int16))
    err = ws.numel() - 32 - 8 * B * H                     # the error word precedes magic, padding and the per-head tickets
    assert int(ws[err:err + 8].view(torch.int64)[0]) == 0     # no bounded wait ever timed out


def test_state_call_graph_replays():
    import torch
    B, H, N, d = 1, 32, 5000, 64
    say("graph replay of sv_linattn_state + sv_linattn_apply")
    Q, K, V = wl.draw_tensors(8900, (B, H, N, d), 0.5, "bf16")
    O_ref, S_ref, z_ref = orc.bidirectional(Q, K, V, 1e-6)
    Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
    S, z = new_state(B, H, d)
    ws = new_workspace(B, H, N, d)
    sv.sv_linattn_workspace_init(ws, B, H, d)
    O = torch.empty_like(Qd)
    dsc = sv.desc_of(Qd)

    def enqueue(stream=None):
        sv.sv_linattn_state(Kd, Vd, dsc, 0, N, 0, S, z, ws, stream=stream)
        sv.sv_linattn_apply(Qd, dsc, 0, N, S, z, 1e-6, O, stream=stream)

    enqueue()
    torch.cuda.synchronize()
    metrics.check(to_host(O), O_ref, "bf16", "eager")
    O_eager, S_eager = O.clone(), S.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue(stream=torch.cuda.current_stream())
    for rep in range(3):
        O.fill_(1.0)
        S.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(O.view(torch.int16), O_eager.view(torch.int16)) and torch.equal(S, S_eager), f"replay {rep}"
        enqueue()                                  # eager call between replays
        torch.cuda.synchronize()


def test_tconv_stream_graph_replays():
    """Three blocks of the temporal convolution with the cache updated in place, captured once and
    replayed; the cache is reset by a copy kernel inside the graph."""
    import torch
    from oracle import tconv_oracle as torc
    w = wl.TCONV_WORKLOADS["tconv_tiny"]
    say(f"graph replay of sv_tconv_block_step: B={w.B} T={w.T} HW={w.HW} D={w.D}, {w.n_blocks} blocks")
    xb, Wb = wl.draw_tconv(w)
    blocks = [np.ascontiguousarray(xb[:, m * w.T:(m + 1) * w.T]) for m in range(w.n_blocks)]
    xs, Wd = [to_dev(b) for b in blocks], to_dev(Wb)
    ys = [torch.empty_like(x) for x in xs]
    start = to_dev(np.ascontiguousarray(xb[:, 0]))            # some frame as the cache before block 0
    cache = torch.empty_like(start)

    def enqueue(stream=None):
        for x, y in zip(xs, ys):
            sv.sv_tconv_block_step(x, Wd, cache, y, cache, w.B, w.T, w.HW, w.D, stream=stream)

    cache.copy_(start)
    enqueue()                                                 # first call: one-time set-up happens outside the capture
    torch.cuda.synchronize()
    ref_cache = xb[:, 0]
    for m, blk in enumerate(blocks):
        y_ref, ref_cache = torc.tconv_block(blk, Wb, ref_cache)
        metrics.check(to_host(ys[m]), y_ref, "bf16", f"eager tconv block {m}")
    eager = [y.clone() for y in ys]
    cache_eager = cache.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        cache.copy_(start)
        enqueue(stream=torch.cuda.current_stream())
    for rep in range(3):
        for y in ys:
            y.fill_(5.0)
        cache.fill_(9.0)
        graph.replay()
        torch.cuda.synchronize()
        for m in range(w.n_blocks):
            assert torch.equal(ys[m].view(torch.int16), eager[m].view(torch.int16)), f"replay {rep} block {m}"
        assert torch.equal(cache.view(torch.int16), cache_eager.view(torch.int16)), f"replay {rep} cache"
        cache.copy_(start)                                    # eager work between the replays
        enqueue()
        torch.cuda.synchronize()
