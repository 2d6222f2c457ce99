"""The yardsticks of include/sv_measure.h: the copy moves every byte (whole unrolled rounds, a
ragged tail, more workgroups than vectors), the read runs and leaves its input alone, the
matrix-core stream runs, scales with its step count and writes nothing."""
import pytest

import paper_2509_24695_amd as sv

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("nbytes,wgs", [(16, 1), (16 * 255, 3), (16 * (8 * 256 * 5 + 77), 7), (1 << 20, 4096),
                                        (268369920 // 2, 2048)])
def test_stream_copy_is_exact(nbytes, wgs):
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(nbytes % 9973 + wgs)
    src = torch.randint(0, 256, (nbytes + 64,), dtype=torch.uint8, device="cuda", generator=gen)
    dst = torch.full((nbytes + 64,), 0xA5, dtype=torch.uint8, device="cuda")
    keep = src.clone()
    sv.sv_stream_copy(src, dst, nbytes, wgs)
    torch.cuda.synchronize()
    assert torch.equal(dst[:nbytes], src[:nbytes])
    assert bool((dst[nbytes:] == 0xA5).all())            # nothing past the end
    assert torch.equal(src, keep)


def test_stream_read_runs():
    import torch
    src = torch.arange(1 << 22, dtype=torch.int32, device="cuda")
    keep = src.clone()
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    for wgs in (1, 256, 2048):
        sv.sv_stream_read(src, src.numel() * 4, sink, wgs)
    torch.cuda.synchronize()
    assert torch.equal(src, keep)


def test_mfma_stream_runs_and_scales():
    import torch
    sink = torch.full((4,), 7.0, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def us(wgs, steps):
        sv.sv_mfma_stream(wgs, steps, sink)
        torch.cuda.synchronize()
        a.record(stream)
        for _ in range(5):
            sv.sv_mfma_stream(wgs, steps, sink)
        b.record(stream)
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / 5

    short, long = us(8, 210), us(8, 840)
    assert bool((sink == 7.0).all())                     # the guarded store practically never happens
    # 32 MFMAs of 32x32x16 per wave and step: a step cannot take less than 32 * 8 passes * 4 cycles at 2.4 GHz
    assert short >= 210 * 32 * 32 / 2400.0 * 0.95, short
    assert 3.0 < long / short < 4.5, (short, long)       # four times the steps: about four times the time
    sv.sv_mfma_stream(1152, 1, sink)                     # many workgroups, one step
    torch.cuda.synchronize()


@pytest.mark.parametrize("B,H,N", [(1, 2, 100), (2, 3, 4681), (1, 32, 4680)])
def test_apply_variants_match_the_oracle_and_each_other(B, H, N):
    """sv_measure_apply_variant: the four forms of the d = 64 apply kernel (S in registers or in LDS,
    denominators through the matrix core or on the vector ALU) against the float64 oracle to the bf16
    tolerances; variant 0 is the kernel sv_linattn_apply runs, bit for bit; a sub-range leaves other rows alone."""
    import numpy as np
    import torch
    import sv_workloads as wl
    from oracle import linattn_oracle as orc
    from sv_workloads import metrics
    from tests.gpu_util import gpu_bidirectional, say, to_dev, to_host
    say(f"apply variants B={B} H={H} N={N}")
    Q, K, V = wl.draw_tensors(9900 + N, (B, H, N, 64), 0.5, "bf16")
    Qd = to_dev(Q)
    O0, S, z = gpu_bidirectional(Qd, to_dev(K), to_dev(V), 1e-6)
    O_ref, _, _ = orc.bidirectional(Q, K, V, 1e-6)
    dsc = sv.desc_of(Qd)
    outs = []
    for variant in range(4):
        O = torch.full_like(Qd, float("nan"))
        sv.sv_measure_apply_variant(variant, Qd, dsc, 0, N, S, z, 1e-6, O)
        torch.cuda.synchronize()
        metrics.check(to_host(O), O_ref, "bf16", f"variant {variant}")
        outs.append(O)
    assert torch.equal(outs[0].view(torch.int16), O0.view(torch.int16))
    assert torch.equal(outs[1].view(torch.int16), outs[0].view(torch.int16))      # same operands, read from LDS
    assert torch.equal(outs[3].view(torch.int16), outs[2].view(torch.int16))
    assert metrics.rel_l2(to_host(outs[2]), to_host(O0)) <= 2e-3                  # denominators summed in another order
    if N > 50:
        O = torch.full_like(Qd, 5.0)
        sv.sv_measure_apply_variant(3, Qd, dsc, 17, N - 9, S, z, 1e-6, O)
        torch.cuda.synchronize()
        assert torch.equal(O[:, :, 17:N - 9].view(torch.int16), outs[3][:, :, 17:N - 9].view(torch.int16))
        assert bool((O[:, :, :17] == 5.0).all()) and bool((O[:, :, N - 9:] == 5.0).all())
