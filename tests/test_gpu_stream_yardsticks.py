"""The streaming yardsticks of include/sv_measure.h: the copy moves every byte (whole unrolled
rounds, a ragged tail, more workgroups than vectors), the read runs and leaves its input alone."""
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
