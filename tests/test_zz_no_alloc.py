"""sv_block_linattn_step_static: the block step on the library's own file-scope workspace, for callers
that cannot allocate.  It must give what sv_block_linattn_step gives with a caller's workspace - the same
kernels run, so bit for bit - on calls in a row that share the one array, later ones with smaller inputs
that leave the earlier calls' partial states and flags lying in it."""
import numpy as np
import pytest

import paper_2509_24695_amd as sv
import sv_workloads as wl
from oracle import linattn_oracle as orc
from sv_workloads import metrics
from tests.gpu_util import new_state, new_workspace, say, to_dev, to_host

FAKE = 0x10000


def test_static_step_rejects_what_does_not_fit():
    """Checked on the host before any launch (runs without a GPU): the largest head counts per head dimension
    whose workspace fits SV_STATIC_SCRATCH_BYTES are accepted up to the next check, one more is refused."""
    def status(H, d, q=FAKE):
        dsc = sv.TensorDesc(1, H, 64, d, H * 64 * d, 64 * d, d, sv.SV_BF16)
        with pytest.raises(sv.SvError) as e:
            sv.sv_block_linattn_step_static(q, FAKE, FAKE, dsc, FAKE, FAKE, 1e-6, FAKE)
        return e.value.status
    limit = 48 << 20
    for d, most in ((64, 91), (112, 30), (128, 23)):
        assert sv.sv_linattn_workspace_bytes(1, most, 64, d) <= limit < sv.sv_linattn_workspace_bytes(1, most + 1, 64, d)
        assert status(most + 1, d) == 6                    # SV_ERR_WORKSPACE
        assert status(most, d, q=None) == 1                # fits: gets as far as the pointer checks
    with pytest.raises(sv.SvError) as e:
        sv.sv_block_linattn_step_static(FAKE, FAKE, FAKE, None, FAKE, FAKE, 1e-6, FAKE)
    assert e.value.status == 1


@pytest.mark.gpu
def test_static_step_equals_workspace_step_on_calls_in_a_row():
    import torch
    shapes = [(1, 32, 4680, 64), (1, 8, 1000, 64), (1, 20, 900, 112), (2, 3, 33, 64), (1, 32, 4680, 64)]
    for i, (B, H, N, d) in enumerate(shapes):
        say(f"static step call {i}: B={B} H={H} N={N} d={d}")
        blocks = [wl.draw_tensors(9100 + 10 * i + m, (B, H, N, d), 0.5, "bf16") for m in range(2)]
        ws = new_workspace(B, H, N, d)
        S_a, z_a = new_state(B, H, d)
        S_b, z_b = new_state(B, H, d)
        S_ref, z_ref = orc.zero_state(B, H, d)
        for m, (Q, K, V) in enumerate(blocks):               # the second block starts from a carried state
            Qd, Kd, Vd = to_dev(Q), to_dev(K), to_dev(V)
            dsc = sv.desc_of(Qd)
            O_a = torch.full_like(Qd, float("nan"))
            O_b = torch.full_like(Qd, float("nan"))
            sv.sv_block_linattn_step(Qd, Kd, Vd, dsc, S_a, z_a, 1e-6, O_a, ws)
            sv.sv_block_linattn_step_static(Qd, Kd, Vd, dsc, S_b, z_b, 1e-6, O_b)
            torch.cuda.synchronize()
            assert torch.equal(O_a.view(torch.int16), O_b.view(torch.int16)), f"call {i} block {m}: O differs"
            assert torch.equal(S_a, S_b) and torch.equal(z_a, z_b), f"call {i} block {m}: state differs"
            O_ref, S_ref, z_ref = orc.block_step(Q, K, V, S_ref, z_ref, 1e-6)
            metrics.check(to_host(O_b), O_ref, "bf16", f"static step call {i} block {m}")
        assert metrics.rel_l2(to_host(S_b), S_ref) <= 1e-5 and metrics.rel_l2(to_host(z_b), z_ref) <= 1e-5
