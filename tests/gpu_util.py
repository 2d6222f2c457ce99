"""Helpers shared by the GPU parity tests: host<->device movement of stored
token tensors and small wrappers that call the library through its C ABI
binding.  No arithmetic of the method lives here."""
from __future__ import annotations

import sys

import numpy as np

import paper_2509_24695_amd as sv


def say(msg: str) -> None:
    """Name the case before each GPU step, flushed, so a fault can be attributed."""
    print(f"[gpu-case] {msg}", flush=True)
    sys.stdout.flush()


def to_dev(x: np.ndarray):
    """Stored tokens (uint16 bf16 bits or float32) -> device tensor of that dtype."""
    import torch
    if x.dtype == np.uint16:
        return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def to_host(t) -> np.ndarray:
    """Device tensor -> float32 numpy holding the stored values exactly."""
    import torch
    if t.dtype == torch.bfloat16:
        bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return t.contiguous().cpu().numpy()


def new_state(B, H, d):
    import torch
    S = torch.zeros((B, H, d, d), dtype=torch.float32, device="cuda")
    z = torch.zeros((B, H, d), dtype=torch.float32, device="cuda")
    return S, z


def new_workspace(B, H, n_tokens, d):
    import torch
    nbytes = sv.sv_linattn_workspace_bytes(B, H, n_tokens, d)
    assert nbytes > 0
    return torch.empty(nbytes, dtype=torch.uint8, device="cuda")


def gpu_bidirectional(Qd, Kd, Vd, eps, ws=None, poison=True):
    """state over all tokens (overwrite) + apply over all tokens, via the C ABI."""
    import torch
    B, H, N, d = Qd.shape
    S, z = new_state(B, H, d)
    if poison:                       # overwrite mode must not depend on old contents
        S.fill_(float("nan"))
        z.fill_(float("nan"))
    if ws is None:
        ws = new_workspace(B, H, N, d)
    O = torch.full_like(Qd, float("nan"))      # a row no kernel writes must not pass a comparison
    dsc = sv.desc_of(Kd)
    sv.sv_linattn_state(Kd, Vd, dsc, 0, N, 0, S, z, ws)
    sv.sv_linattn_apply(Qd, sv.desc_of(Qd), 0, N, S, z, eps, O)
    torch.cuda.synchronize()
    return O, S, z
