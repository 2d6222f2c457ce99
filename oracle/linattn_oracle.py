"""ctypes front end of the float64 CPU oracle in linattn_oracle.c.

Test infrastructure only: tests, the smoke check and the benchmark's
CPU-baseline leg call this; the GPU library never does.  Inputs may be bf16 bit
patterns (uint16) or float32 arrays; both are widened exactly before the C code
sees them.  All results are float64 numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "linattn_oracle.c")
_LIB = os.path.join(_HERE, "liblinattn_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O3, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-std=c11",
               "-Wall", "-Wextra", "-shared", "-fPIC", _SRC, "-o", _LIB + ".tmp"]
        subprocess.run(cmd, check=True)
        os.replace(_LIB + ".tmp", _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, dbl, vp = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.orc_num_threads.restype = ctypes.c_int
        lib.orc_state.argtypes = [vp, vp, vp, i64, i64, i64, i64, i64, i64, ctypes.c_int, vp, vp]
        lib.orc_apply.argtypes = [vp, vp, i64, i64, i64, i64, i64, i64, vp, vp, dbl, vp]
        lib.orc_bidirectional.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, dbl, vp, vp, vp]
        lib.orc_block_step.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, dbl, vp, vp,
                                       ctypes.c_int, vp, vp, vp]
        for f in (lib.orc_state, lib.orc_apply, lib.orc_bidirectional, lib.orc_block_step):
            f.restype = None
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().orc_num_threads())


def _widen(x: np.ndarray) -> np.ndarray:
    """Stored tokens -> contiguous float32 [B][H][N][d], exactly."""
    x = np.asarray(x)
    if x.dtype == np.uint16:      # bf16 bit patterns
        x = (x.astype(np.uint32) << np.uint32(16)).view(np.float32)
    elif x.dtype != np.float32:
        raise TypeError(f"tokens must be uint16 (bf16 bits) or float32, got {x.dtype}")
    if x.ndim != 4:
        raise ValueError("tokens must be [B][H][N][d]")
    if x.shape[3] > 256:
        raise ValueError("head dim above the oracle's limit of 256")
    return np.ascontiguousarray(x)


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _rope(rope, N, d):
    """Rotation table [N][d/2][2] (cos, sin) as contiguous float32, or None."""
    if rope is None:
        return None
    r = np.ascontiguousarray(rope, dtype=np.float32)
    if r.shape != (N, d // 2, 2):
        raise ValueError(f"rope table must be [N][d/2][2] = {(N, d // 2, 2)}, got {r.shape}")
    return r


def state(K, V, t0=None, t1=None, S=None, z=None, rope=None):
    """S, z over tokens [t0, t1); if S and z are given the sums are added to
    copies of them (the caller's arrays are not modified)."""
    K, V = _widen(K), _widen(V)
    if K.shape != V.shape:
        raise ValueError("K and V shapes differ")
    B, H, N, d = K.shape
    t0 = 0 if t0 is None else int(t0)
    t1 = N if t1 is None else int(t1)
    if not 0 <= t0 <= t1 <= N:
        raise ValueError("token range out of bounds")
    acc = S is not None
    if acc:
        S = np.array(S, dtype=np.float64, copy=True).reshape(B, H, d, d)
        z = np.array(z, dtype=np.float64, copy=True).reshape(B, H, d)
    else:
        S = np.empty((B, H, d, d), np.float64)
        z = np.empty((B, H, d), np.float64)
    _load().orc_state(_p(K), _p(V), _p(_rope(rope, N, d)), B, H, N, d, t0, t1, int(acc), _p(S), _p(z))
    return S, z


def apply(Q, S, z, eps, t0=None, t1=None, rope=None):
    """O for tokens [t0, t1) (shape [B][H][t1-t0][d]) from a given state."""
    Q = np.asarray(Q)
    if Q.ndim != 4:
        raise ValueError("tokens must be [B][H][N][d]")
    N = Q.shape[2]
    t0 = 0 if t0 is None else int(t0)
    t1 = N if t1 is None else int(t1)
    if not 0 <= t0 <= t1 <= N:
        raise ValueError("token range out of bounds")
    Q = _widen(Q[:, :, t0:t1, :])                 # only the rows that are asked for
    B, H, n, d = Q.shape
    rope = None if rope is None else _rope(np.asarray(rope)[t0:t1], n, d)
    S = np.ascontiguousarray(S, dtype=np.float64).reshape(B, H, d, d)
    z = np.ascontiguousarray(z, dtype=np.float64).reshape(B, H, d)
    O = np.zeros((B, H, n, d), np.float64)
    _load().orc_apply(_p(Q), _p(rope), B, H, n, d, 0, n, _p(S), _p(z), float(eps), _p(O))
    return O


def bidirectional(Q, K, V, eps, rope=None):
    """O, S, z of a bidirectional layer."""
    Q, K, V = _widen(Q), _widen(K), _widen(V)
    if not (Q.shape == K.shape == V.shape):
        raise ValueError("Q, K, V shapes differ")
    B, H, N, d = Q.shape
    O = np.empty((B, H, N, d), np.float64)
    S = np.empty((B, H, d, d), np.float64)
    z = np.empty((B, H, d), np.float64)
    _load().orc_bidirectional(_p(Q), _p(K), _p(V), _p(_rope(rope, N, d)), B, H, N, d, float(eps), _p(O), _p(S),
                              _p(z))
    return O, S, z


def block_step(Qb, Kb, Vb, S, z, eps, commit=True, rope=None):
    """One block of the block-causal stream. Returns (O_b, S_new, z_new); with
    commit=False the returned state equals the state passed in."""
    Qb, Kb, Vb = _widen(Qb), _widen(Kb), _widen(Vb)
    if not (Qb.shape == Kb.shape == Vb.shape):
        raise ValueError("Q, K, V shapes differ")
    B, H, Nb, d = Qb.shape
    S = np.array(S, dtype=np.float64, copy=True).reshape(B, H, d, d)
    z = np.array(z, dtype=np.float64, copy=True).reshape(B, H, d)
    St, zt = np.empty_like(S), np.empty_like(z)
    Ob = np.empty((B, H, Nb, d), np.float64)
    _load().orc_block_step(_p(Qb), _p(Kb), _p(Vb), _p(_rope(rope, Nb, d)), B, H, Nb, d, float(eps), _p(S), _p(z),
                           int(bool(commit)), _p(St), _p(zt), _p(Ob))
    return Ob, S, z


def zero_state(B, H, d):
    """Empty cache: the state before the first block (Alg. 1 starts from none)."""
    return np.zeros((B, H, d, d), np.float64), np.zeros((B, H, d), np.float64)


def block_stream(blocks, eps, S=None, z=None, ropes=None):
    """Run block_step over an iterable of (Qb, Kb, Vb); yields (O_b, S, z) after
    each block, starting from the given state or from the empty cache.  `ropes`
    is an optional sequence of per-block rotation tables."""
    for m, (Qb, Kb, Vb) in enumerate(blocks):
        if S is None:
            B, H, _, d = np.asarray(Qb).shape
            S, z = zero_state(B, H, d)
        Ob, S, z = block_step(Qb, Kb, Vb, S, z, eps, commit=True, rope=None if ropes is None else ropes[m])
        yield Ob, S, z
