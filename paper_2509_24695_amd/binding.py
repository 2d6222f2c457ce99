"""ctypes binding of libsvlinattn.so: argument marshalling only.

The functions carry the names and argument order of the C ABI
(include/sv_linattn.h, include/sv_tconv.h, include/sv_measure.h).  Device buffers are torch tensors (or raw integer
device addresses); nothing here computes, and there is no fallback: if the
shared library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

SV_BF16, SV_F32 = 0, 1

EXPORTS = (
    "sv_linattn_workspace_bytes", "sv_linattn_state", "sv_linattn_apply",
    "sv_block_linattn_step", "sv_block_linattn_lookahead", "sv_status_string", "sv_version",
    "sv_linattn_state_rope", "sv_linattn_apply_rope", "sv_block_linattn_step_rope",
    "sv_block_linattn_lookahead_rope", "sv_linattn_workspace_init",
    "sv_linattn_state_rope3d", "sv_linattn_apply_rope3d", "sv_block_linattn_step_rope3d",
    "sv_block_linattn_lookahead_rope3d", "sv_tconv_block_step", "sv_stream_read", "sv_stream_copy",
    "sv_linattn_workspace_status_offset", "sv_linattn_workspace_status", "sv_linattn_set_wait_limit",
    "sv_block_linattn_step_static", "sv_measure_apply_variant",
    "sv_measure_assume_dies", "sv_mfma_stream", "sv_measure_tconv_variant",
)

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libsvlinattn.so")
_lib = None


class SvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__(f"{where}: {sv_status_string(status)} (status {int(status)})")


class _CDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("N", ctypes.c_int32), ("d", ctypes.c_int32),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64), ("stride_n", ctypes.c_int64),
                ("dtype", ctypes.c_int32)]


@dataclass
class TensorDesc:
    """Mirror of sv_tensor_desc: [B][H][N][d] token tensor, strides in elements."""
    B: int
    H: int
    N: int
    d: int
    stride_b: int
    stride_h: int
    stride_n: int
    dtype: int

    def _c(self) -> _CDesc:
        return _CDesc(self.B, self.H, self.N, self.d, self.stride_b, self.stride_h, self.stride_n, self.dtype)


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libsvlinattn.so; raises if it has not been built (no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2509_24695_amd.build` "
            "(hipcc, --offload-arch=gfx950). There is no CPU or PyTorch fallback.")
    # PyTorch ships its own copy of the HIP runtime.  Callers hand this library device pointers
    # and streams that PyTorch made, so both must talk to one runtime: PyTorch's is loaded first
    # and the library's dependency on libamdhip64 then resolves to it.  Loaded the other way round
    # the process holds two runtimes and the first launch fails.
    import torch  # noqa: F401
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    dp = ctypes.POINTER(_CDesc)
    lib.sv_linattn_workspace_bytes.argtypes = [i32, i32, i32, i32]
    lib.sv_linattn_workspace_bytes.restype = sz
    lib.sv_linattn_state.argtypes = [vp, vp, dp, i32, i32, ctypes.c_int, vp, vp, vp, sz, vp]
    lib.sv_linattn_state.restype = ctypes.c_int
    lib.sv_linattn_apply.argtypes = [vp, dp, i32, i32, vp, vp, ctypes.c_float, vp, vp]
    lib.sv_linattn_apply.restype = ctypes.c_int
    lib.sv_block_linattn_step.argtypes = [vp, vp, vp, dp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
    lib.sv_block_linattn_step.restype = ctypes.c_int
    lib.sv_block_linattn_step_static.argtypes = [vp, vp, vp, dp, vp, vp, ctypes.c_float, vp, vp]
    lib.sv_block_linattn_step_static.restype = ctypes.c_int
    lib.sv_block_linattn_lookahead.argtypes = [vp, vp, vp, dp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
    lib.sv_block_linattn_lookahead.restype = ctypes.c_int
    lib.sv_linattn_state_rope.argtypes = [vp, vp, dp, vp, i32, i32, ctypes.c_int, vp, vp, vp, sz, vp]
    lib.sv_linattn_apply_rope.argtypes = [vp, dp, vp, i32, i32, vp, vp, ctypes.c_float, vp, vp]
    lib.sv_block_linattn_step_rope.argtypes = [vp, vp, vp, dp, vp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
    lib.sv_block_linattn_lookahead_rope.argtypes = [vp, vp, vp, dp, vp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
    for f in (lib.sv_linattn_state_rope, lib.sv_linattn_apply_rope, lib.sv_block_linattn_step_rope,
              lib.sv_block_linattn_lookahead_rope):
        f.restype = ctypes.c_int
    rp = ctypes.POINTER(_CRope3D)
    lib.sv_linattn_state_rope3d.argtypes = [vp, vp, dp, rp, i32, i32, ctypes.c_int, vp, vp, vp, sz, vp]
    lib.sv_linattn_apply_rope3d.argtypes = [vp, dp, rp, i32, i32, vp, vp, ctypes.c_float, vp, vp]
    lib.sv_block_linattn_step_rope3d.argtypes = [vp, vp, vp, dp, rp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
    lib.sv_block_linattn_lookahead_rope3d.argtypes = [vp, vp, vp, dp, rp, vp, vp, ctypes.c_float, vp, vp, sz, vp]
    for f in (lib.sv_linattn_state_rope3d, lib.sv_linattn_apply_rope3d, lib.sv_block_linattn_step_rope3d,
              lib.sv_block_linattn_lookahead_rope3d):
        f.restype = ctypes.c_int
    lib.sv_tconv_block_step.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp]
    lib.sv_tconv_block_step.restype = ctypes.c_int
    lib.sv_measure_apply_variant.argtypes = [i32, vp, dp, i32, i32, vp, vp, ctypes.c_float, vp, vp]
    lib.sv_measure_apply_variant.restype = ctypes.c_int
    lib.sv_measure_assume_dies.argtypes = [i32]
    lib.sv_measure_assume_dies.restype = None
    lib.sv_mfma_stream.argtypes = [i32, i32, vp, vp]
    lib.sv_measure_tconv_variant.argtypes = [i32, vp, vp, vp, vp, i32, i32, i32, i32, vp]
    lib.sv_measure_tconv_variant.restype = ctypes.c_int
    lib.sv_mfma_stream.restype = ctypes.c_int
    lib.sv_stream_read.argtypes = [vp, sz, vp, i32, vp]
    lib.sv_stream_read.restype = ctypes.c_int
    lib.sv_stream_copy.argtypes = [vp, vp, sz, i32, vp]
    lib.sv_stream_copy.restype = ctypes.c_int
    lib.sv_linattn_workspace_init.argtypes = [vp, sz, i32, i32, i32, vp]
    lib.sv_linattn_workspace_init.restype = ctypes.c_int
    lib.sv_linattn_workspace_status_offset.argtypes = [i32, i32, i32]
    lib.sv_linattn_workspace_status_offset.restype = sz
    lib.sv_linattn_workspace_status.argtypes = [vp, sz, i32, i32, i32, vp, ctypes.POINTER(ctypes.c_int32)]
    lib.sv_linattn_workspace_status.restype = ctypes.c_int
    lib.sv_linattn_set_wait_limit.argtypes = [ctypes.c_int64]
    lib.sv_linattn_set_wait_limit.restype = None
    lib.sv_status_string.argtypes = [ctypes.c_int]
    lib.sv_status_string.restype = ctypes.c_char_p
    lib.sv_version.argtypes = []
    lib.sv_version.restype = ctypes.c_int
    _lib = lib
    return lib


def _ptr(x):
    """Device address of a torch tensor, or an integer address / None as given."""
    if x is None:
        return None
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    return ctypes.c_void_p(x.data_ptr())


def _nbytes(x) -> int:
    return int(x.numel() * x.element_size())


def _stream(stream):
    if stream is None:
        return None
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)       # torch.cuda.Stream


def desc_of(t) -> TensorDesc:
    """Descriptor of a 4-D torch tensor [B][H][N][d] (bf16 or fp32, last dim contiguous)."""
    import torch
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("token tensors are [B][H][N][d] with d contiguous")
    if t.dtype == torch.bfloat16:
        dt = SV_BF16
    elif t.dtype == torch.float32:
        dt = SV_F32
    else:
        raise ValueError(f"unsupported dtype {t.dtype}")
    B, H, N, d = t.shape
    return TensorDesc(B, H, N, d, t.stride(0), t.stride(1), t.stride(2), dt)


def sv_status_string(status: int) -> str:
    return load_library().sv_status_string(int(status)).decode()


def sv_version() -> int:
    return int(load_library().sv_version())


def sv_linattn_workspace_bytes(B: int, H: int, n_tokens: int, d: int) -> int:
    return int(load_library().sv_linattn_workspace_bytes(B, H, n_tokens, d))


def _check(status: int, where: str):
    if status != 0:
        raise SvError(status, where)


def sv_linattn_state(K, V, kv: TensorDesc, tok_begin: int, tok_end: int, accumulate: int, S, z,
                     workspace, workspace_bytes: int | None = None, stream=None) -> None:
    d = kv._c() if kv is not None else None
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    _check(load_library().sv_linattn_state(_ptr(K), _ptr(V), ctypes.byref(d) if d else None, tok_begin, tok_end,
                                           int(accumulate), _ptr(S), _ptr(z), _ptr(workspace), wb,
                                           _stream(stream)), "sv_linattn_state")


def sv_linattn_apply(Q, q: TensorDesc, tok_begin: int, tok_end: int, S, z, eps: float, O, stream=None) -> None:
    d = q._c() if q is not None else None
    _check(load_library().sv_linattn_apply(_ptr(Q), ctypes.byref(d) if d else None, tok_begin, tok_end, _ptr(S),
                                           _ptr(z), float(eps), _ptr(O), _stream(stream)), "sv_linattn_apply")


def sv_block_linattn_step(Qb, Kb, Vb, blk: TensorDesc, S, z, eps: float, Ob, workspace,
                          workspace_bytes: int | None = None, stream=None) -> None:
    d = blk._c() if blk is not None else None
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    _check(load_library().sv_block_linattn_step(_ptr(Qb), _ptr(Kb), _ptr(Vb), ctypes.byref(d) if d else None,
                                                _ptr(S), _ptr(z), float(eps), _ptr(Ob), _ptr(workspace), wb,
                                                _stream(stream)), "sv_block_linattn_step")


def sv_block_linattn_step_static(Qb, Kb, Vb, blk: TensorDesc, S, z, eps: float, Ob, stream=None) -> None:
    """sv_block_linattn_step on the library's own static workspace (no allocation anywhere)."""
    d = blk._c() if blk is not None else None
    _check(load_library().sv_block_linattn_step_static(_ptr(Qb), _ptr(Kb), _ptr(Vb), ctypes.byref(d) if d else None,
                                                       _ptr(S), _ptr(z), float(eps), _ptr(Ob), _stream(stream)),
           "sv_block_linattn_step_static")


def sv_block_linattn_lookahead(Qb, Kb, Vb, blk: TensorDesc, S, z, eps: float, Ob, workspace,
                               workspace_bytes: int | None = None, stream=None) -> None:
    d = blk._c() if blk is not None else None
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    _check(load_library().sv_block_linattn_lookahead(_ptr(Qb), _ptr(Kb), _ptr(Vb), ctypes.byref(d) if d else None,
                                                     _ptr(S), _ptr(z), float(eps), _ptr(Ob), _ptr(workspace), wb,
                                                     _stream(stream)), "sv_block_linattn_lookahead")


def sv_linattn_state_rope(K, V, kv: TensorDesc, rope, tok_begin: int, tok_end: int, accumulate: int, S, z,
                          workspace, workspace_bytes: int | None = None, stream=None) -> None:
    d = kv._c() if kv is not None else None
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    _check(load_library().sv_linattn_state_rope(_ptr(K), _ptr(V), ctypes.byref(d) if d else None, _ptr(rope),
                                                tok_begin, tok_end, int(accumulate), _ptr(S), _ptr(z),
                                                _ptr(workspace), wb, _stream(stream)), "sv_linattn_state_rope")


def sv_linattn_apply_rope(Q, q: TensorDesc, rope, tok_begin: int, tok_end: int, S, z, eps: float, O,
                          stream=None) -> None:
    d = q._c() if q is not None else None
    _check(load_library().sv_linattn_apply_rope(_ptr(Q), ctypes.byref(d) if d else None, _ptr(rope), tok_begin,
                                                tok_end, _ptr(S), _ptr(z), float(eps), _ptr(O), _stream(stream)),
           "sv_linattn_apply_rope")


def _block_rope(fn_name, Qb, Kb, Vb, blk, rope, S, z, eps, Ob, workspace, workspace_bytes, stream):
    d = blk._c() if blk is not None else None
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    fn = getattr(load_library(), fn_name)
    _check(fn(_ptr(Qb), _ptr(Kb), _ptr(Vb), ctypes.byref(d) if d else None, _ptr(rope), _ptr(S), _ptr(z), float(eps),
              _ptr(Ob), _ptr(workspace), wb, _stream(stream)), fn_name)


def sv_block_linattn_step_rope(Qb, Kb, Vb, blk: TensorDesc, rope, S, z, eps: float, Ob, workspace,
                               workspace_bytes: int | None = None, stream=None) -> None:
    _block_rope("sv_block_linattn_step_rope", Qb, Kb, Vb, blk, rope, S, z, eps, Ob, workspace, workspace_bytes, stream)


def sv_block_linattn_lookahead_rope(Qb, Kb, Vb, blk: TensorDesc, rope, S, z, eps: float, Ob, workspace,
                                    workspace_bytes: int | None = None, stream=None) -> None:
    _block_rope("sv_block_linattn_lookahead_rope", Qb, Kb, Vb, blk, rope, S, z, eps, Ob, workspace, workspace_bytes,
                stream)


def sv_linattn_workspace_init(workspace, B: int, H: int, d: int, workspace_bytes: int | None = None,
                              stream=None) -> None:
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    _check(load_library().sv_linattn_workspace_init(_ptr(workspace), wb, int(B), int(H), int(d), _stream(stream)),
           "sv_linattn_workspace_init")


def sv_linattn_workspace_status_offset(B: int, H: int, d: int) -> int:
    return int(load_library().sv_linattn_workspace_status_offset(int(B), int(H), int(d)))


def sv_linattn_workspace_status(workspace, B: int, H: int, d: int, workspace_bytes: int | None = None,
                                stream=None) -> int:
    """1 if an in-kernel wait of a call on this workspace has timed out, else 0.  Synchronises `stream`."""
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    out = ctypes.c_int32(-1)
    _check(load_library().sv_linattn_workspace_status(_ptr(workspace), wb, int(B), int(H), int(d), _stream(stream),
                                                      ctypes.byref(out)), "sv_linattn_workspace_status")
    return int(out.value)


def sv_linattn_set_wait_limit(polls: int) -> None:
    """Bound of the in-kernel waits in polls; negative restores the default, 0 makes every wait fail."""
    load_library().sv_linattn_set_wait_limit(int(polls))


class _CRope3D(ctypes.Structure):
    _fields_ = [("frames", ctypes.c_int32), ("rows", ctypes.c_int32), ("cols", ctypes.c_int32),
                ("n_t", ctypes.c_int32), ("n_h", ctypes.c_int32), ("n_w", ctypes.c_int32),
                ("cs_t", ctypes.c_void_p), ("cs_h", ctypes.c_void_p), ("cs_w", ctypes.c_void_p)]


class Rope3D:
    """Factored 3-D rotary tables (sv_rope3d): device tensors (or raw pointers) cs_t [frames][n_t][2],
    cs_h [rows][n_h][2], cs_w [cols][n_w][2], fp32."""

    def __init__(self, frames, rows, cols, n_t, n_h, n_w, cs_t, cs_h, cs_w):
        self.frames, self.rows, self.cols = int(frames), int(rows), int(cols)
        self.n_t, self.n_h, self.n_w = int(n_t), int(n_h), int(n_w)
        self.cs_t, self.cs_h, self.cs_w = cs_t, cs_h, cs_w      # keeps the tensors alive

    @classmethod
    def from_tensors(cls, cs_t, cs_h, cs_w):
        return cls(cs_t.shape[0], cs_h.shape[0], cs_w.shape[0], cs_t.shape[1], cs_h.shape[1], cs_w.shape[1],
                   cs_t, cs_h, cs_w)

    def _c(self):
        def p(x):
            v = _ptr(x)
            return v.value if isinstance(v, ctypes.c_void_p) else v
        return _CRope3D(self.frames, self.rows, self.cols, self.n_t, self.n_h, self.n_w, p(self.cs_t), p(self.cs_h),
                        p(self.cs_w))


def _r3(rope):
    return ctypes.byref(rope._c()) if rope is not None else None


def sv_linattn_state_rope3d(K, V, kv: TensorDesc, rope: Rope3D, tok_begin: int, tok_end: int, accumulate: int, S, z,
                            workspace, workspace_bytes: int | None = None, stream=None) -> None:
    d = kv._c() if kv is not None else None
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    _check(load_library().sv_linattn_state_rope3d(_ptr(K), _ptr(V), ctypes.byref(d) if d else None, _r3(rope),
                                                  tok_begin, tok_end, int(accumulate), _ptr(S), _ptr(z),
                                                  _ptr(workspace), wb, _stream(stream)), "sv_linattn_state_rope3d")


def sv_linattn_apply_rope3d(Q, q: TensorDesc, rope: Rope3D, tok_begin: int, tok_end: int, S, z, eps: float, O,
                            stream=None) -> None:
    d = q._c() if q is not None else None
    _check(load_library().sv_linattn_apply_rope3d(_ptr(Q), ctypes.byref(d) if d else None, _r3(rope), tok_begin,
                                                  tok_end, _ptr(S), _ptr(z), float(eps), _ptr(O), _stream(stream)),
           "sv_linattn_apply_rope3d")


def _block_rope3d(fn_name, Qb, Kb, Vb, blk, rope, S, z, eps, Ob, workspace, workspace_bytes, stream):
    d = blk._c() if blk is not None else None
    wb = _nbytes(workspace) if workspace_bytes is None else int(workspace_bytes)
    fn = getattr(load_library(), fn_name)
    _check(fn(_ptr(Qb), _ptr(Kb), _ptr(Vb), ctypes.byref(d) if d else None, _r3(rope), _ptr(S), _ptr(z), float(eps),
              _ptr(Ob), _ptr(workspace), wb, _stream(stream)), fn_name)


def sv_block_linattn_step_rope3d(Qb, Kb, Vb, blk: TensorDesc, rope: Rope3D, S, z, eps: float, Ob, workspace,
                                 workspace_bytes: int | None = None, stream=None) -> None:
    _block_rope3d("sv_block_linattn_step_rope3d", Qb, Kb, Vb, blk, rope, S, z, eps, Ob, workspace, workspace_bytes,
                  stream)


def sv_block_linattn_lookahead_rope3d(Qb, Kb, Vb, blk: TensorDesc, rope: Rope3D, S, z, eps: float, Ob, workspace,
                                      workspace_bytes: int | None = None, stream=None) -> None:
    _block_rope3d("sv_block_linattn_lookahead_rope3d", Qb, Kb, Vb, blk, rope, S, z, eps, Ob, workspace,
                  workspace_bytes, stream)


def sv_tconv_block_step(x, W, cache_in, y, cache_out, B: int, T: int, HW: int, D: int, dtype: int = SV_BF16,
                        stream=None) -> None:
    """One block through the Mix-FFN's temporal convolution with shortcut (include/sv_tconv.h):
    x, y [B][T][HW][D], W [3][D][D], cache_in / cache_out [B][HW][D] or None."""
    rc = load_library().sv_tconv_block_step(_ptr(x), _ptr(W), _ptr(cache_in), _ptr(y), _ptr(cache_out), B, T, HW, D,
                                            dtype, _stream(stream))
    if rc != 0:
        raise SvError(rc, "sv_tconv_block_step")


def sv_measure_apply_variant(variant: int, Q, q: TensorDesc, tok_begin: int, tok_end: int, S, z, eps: float, O,
                             stream=None) -> None:
    """sv_linattn_apply (bf16, d = 64) in one of four kernel forms (include/sv_measure.h)."""
    d = q._c() if q is not None else None
    _check(load_library().sv_measure_apply_variant(int(variant), _ptr(Q), ctypes.byref(d) if d else None, tok_begin,
                                                   tok_end, _ptr(S), _ptr(z), float(eps), _ptr(O), _stream(stream)),
           "sv_measure_apply_variant")


def sv_measure_assume_dies(dies: int) -> None:
    """Test hook (include/sv_measure.h): place heads as if the device had `dies` dies; 8 or 0 restores."""
    load_library().sv_measure_assume_dies(int(dies))


def sv_measure_tconv_variant(variant: int, x, W, cache_in, y, B: int, T: int, HW: int, D: int, stream=None) -> None:
    """Measurement variants of the temporal-convolution kernel (include/sv_measure.h); 0 is the library's kernel."""
    _check(load_library().sv_measure_tconv_variant(int(variant), _ptr(x), _ptr(W), _ptr(cache_in), _ptr(y), int(B), int(T),
                                                   int(HW), int(D), _stream(stream)), "sv_measure_tconv_variant")


def sv_mfma_stream(wgs: int, steps: int, sink, stream=None) -> None:
    """Matrix-core yardstick (include/sv_measure.h): wgs workgroups x 4 waves x 32*steps bf16 MFMAs, no memory traffic."""
    _check(load_library().sv_mfma_stream(int(wgs), int(steps), _ptr(sink), _stream(stream)), "sv_mfma_stream")


def sv_stream_read(src, nbytes: int, sink, wgs: int, stream=None) -> None:
    """Streaming yardstick (include/sv_measure.h): reads src[0, nbytes) once."""
    _check(load_library().sv_stream_read(_ptr(src), int(nbytes), _ptr(sink), int(wgs), _stream(stream)),
           "sv_stream_read")


def sv_stream_copy(src, dst, nbytes: int, wgs: int, stream=None) -> None:
    """Streaming yardstick (include/sv_measure.h): dst[0, nbytes) = src[0, nbytes)."""
    _check(load_library().sv_stream_copy(_ptr(src), _ptr(dst), int(nbytes), int(wgs), _stream(stream)),
           "sv_stream_copy")
