"""Host-side checks that need no GPU: the shared library loads, exports every
symbol the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

import paper_2509_24695_amd as sv
from paper_2509_24695_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include")))
                   if h.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sv_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    if not os.path.exists(sv.library_path()):
        from paper_2509_24695_amd import build
        build.build()
    lib = ctypes.CDLL(sv.library_path())
    declared = _declared_symbols()
    assert set(declared) == set(sv.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert sv.sv_version() >= 100


def test_status_strings():
    assert sv.sv_status_string(0) == "ok"
    assert len({sv.sv_status_string(i) for i in range(8)}) == 8


def test_workspace_bytes():
    assert sv.sv_linattn_workspace_bytes(1, 32, 4680, 64) == sv.sv_linattn_workspace_bytes(1, 32, 864000, 64)
    assert sv.sv_linattn_workspace_bytes(1, 32, 100, 64) >= 32 * (64 * 64 + 64) * 4
    assert sv.sv_linattn_workspace_bytes(1, 32, 100, 48) == 0
    assert sv.sv_linattn_workspace_bytes(0, 32, 100, 64) == 0


FAKE = 0x10000          # aligned, never dereferenced: every call below fails before a launch


def _desc(**kw):
    base = dict(B=1, H=2, N=128, d=64, stride_b=2 * 128 * 64, stride_h=128 * 64, stride_n=64, dtype=sv.SV_BF16)
    base.update(kw)
    return sv.TensorDesc(**base)


@pytest.mark.parametrize("kwargs,status", [
    (dict(d=48), 3), (dict(dtype=5), 3), (dict(N=0), 2), (dict(B=0), 2), (dict(stride_n=32), 2),
    (dict(stride_n=68), 4), (dict(stride_h=128 * 64 + 4), 4),
    # rows of different heads or batches on top of each other
    (dict(stride_h=127 * 64), 2), (dict(stride_h=64), 2), (dict(B=2, stride_b=128 * 64), 2),
    (dict(stride_h=64, stride_n=64 * 2 - 8), 2),           # [N][H][d] with rows shorter than the heads they hold
])
def test_bad_descriptors(kwargs, status):
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_state(FAKE, FAKE, _desc(**kwargs), 0, 1, 0, FAKE, FAKE, FAKE, workspace_bytes=1 << 30)
    assert e.value.status == status
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_apply(FAKE, _desc(**kwargs), 0, 1, FAKE, FAKE, 1e-6, FAKE)
    assert e.value.status == status
    for step in (sv.sv_block_linattn_step, sv.sv_block_linattn_lookahead):
        with pytest.raises(sv.SvError) as e:
            step(FAKE, FAKE, FAKE, _desc(**kwargs), FAKE, FAKE, 1e-6, FAKE, FAKE, workspace_bytes=1 << 30)
        assert e.value.status == status


def test_interleaved_layouts_are_accepted_up_to_the_launch():
    """[B][N][H][d] (heads interleaved inside a token row) and token slices of a longer tensor pass the
    descriptor checks: the calls get as far as the workspace check."""
    for kw in (dict(stride_h=64, stride_n=2 * 64, stride_b=128 * 2 * 64),
               dict(stride_h=1000 * 64), dict(H=1, stride_h=0), dict(B=1, stride_b=0)):
        with pytest.raises(sv.SvError) as e:
            sv.sv_linattn_state(FAKE, FAKE, _desc(**kw), 0, 1, 0, FAKE, FAKE, FAKE, workspace_bytes=16)
        assert e.value.status == 6, kw


def test_workspace_status_word():
    """The word that records a timed-out wait lies inside the workspace, behind the partials, the look-ahead
    state and the flags, 8-byte aligned; the query checks its arguments like the other workspace calls."""
    for (B, H, d) in ((1, 32, 64), (2, 32, 64), (1, 20, 112), (1, 7, 128), (1, 2, 32)):
        off = sv.sv_linattn_workspace_status_offset(B, H, d)
        total = sv.sv_linattn_workspace_bytes(B, H, 1, d)
        assert off % 8 == 0 and 0 < off <= total - 8
        assert off >= B * H * (32 + 1) * (d * d + d) * 4        # partials of 32 chunks + look-ahead state
        assert total - off == (4 + B * H) * 8                    # [error, magic, pad, pad, tickets[B*H]]
    assert sv.sv_linattn_workspace_status_offset(1, 2, 48) == 0
    assert sv.sv_linattn_workspace_status_offset(0, 2, 64) == 0
    big = 1 << 30
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_workspace_status(None, 1, 2, 64, workspace_bytes=big)
    assert e.value.status == 1
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_workspace_status(FAKE, 1, 2, 48, workspace_bytes=big)
    assert e.value.status == 3
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_workspace_status(FAKE, 1, 2, 64, workspace_bytes=100)
    assert e.value.status == 6
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_workspace_status(FAKE + 8, 1, 2, 64, workspace_bytes=big)
    assert e.value.status == 4
    lib = sv.load_library()
    assert lib.sv_linattn_workspace_status(ctypes.c_void_p(FAKE), big, 1, 2, 64, None, None) == 1   # no result pointer


def test_null_range_alignment_workspace_eps():
    d = _desc()
    big = 1 << 30
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_state(None, FAKE, d, 0, 1, 0, FAKE, FAKE, FAKE, workspace_bytes=big)
    assert e.value.status == 1
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_state(FAKE, FAKE, None, 0, 1, 0, FAKE, FAKE, FAKE, workspace_bytes=big)
    assert e.value.status == 1
    for t0, t1 in [(-1, 4), (5, 4), (0, 129)]:
        with pytest.raises(sv.SvError) as e:
            sv.sv_linattn_state(FAKE, FAKE, d, t0, t1, 0, FAKE, FAKE, FAKE, workspace_bytes=big)
        assert e.value.status == 5
        with pytest.raises(sv.SvError) as e:
            sv.sv_linattn_apply(FAKE, d, t0, t1, FAKE, FAKE, 1e-6, FAKE)
        assert e.value.status == 5
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_state(FAKE + 8, FAKE, d, 0, 1, 0, FAKE, FAKE, FAKE, workspace_bytes=big)
    assert e.value.status == 4
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_state(FAKE, FAKE, d, 0, 1, 0, FAKE, FAKE, FAKE, workspace_bytes=1024)
    assert e.value.status == 6
    for eps in (-1.0, float("nan"), float("inf")):
        with pytest.raises(sv.SvError) as e:
            sv.sv_linattn_apply(FAKE, d, 0, 1, FAKE, FAKE, eps, FAKE)
        assert e.value.status == 5
        with pytest.raises(sv.SvError) as e:
            sv.sv_block_linattn_step(FAKE, FAKE, FAKE, d, FAKE, FAKE, eps, FAKE, FAKE, workspace_bytes=big)
        assert e.value.status == 5


def test_product_path_does_not_import_the_oracle():
    """The library and its binding must never reach into oracle/ (no CPU fallback)."""
    pkg = os.path.join(ROOT, "paper_2509_24695_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f
    assert binding.load_library() is not None


def test_rope_entry_points_check_arguments():
    d = _desc()
    big = 1 << 30
    with pytest.raises(sv.SvError) as e:      # table is required
        sv.sv_linattn_state_rope(FAKE, FAKE, d, None, 0, 1, 0, FAKE, FAKE, FAKE, workspace_bytes=big)
    assert e.value.status == 1
    with pytest.raises(sv.SvError) as e:      # and must be 16-byte aligned
        sv.sv_linattn_apply_rope(FAKE, d, FAKE + 4, 0, 1, FAKE, FAKE, 1e-6, FAKE)
    assert e.value.status == 4
    with pytest.raises(sv.SvError) as e:
        sv.sv_block_linattn_step_rope(FAKE, FAKE, FAKE, _desc(d=48), FAKE, FAKE, FAKE, 1e-6, FAKE, FAKE,
                                      workspace_bytes=big)
    assert e.value.status == 3
    with pytest.raises(sv.SvError) as e:
        sv.sv_block_linattn_lookahead_rope(FAKE, FAKE, FAKE, d, FAKE, FAKE, FAKE, -1.0, FAKE, FAKE,
                                           workspace_bytes=big)
    assert e.value.status == 5


def test_workspace_init_checks_arguments():
    big = 1 << 30
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_workspace_init(None, 1, 2, 64, workspace_bytes=big)
    assert e.value.status == 1
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_workspace_init(FAKE, 1, 2, 48, workspace_bytes=big)
    assert e.value.status == 3
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_workspace_init(FAKE, 1, 2, 64, workspace_bytes=sv.sv_linattn_workspace_bytes(1, 2, 10, 64) - 1)
    assert e.value.status == 6
    with pytest.raises(sv.SvError) as e:
        sv.sv_linattn_workspace_init(FAKE + 8, 1, 2, 64, workspace_bytes=big)
    assert e.value.status == 4


def test_rope3d_entry_points_check_arguments():
    d = _desc()                                  # N tokens, d features as in the other tests
    big = 1 << 30
    N, dim = d.N, d.d

    def rope(frames=1, rows=1, cols=N, n_t=0, n_h=0, n_w=dim // 2, cs_t=None, cs_h=None, cs_w=FAKE):
        return sv.Rope3D(frames, rows, cols, n_t, n_h, n_w, cs_t, cs_h, cs_w)

    with pytest.raises(sv.SvError) as e:          # descriptor of the tables is required
        sv.sv_linattn_state_rope3d(FAKE, FAKE, d, None, 0, 1, 0, FAKE, FAKE, FAKE, workspace_bytes=big)
    assert e.value.status == 1
    with pytest.raises(sv.SvError) as e:          # frames*rows*cols must be N
        sv.sv_linattn_apply_rope3d(FAKE, d, rope(cols=N + 1), 0, 1, FAKE, FAKE, 1e-6, FAKE)
    assert e.value.status == 2
    with pytest.raises(sv.SvError) as e:          # pairs must add up to d/2
        sv.sv_linattn_apply_rope3d(FAKE, d, rope(n_w=dim // 2 - 1), 0, 1, FAKE, FAKE, 1e-6, FAKE)
    assert e.value.status == 2
    with pytest.raises(sv.SvError) as e:          # an axis with pairs needs its table
        sv.sv_block_linattn_step_rope3d(FAKE, FAKE, FAKE, d, rope(cs_w=None), FAKE, FAKE, 1e-6, FAKE, FAKE,
                                        workspace_bytes=big)
    assert e.value.status == 1
    with pytest.raises(sv.SvError) as e:          # 8-byte alignment of the tables
        sv.sv_block_linattn_lookahead_rope3d(FAKE, FAKE, FAKE, d, rope(cs_w=FAKE + 4), FAKE, FAKE, 1e-6, FAKE, FAKE,
                                             workspace_bytes=big)
    assert e.value.status == 4


def test_tconv_checks_arguments():
    def call(x=FAKE, W=FAKE + (1 << 28), cache_in=None, y=FAKE + (1 << 29), cache_out=None, B=1, T=3, HW=100, D=64,
             dtype=sv.SV_BF16):
        with pytest.raises(sv.SvError) as e:
            sv.sv_tconv_block_step(x, W, cache_in, y, cache_out, B, T, HW, D, dtype)
        return e.value.status

    assert call(x=None) == 1 and call(W=None) == 1 and call(y=None) == 1
    assert call(B=0) == 2 and call(T=0) == 2 and call(HW=-1) == 2 and call(D=0) == 2
    assert call(dtype=sv.SV_F32) == 3
    assert call(D=60) == 3                                  # not a multiple of 8
    assert call(B=1 << 12, T=1 << 10, HW=1 << 10) == 2      # 2^32 token rows
    assert call(D=1 << 15) == 2                             # 3 * D * D does not fit
    assert call(x=FAKE + 8) == 4 and call(cache_in=FAKE + (1 << 27) + 4) == 4 and call(cache_out=FAKE + 2) == 4
    assert call(y=FAKE) == 2                                # y on top of x
    assert call(y=FAKE + 64) == 2                           # y inside x
    assert call(cache_in=FAKE + (1 << 29) + 1024) == 2      # cache_in inside y
    assert call(cache_out=FAKE + (1 << 29) + 2048) == 2     # cache_out inside y
    assert call(cache_out=FAKE + 4096) == 2                 # cache_out inside x
    assert call(cache_out=FAKE + (1 << 28)) == 2            # cache_out on top of W


def test_tconv_variant_checks_arguments():
    def call(variant=1, x=FAKE, W=FAKE + (1 << 28), cache_in=None, y=FAKE + (1 << 29), B=1, T=3, HW=100, D=64):
        with pytest.raises(sv.SvError) as e:
            sv.sv_measure_tconv_variant(variant, x, W, cache_in, y, B, T, HW, D)
        return e.value.status

    assert call(variant=-1) == 5 and call(variant=4) == 5      # SV_ERR_RANGE
    assert call(x=None) == 1 and call(y=None) == 1 and call(T=0) == 2 and call(y=FAKE + 64) == 2
    assert call(variant=2, D=40) == 3                       # variants 1-3 need whole K-steps


def test_stream_yardsticks_check_arguments():
    def status(fn, *args):
        with pytest.raises(sv.SvError) as e:
            fn(*args)
        return e.value.status

    A, B = FAKE, FAKE + (1 << 28)
    assert status(sv.sv_stream_read, None, 1024, B, 64) == 1 and status(sv.sv_stream_read, A, 1024, None, 64) == 1
    assert status(sv.sv_stream_copy, None, B, 1024, 64) == 1 and status(sv.sv_stream_copy, A, None, 1024, 64) == 1
    assert status(sv.sv_stream_read, A + 8, 1024, B, 64) == 4 and status(sv.sv_stream_read, A, 1000, B, 64) == 4
    assert status(sv.sv_stream_copy, A, B + 4, 1024, 64) == 4 and status(sv.sv_stream_copy, A, B, 1032, 64) == 4
    assert status(sv.sv_stream_read, A, 1024, B, 0) == 2 and status(sv.sv_stream_copy, A, B, 1024, (1 << 20) + 1) == 2
    assert status(sv.sv_stream_copy, A, A + 512, 1024, 64) == 2          # overlapping buffers
    sv.sv_stream_read(A, 0, B, 64)                                        # nothing to do: no launch, no error
    sv.sv_stream_copy(A, B, 0, 64)
    assert status(sv.sv_mfma_stream, 8, 10, None) == 1 and status(sv.sv_mfma_stream, 8, 10, A + 2) == 4
    assert status(sv.sv_mfma_stream, 0, 10, A) == 2 and status(sv.sv_mfma_stream, 8, -1, A) == 2
    assert status(sv.sv_mfma_stream, (1 << 20) + 1, 10, A) == 2 and status(sv.sv_mfma_stream, 8, (1 << 20) + 1, A) == 2
    sv.sv_mfma_stream(8, 0, A)


def test_apply_variant_checks_arguments():
    d = _desc()
    def status(variant=0, Q=FAKE, dsc=d, t0=0, t1=1, S=FAKE, eps=1e-6):
        with pytest.raises(sv.SvError) as e:
            sv.sv_measure_apply_variant(variant, Q, dsc, t0, t1, S, FAKE, eps, FAKE)
        return e.value.status
    assert status(Q=None) == 1 and status(S=None) == 1 and status(dsc=None) == 1
    assert status(variant=4) == 5 and status(variant=-1) == 5 and status(t1=129) == 5 and status(eps=-1.0) == 5
    assert status(dsc=_desc(d=48)) == 3 and status(dsc=_desc(d=32)) == 3 and status(dsc=_desc(dtype=sv.SV_F32)) == 3
    assert status(dsc=_desc(d=128, stride_n=128, stride_h=128 * 128, stride_b=2 * 128 * 128)) == 3
    assert status(Q=FAKE + 8) == 4


def test_build_rejects_kernels_that_use_scratch_memory():
    """build() reads hipcc's per-kernel resource remarks and refuses a library in which a kernel keeps data in
    scratch memory (such a kernel passes every parity test and runs many times slower)."""
    from paper_2509_24695_amd import build as b

    def remarks(name, scratch, spill):
        tag = "[-Rpass-analysis=kernel-resource-usage]"
        rows = [f"Function Name: {name}", "    VGPRs: 512", "    AGPRs: 256", f"    ScratchSize [bytes/lane]: {scratch}",
                "    Dynamic Stack: False", "    Occupancy [waves/SIMD]: 1", "    SGPRs Spill: 0", f"    VGPRs Spill: {spill}",
                "    LDS Size [bytes/block]: 0"]
        return "\n".join(f"x.hip:1:1: remark: {r} {tag}\n    1 | {{\n      | ^" for r in rows)

    good = b.kernel_resources(remarks("_ZN2sv1aEv", 0, 0) + "\n" + remarks("_ZN2sv1bEv", 0, 0))
    assert set(good) == {"_ZN2sv1aEv", "_ZN2sv1bEv"} and good["_ZN2sv1aEv"]["ScratchSize"] == "0"
    assert good["_ZN2sv1aEv"]["VGPRs"] == "512" and good["_ZN2sv1bEv"]["Occupancy"] == "1"
    b.check_resources(good)
    for scratch, spill in ((448, 0), (0, 3)):
        bad = b.kernel_resources(remarks("_ZN2sv1aEv", 0, 0) + "\n" + remarks("_ZN2sv1cEv", scratch, spill))
        with pytest.raises(RuntimeError, match="_ZN2sv1cEv"):
            b.check_resources(bad)
    # the library built in-tree went through the same check; its record says so
    if os.path.exists(b.RESOURCES):
        lines = open(b.RESOURCES).read().splitlines()
        assert len(lines) >= 40 and all(" scratch=0 " in l for l in lines)
