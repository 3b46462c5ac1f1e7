"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments with a status before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def m():
    import paper_2603_20586_amd as mod

    if not os.path.exists(mod.lib_path()):
        from paper_2603_20586_amd.build import build_library

        build_library(verbose=False)
    mod.lib()
    return mod


def _declared(header):
    hdr = open(os.path.join(ROOT, "include", header)).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    return set(re.findall(r"\b(mka_[a-z_0-9]+)\s*\(", hdr))


def test_every_declared_symbol_is_exported(m):
    names = _declared("mka.h")
    assert {"mka_route", "mka_fused_attn_fwd", "mka_fused_attn_decode", "mka_fused_attn_bwd",
            "mka_workspace_bytes", "mka_status_string", "mka_version"} <= names
    L = m.lib()
    for n in names:
        assert hasattr(L, n), n
    assert L.mka_version() >= 100
    # the measurement micro-benchmarks live in a library of their own, not in the product's
    from paper_2603_20586_amd import measure

    mnames = _declared("mka_measure.h")
    assert mnames == {"mka_measure_mfma_loop", "mka_measure_mfma_loop_data",
                      "mka_measure_stream_read"}
    for n in mnames:
        assert hasattr(measure.lib(), n), n
        assert not hasattr(L, n), n
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["mka.h", "mka_measure.h"]


def test_status_strings(m):
    for code, word in [(0, "OK"), (1, "NULL"), (2, "SHAPE"), (3, "DTYPE"), (4, "ALIGN"),
                       (5, "WORKSPACE"), (6, "UNSUPPORTED"), (7, "LAUNCH")]:
        assert word in m.status_string(code)


def _shape(m, **kw):
    from paper_2603_20586_amd.binding import MkaShape

    s = MkaShape()
    s.B, s.H, s.Tq, s.S, s.d = 1, 2, 16, 16, 64
    s.len[0] = s.len[1] = s.len[2] = 16
    s.dtype, s.causal, s.scale = 1, 1, 0.125
    for k, v in kw.items():
        if k == "len":
            for i in range(3):
                s.len[i] = v[i]
        else:
            setattr(s, k, v)
    return s


FAKE = 0x10000  # 16-byte aligned, never dereferenced: validation fails first


def _fwd(m, s, Q=FAKE, K=(FAKE, FAKE, FAKE), V=(FAKE, FAKE, FAKE), W=FAKE, G=FAKE, O=FAKE):
    from paper_2603_20586_amd.binding import _P3

    k3, v3 = _P3(*K), _P3(*V)
    return m.lib().mka_fused_attn_fwd(Q, ctypes.byref(k3), ctypes.byref(v3), W, None, G, O, None,
                                      None, ctypes.byref(s), None, 0, None)


def test_fwd_rejects_bad_arguments_before_launch(m):
    assert _fwd(m, _shape(m, dtype=7)) == 3
    assert _fwd(m, _shape(m, Tq=32, S=16)) == 2          # S < Tq
    assert _fwd(m, _shape(m, B=-1)) == 2
    assert _fwd(m, _shape(m, len=(17, 0, 0))) == 2        # len > S
    assert _fwd(m, _shape(m, d=96)) == 6
    assert _fwd(m, _shape(m, scale=-1.0)) == 6
    assert _fwd(m, _shape(m, scale=float("nan"))) == 6
    assert _fwd(m, _shape(m), Q=None) == 1
    assert _fwd(m, _shape(m), G=None) == 1
    assert _fwd(m, _shape(m), Q=FAKE + 2) == 4
    assert _fwd(m, _shape(m), K=(FAKE + 8, FAKE, FAKE)) == 4
    # a valid problem with no rows is a no-op
    assert _fwd(m, _shape(m, B=0)) == 0
    assert _fwd(m, _shape(m, Tq=0, S=0, len=(0, 0, 0))) == 0


def test_route_and_bwd_reject_bad_arguments(m):
    from paper_2603_20586_amd.binding import _P3

    L = m.lib()
    s = _shape(m)
    assert L.mka_route(None, FAKE, None, FAKE, None, ctypes.byref(s), None) == 1
    assert L.mka_route(FAKE, None, None, FAKE, None, ctypes.byref(s), None) == 1
    assert L.mka_route(FAKE, FAKE, None, FAKE, None, None, None) == 1
    assert L.mka_route(FAKE, FAKE, None, FAKE + 4, None, ctypes.byref(s), None) == 4
    # routing variants: same checks, and the mode must be one of the four
    assert L.mka_route_variant(FAKE, FAKE, None, 4, FAKE, None, ctypes.byref(s), None) == 6
    assert L.mka_route_variant(FAKE, FAKE, None, -1, FAKE, None, ctypes.byref(s), None) == 6
    assert L.mka_route_variant(FAKE, None, None, 1, FAKE, None, ctypes.byref(s), None) == 1
    p3 = _P3(FAKE, FAKE, FAKE)
    args = lambda shp, ws, wsb: L.mka_fused_attn_bwd(  # noqa: E731
        FAKE, FAKE, ctypes.byref(p3), ctypes.byref(p3), FAKE, FAKE, FAKE, FAKE, FAKE,
        ctypes.byref(p3), ctypes.byref(p3), FAKE, FAKE, ctypes.byref(shp), ws, wsb, None)
    assert args(_shape(m, dtype=0), FAKE, 1 << 30) == 6   # f32 backward not provided
    assert args(_shape(m), None, 0) == 5                  # workspace required
    assert args(_shape(m), FAKE, 16) == 5
    assert m.mka_workspace_bytes(3, _shape(m)) > 0
    # backward sizes: 8 = the least accepted (recomputation), 7 = stored score gradients (0 where
    # that route is not provided), 3 = the recommended one: the stored route's where provided
    c5 = _shape(m, B=8, H=16, Tq=4096, S=4096, d=128)
    rec, sto = m.mka_workspace_bytes(8, c5), m.mka_workspace_bytes(7, c5)
    assert 0 < rec < sto and m.mka_workspace_bytes(3, c5) == sto
    assert sto > 8 * 16 * (4096 // 128) * (4096 // 32) * 8192   # holds 8 KiB per tile pair
    huge = _shape(m, B=64, H=64, Tq=16384, S=16384, d=128)   # dS would exceed 32 GiB
    assert m.mka_workspace_bytes(7, huge) == 0
    assert m.mka_workspace_bytes(3, huge) == m.mka_workspace_bytes(8, huge) > 0
    # forward: no workspace recommended for a short block; the materialised route's size is
    # two [B,H,S,d] bf16 tensors; long blocks get it recommended; f32 has no such route
    assert m.mka_workspace_bytes(1, _shape(m)) == 0
    assert m.mka_workspace_bytes(4, _shape(m)) == 2 * 1 * 2 * 16 * 64 * 2
    long_ = _shape(m, Tq=4096, S=4096, d=128)
    assert m.mka_workspace_bytes(1, long_) == m.mka_workspace_bytes(4, long_) == 2 * 2 * 4096 * 128 * 2
    assert m.mka_workspace_bytes(4, _shape(m, dtype=0)) == 0


def test_decode_rejects_bad_arguments(m):
    from paper_2603_20586_amd.binding import MkaDecodeShape, _P3

    L = m.lib()

    def call(len3=(8, 8, 8), cap=(16, 8, 8), capG=16, knew=(FAKE, None, None), ws=FAKE << 4,
             wsb=1 << 30, **kw):
        s = MkaDecodeShape()
        s.B, s.H, s.d, s.capG, s.dtype, s.n_splits, s.scale = 1, 2, 64, capG, 1, 0, 0.125
        for i in range(3):
            s.cap[i] = cap[i]
        for k, v in kw.items():
            setattr(s, k, v)
        ln = (ctypes.c_int32 * 3)(*len3)
        kn = _P3(*knew)
        kc = _P3(FAKE, FAKE, FAKE)
        rc = L.mka_fused_attn_decode(FAKE, ctypes.byref(kn), ctypes.byref(kn), ctypes.byref(kc),
                                     ctypes.byref(kc), FAKE, ctypes.byref(ln), FAKE, None, FAKE,
                                     None, None, ctypes.byref(s), ws, wsb, None)
        return rc, list(ln)

    assert call(knew=(None, None, None))[0] == 2          # nothing appended
    assert call(len3=(8, 7, 8), knew=(FAKE, FAKE, None))[0] == 2   # level 2 lags: cannot rejoin
    assert call(cap=(8, 8, 8))[0] == 2                    # level 1 cache full
    assert call(capG=8)[0] == 2                           # gate cache full
    assert call(ws=None, wsb=0)[0] == 5
    assert call(d=100)[0] == 6
    assert call(routing=4)[0] == 6 and call(routing=-1)[0] == 6   # unknown routing variant
    rc, ln = call(dtype=9)
    assert rc == 3 and ln == [8, 8, 8]                    # lengths untouched on error


def test_static_decode_validates_like_decode_and_enforces_its_size_limit(m):
    """The entry point that allocates nothing: same argument checks as mka_fused_attn_decode, in
    the same order, plus the limit of its fixed scratch buffer - all before any device is
    touched."""
    from paper_2603_20586_amd.binding import MkaDecodeShape, _P3

    L = m.lib()

    def call(B=1, H=2, d=64, n_splits=0, len3=(8, 8, 8), cap=(16, 8, 8), q=FAKE, dtype=1):
        s = MkaDecodeShape()
        s.B, s.H, s.d, s.capG, s.dtype, s.n_splits, s.scale = B, H, d, 16, dtype, n_splits, 0.125
        for i in range(3):
            s.cap[i] = cap[i]
        ln = (ctypes.c_int32 * 3)(*len3)
        kn, kc = _P3(FAKE, None, None), _P3(FAKE, FAKE, FAKE)
        return L.mka_fused_attn_decode_static(q, ctypes.byref(kn), ctypes.byref(kn), ctypes.byref(kc),
                                              ctypes.byref(kc), FAKE, ctypes.byref(ln), FAKE, None,
                                              FAKE, None, None, ctypes.byref(s), None)

    assert L.mka_fused_attn_decode_static(FAKE, None, None, None, None, FAKE, None, FAKE, None, FAKE,
                                          None, None, None, None) == 1
    assert call(dtype=9) == 3
    assert call(d=100) == 6
    assert call(q=None) == 1
    assert call(q=FAKE + 4) == 4
    assert call(len3=(8, 9, 8)) == 2                       # a lagging level cannot be appended to
    assert call(B=0) == 0                                  # no heads: nothing to do
    # 8 MiB of partials: 4096 heads x 66 floats x 4 B = 1.03 MiB per split
    assert call(B=64, H=64, n_splits=8) == 5               # 8.25 MiB: refused
    assert call(B=255, H=257) == 5                         # 65 535 heads do not fit even unsplit


def test_measure_helpers_reject_bad_arguments_on_the_host(m):
    import ctypes
    from paper_2603_20586_amd import measure

    L = measure.lib()
    assert L.mka_measure_mfma_loop(None, 4, 10, None, None) == 2      # no output buffer
    assert L.mka_measure_mfma_loop(ctypes.c_void_p(256), 0, 10, None, None) == 2
    assert L.mka_measure_mfma_loop(ctypes.c_void_p(256), 4, 0, None, None) == 2
    assert L.mka_measure_mfma_loop_data(ctypes.c_void_p(256), None, 4, 10, None, None) == 2  # no operands
    assert L.mka_measure_mfma_loop_data(ctypes.c_void_p(256), ctypes.c_void_p(4100), 4, 10, None, None) == 4
    assert L.mka_measure_mfma_loop_data(ctypes.c_void_p(256), ctypes.c_void_p(4096), 4, 0, None, None) == 2
    assert L.mka_measure_stream_read(None, 1 << 20, None, None) == 2
    assert L.mka_measure_stream_read(ctypes.c_void_p(4096), 64, None, None) == 2   # too small
    assert L.mka_measure_stream_read(ctypes.c_void_p(4100), 1 << 20, None, None) == 4  # misaligned


def test_widened_entry_points_reject_bad_arguments(m):
    """Host-side validation of the entry points beyond the four core ones (no GPU work: every
    call returns before a launch)."""
    from paper_2603_20586_amd.binding import MkaPagedShape, _P3

    L = m.lib()
    p3 = _P3(FAKE, FAKE, FAKE)
    s = _shape(m, d=128)
    # full MKA: gates and workspace are required, f32 has no kernel, causal needs len >= Tq
    full = lambda shp, g, ws, wsb: L.mka_full_attn_fwd(  # noqa: E731
        FAKE, ctypes.byref(p3), ctypes.byref(p3), g, FAKE, ctypes.byref(shp), ws, wsb, None)
    assert full(s, None, FAKE, 1 << 30) == 1
    assert full(s, FAKE, None, 0) == 5
    assert full(s, FAKE, FAKE, 16) == 5
    assert full(_shape(m, d=128, dtype=0), FAKE, FAKE, 1 << 30) == 6
    assert full(_shape(m, d=128, len=(8, 16, 16)), FAKE, FAKE, 1 << 30) == 2
    assert m.mka_workspace_bytes(5, s) == 3 * 1 * 2 * 16 * 128 * 2
    # prefix mean
    pm = lambda shp, ws, wsb: L.mka_prefix_mean(FAKE, FAKE, ctypes.byref(shp), ws, wsb, None)  # noqa: E731
    assert pm(s, None, 0) == 5
    assert pm(_shape(m, d=96), FAKE, 1 << 20) == 6
    assert L.mka_prefix_mean(None, FAKE, ctypes.byref(s), FAKE, 1 << 20, None) == 1
    assert m.mka_workspace_bytes(6, s) > 0
    # paged decode: page size a power of two >= 16, pool and table sizes positive
    ps = MkaPagedShape()
    ps.B, ps.H, ps.d, ps.page_size, ps.n_pages, ps.max_pages, ps.n_splits, ps.scale = 2, 2, 128, 64, 8, 4, 0, 0.1
    paged = lambda shp, ws, wsb: L.mka_paged_fused_decode(  # noqa: E731
        FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, ctypes.byref(shp), ws, wsb, None)
    assert paged(ps, None, 0) == 5
    ps.page_size = 48
    assert paged(ps, FAKE, 1 << 30) == 2
    ps.page_size = 8
    assert paged(ps, FAKE, 1 << 30) == 2
    ps.page_size, ps.n_pages = 64, 0
    assert paged(ps, FAKE, 1 << 30) == 2
    ps.n_pages, ps.d = 8, 96
    assert paged(ps, FAKE, 1 << 30) == 6
    ps.d = 128
    assert L.mka_paged_fused_decode(FAKE, FAKE, FAKE, None, FAKE, FAKE, None, ctypes.byref(ps),
                                    FAKE, 1 << 30, None) == 1


def test_profile_summary_kernel_names():
    """Host logic of the profile summaries: mangled kernel names keep every template argument
    (two instantiations of one kernel must not be merged into one line)."""
    from paper_2603_20586_amd.measure.prof_summary import short

    a = short("_ZN3mka12_GLOBAL__N_119decode_split_kernelIDF16bLi128ELi4ELb1EEEvPKT_S4_")
    b = short("_ZN3mka12_GLOBAL__N_119decode_split_kernelIDF16bLi128ELi4ELb0EEEvPKT_S4_")
    assert a == "mka::decode_split_kernel<bf16,128,4,true>"
    assert b == "mka::decode_split_kernel<bf16,128,4,false>"
    assert short("_ZN3mka12_GLOBAL__N_119decode_split_kernelIfLi64ELi4ELb0EEEvPKT_") == \
        "mka::decode_split_kernel<f32,64,4,false>"
    assert short("_ZN3mka12_GLOBAL__N_117bwd_reduce_kernelEPKfiiPfS3_") == "mka::bwd_reduce_kernel"
    assert short("_ZN3mka12route_kernelIDF16bLi128EEEvPKT_PKfS5_PfPiliii") == "mka::route_kernel<bf16,128>"
    assert short("void at::native::foo<int>(int)") == "at::native::foo<int>"
