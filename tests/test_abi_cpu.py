"""Host-side checks of liblasad that need no GPU: the library loads, exports every symbol
the header declares, and rejects invalid arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2507_01652_amd", "liblasad.so")
HEADER = os.path.join(ROOT, "include", "lasad.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} not built: run `python -m paper_2507_01652_amd.build`")
    lib = ctypes.CDLL(LIB)
    lib.lasad_last_error.restype = ctypes.c_char_p
    lib.lasad_version.restype = ctypes.c_char_p
    lib.lasad_forward_workspace_bytes.restype = ctypes.c_size_t
    return lib


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lasad_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_exported(lib):
    names = declared_functions()
    assert {"lasad_decay_factors", "lasad_forward_chunked", "lasad_decode_step"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in lasad.h but not exported"


def test_binding_names_match_header():
    import paper_2507_01652_amd.binding as b
    assert sorted(b.EXPORTS) == declared_functions()
    for n in ("lasad_decay_factors", "lasad_forward_chunked", "lasad_decode_step",
              "lasad_forward_workspace_bytes"):
        assert callable(getattr(b, n))


def test_version_and_workspace(lib):
    assert b"gfx950" in lib.lasad_version()
    # high-res stress: 96 sequences of 64 chunks -> 5 segments, 4 partial 64x64 fp32 states each
    assert lib.lasad_forward_workspace_bytes(4, 24, 4096, 64, 1) == 96 * 4 * 64 * 64 * 4
    assert lib.lasad_forward_workspace_bytes(8, 12, 256, 64, 1) == 0       # 4 chunks: not worth two launches
    assert lib.lasad_forward_workspace_bytes(32, 16, 576, 64, 1) == 0      # 512 sequences fill the chip
    assert lib.lasad_forward_workspace_bytes(4, 24, 4096, 64, 0) == 0      # fp32 kernel needs none
    assert lib.lasad_forward_workspace_bytes(4, 24, 4096, 32, 1) == 0


class Layout(ctypes.Structure):
    _fields_ = [("b", ctypes.c_int64), ("n", ctypes.c_int64), ("h", ctypes.c_int64)]


def _forward(lib, **kw):
    a = dict(q=0x1000, k=0x2000, v=0x3000, o=0x4000, lq=Layout(64 * 4 * 2, 2 * 64, 64),
             lo=Layout(64 * 4 * 2, 2 * 64, 64), io=1, out=1, B=1, Hh=2, d=64, gh=2, gw=2, sp=0, n=4,
             gamma=0x5000, mode=0, qs=1.0, s_in=None, s_out=None)
    a.update(kw)
    vp = ctypes.c_void_p
    return lib.lasad_forward_chunked(vp(a["q"]), vp(a["k"]), vp(a["v"]), vp(a["o"]),
                                     ctypes.byref(a["lq"]), ctypes.byref(a["lo"]), a["io"], a["out"],
                                     a["B"], a["Hh"], a["d"], a["gh"], a["gw"], a["sp"], a["n"],
                                     vp(a["gamma"]), a["mode"], ctypes.c_float(a["qs"]),
                                     vp(a["s_in"]), vp(a["s_out"]), vp(a.get("ws")),
                                     ctypes.c_size_t(a.get("ws_bytes", 0)), None)


@pytest.mark.parametrize("kw,code", [
    (dict(d=48), 2), (dict(d=0), 2), (dict(B=0), 1), (dict(Hh=0), 1), (dict(gw=0), 1), (dict(mode=3), 1),
    (dict(sp=2, n=3), 1), (dict(sp=-1), 1), (dict(n=-1), 1), (dict(io=2), 1), (dict(io=0, out=1), 2),
    (dict(q=None), 1), (dict(gamma=None), 1), (dict(q=0x1004), 1), (dict(o=0x1000), 1),
    (dict(lq=Layout(512, 127, 64)), 1), (dict(lq=Layout(512, 32, 64)), 1), (dict(s_in=0x6008), 1),
    (dict(B=4, Hh=24, gh=64, gw=64, n=4096, lq=Layout(4096 * 1536, 1536, 64), lo=Layout(4096 * 1536, 1536, 64),
          ws=0x7000, ws_bytes=1024), 3),
])
def test_forward_rejects_bad_arguments_before_launch(lib, kw, code):
    """Every call here fails validation, so no kernel is launched (the pointers are fake)."""
    assert _forward(lib, **kw) == code
    assert len(lib.lasad_last_error()) > 0


def test_decode_and_decay_reject_bad_arguments(lib):
    vp, cf = ctypes.c_void_p, ctypes.c_float
    dec = lambda **k: lib.lasad_decode_step(vp(k.get("q", 0x1000)), vp(0x2000), vp(0x3000), vp(k.get("o", 0x4000)),
                                            k.get("io", 1), k.get("out", 1), k.get("B", 2), 2, k.get("d", 64), 4, 4,
                                            k.get("pos", 0), vp(0x5000), k.get("mode", 0), cf(1.0),
                                            vp(k.get("state", 0x6000)), None)
    assert dec(d=40) == 2
    assert dec(pos=16) == 1 and dec(pos=-1) == 1
    assert dec(state=None) == 1 and dec(q=None) == 1
    assert dec(io=0, out=1) == 2
    assert dec(mode=7) == 1 and dec(B=0) == 1
    assert dec(o=0x1000) == 1 and dec(state=0x6004) == 1
    dk = lambda **k: lib.lasad_decay_factors(vp(k.get("gamma", 0x1000)), k.get("Hh", 2), 4, k.get("gw", 4),
                                             k.get("sp", 0), k.get("n", 16), k.get("mode", 0),
                                             vp(0x2000), vp(0x3000), None)
    assert dk(sp=1) == 1 and dk(n=-2) == 1 and dk(gw=0) == 1 and dk(mode=-1) == 1
    assert dk(Hh=0) == 1 and dk(gamma=None) == 1


def test_gated_cached_decode_rejects_bad_arguments(lib):
    """Every check comes before the launch, so the error paths run without a GPU."""
    vp, cf = ctypes.c_void_p, ctypes.c_float
    lib.lasad_decode_step_gated_cached.argtypes = [vp] * 8 + [ctypes.c_int] * 10 + [cf, vp]
    lib.lasad_decode_step_gated_cached.restype = ctypes.c_int
    def dec(**k):
        return lib.lasad_decode_step_gated_cached(
            vp(k.get("q", 0x1000)), vp(k.get("lam", 0x2000)), vp(k.get("k", None)), vp(0x3000), vp(k.get("o", 0x4000)),
            vp(k.get("lc", 0x10000)), vp(k.get("kc", None)), vp(k.get("vc", 0x20000)), k.get("T", 16),
            k.get("io", 1), k.get("out", 1), k.get("B", 2), 2, k.get("d", 64), 4, 4, k.get("pos", 0), k.get("mode", 0),
            cf(1.0), None)
    assert dec(d=40) == 2 and dec(io=0, out=1) == 2
    assert dec(pos=16) == 1 and dec(pos=-1) == 1 and dec(pos=8, T=8) == 1 and dec(T=0) == 1
    assert dec(q=None) == 1 and dec(lam=None) == 1 and dec(lc=None) == 1 and dec(vc=None) == 1
    assert dec(k=0x5000) == 1 and dec(kc=0x30000) == 1            # own key and its cache go together
    assert dec(mode=7) == 1 and dec(B=0) == 1
    assert dec(o=0x1000) == 1 and dec(lc=0x20000) == 1 and dec(k=0x5000, kc=0x20000) == 1
    assert dec(lam=0x2004) == 1 and dec(vc=0x20008) == 1
    assert b"alias" in lib.lasad_last_error() or b"aligned" in lib.lasad_last_error()


def _backward_layer(lib, norm_only=False, **kw):
    dense = Layout(4 * 2 * 64, 2 * 64, 64)
    a = dict(q=0x1000, z=0x2000, v=0x3000, g=0x4000, dq=0x5000, dz=0x6000, dv=0x7000, dw=0x8000, d_o=0x5000,
             li=dense, lo=dense, lg=dense, io=1, gd=1, B=1, Hh=2, d=64, gh=2, gw=2, sp=0, n=4, mode=0, qs=1.0,
             w=0x9000, eps=1e-6, ws=0x10000, ws_bytes=0)
    a.update(kw)
    vp, cf = ctypes.c_void_p, ctypes.c_float
    tail = (a["B"], a["Hh"], a["d"], a["gh"], a["gw"], a["sp"], a["n"], a["mode"], cf(a["qs"]), vp(a["w"]), cf(a["eps"]),
            vp(a["ws"]), ctypes.c_size_t(a["ws_bytes"]), None)
    if norm_only:
        return lib.lasad_backward_layer_norm(vp(a["q"]), vp(a["z"]), vp(a["v"]), vp(a["g"]), vp(a["d_o"]), vp(a["dw"]),
                                             ctypes.byref(a["li"]), ctypes.byref(a["lo"]), ctypes.byref(a["lg"]),
                                             a["io"], a.get("d_o_dtype", a["io"]), *tail)
    return lib.lasad_backward_layer(vp(a["q"]), vp(a["z"]), vp(a["v"]), vp(a["g"]), vp(a["dq"]), vp(a["dz"]), vp(a["dv"]),
                                    vp(a["dw"]), ctypes.byref(a["li"]), ctypes.byref(a["lo"]), ctypes.byref(a["lg"]),
                                    a["io"], a["gd"], *tail)


@pytest.mark.parametrize("kw,code", [
    (dict(d=32), 2), (dict(B=0), 1), (dict(gw=0), 1), (dict(mode=5), 1), (dict(sp=3, n=2), 1), (dict(io=3), 1),
    (dict(io=0, gd=1), 2), (dict(q=None), 1), (dict(g=None), 1), (dict(dz=None), 1), (dict(dq=0x1000), 1),
    (dict(dz=0x5000), 1), (dict(dw=0x8004), 1), (dict(w=0x9008), 1), (dict(lo=Layout(512, 100, 64)), 1),
    (dict(lg=Layout(512, 32, 64)), 1), (dict(ws=0x10010), 1),
    (dict(), 3), (dict(ws=None, ws_bytes=1 << 30), 3),          # workspace too small / missing
])
def test_backward_layer_rejects_bad_arguments_before_launch(lib, kw, code):
    """Validation failures only: nothing is launched (the pointers are fake)."""
    assert _backward_layer(lib, **kw) == code
    assert len(lib.lasad_last_error()) > 0


def test_backward_layer_norm_rejects_bad_arguments_and_sizes_its_workspace(lib):
    assert _backward_layer(lib, norm_only=True, d_o=None) == 1
    assert _backward_layer(lib, norm_only=True, eps=-1.0) == 1          # no normalisation to differentiate
    assert _backward_layer(lib, norm_only=True, d_o=0x4000) == 1        # aliases d_out
    assert _backward_layer(lib, norm_only=True) == 3                    # workspace too small
    assert _backward_layer(lib, norm_only=True, d_o_dtype=0) == 3       # fp32 d_o of bf16 inputs is accepted
    assert _backward_layer(lib, norm_only=True, io=0, d_o_dtype=1) == 2 # bf16 d_o of fp32 inputs is not
    assert _backward_layer(lib, norm_only=True, d_o_dtype=5) == 1
    lib.lasad_backward_layer_workspace_bytes.restype = ctypes.c_size_t
    lib.lasad_backward_gated_workspace_bytes.restype = ctypes.c_size_t
    size = lambda l, io=1: lib.lasad_backward_layer_workspace_bytes(2, 3, 100, 64, io, ctypes.byref(l))
    dense = Layout(100 * 3 * 64, 3 * 64, 64)
    wide = Layout(100 * 9 * 64, 9 * 64, 64)                              # q_pre, z, v cut from one projection
    core = lib.lasad_backward_gated_workspace_bytes(2, 3, 100, 64)
    n_el = 2 * 3 * 100 * 64
    # the recurrence's workspace, o in fp32, d_o over the span of the input view (bf16: as a pair of tensors; fp32:
    # one), partial sums of the weight gradient
    assert size(dense) >= core + 4 * n_el + 2 * 2 * n_el + 2 * 3 * 2 * 64 * 4
    assert size(dense) < core + 4 * n_el + 2 * 2 * n_el + 2 * 3 * 2 * 64 * 4 + 6 * 256
    assert size(wide) - size(dense) >= 2 * 2 * (3 * n_el - 3 * 64 * 2 - n_el) - 512
    assert abs(size(dense, io=0) - size(dense)) <= 512
    assert lib.lasad_backward_layer_workspace_bytes(0, 3, 100, 64, 1, ctypes.byref(dense)) == 0
    assert lib.lasad_backward_layer_workspace_bytes(2, 3, 100, 64, 1, None) == 0


def test_static_forward_entry_validates_like_the_workspace_entry(lib):
    """lasad_forward_chunked_static: same argument checks (nothing is launched: the pointers are fake) and an
    8 MiB built-in scratch array that covers every size the segment plan asks for."""
    lib.lasad_forward_static_scratch_bytes.restype = ctypes.c_size_t
    assert lib.lasad_forward_static_scratch_bytes() == 8 << 20
    for B, Hh, n in ((4, 24, 4096), (1, 1, 1 << 20), (2, 100, 8192), (255, 1, 2048)):
        assert lib.lasad_forward_workspace_bytes(B, Hh, n, 64, 1) <= 8 << 20
    vp = ctypes.c_void_p
    lay = Layout(64 * 4 * 2, 2 * 64, 64)
    call = lambda **k: lib.lasad_forward_chunked_static(
        vp(k.get("q", 0x1000)), vp(0x2000), vp(0x3000), vp(k.get("o", 0x4000)), ctypes.byref(lay), ctypes.byref(lay),
        1, 1, k.get("B", 1), 2, k.get("d", 64), 2, 2, 0, k.get("n", 4), vp(k.get("gamma", 0x5000)), 0,
        ctypes.c_float(1.0), None, None, None)
    assert call(d=48) == 2 and call(B=0) == 1 and call(n=5) == 1 and call(q=None) == 1
    assert call(o=0x1000) == 1 and call(gamma=None) == 1


def test_backward_carried_entry_validates_and_sizes_its_workspace(lib):
    """lasad_backward_chunked_carried: the zero-state call's checks plus those of the three states (nothing is
    launched: the pointers are fake); its workspace is the zero-state call's plus five d x d matrices and one sum
    per sequence."""
    lib.lasad_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.lasad_backward_carried_workspace_bytes.restype = ctypes.c_size_t
    base = lib.lasad_backward_workspace_bytes(2, 3, 100, 64, 1)
    carried = lib.lasad_backward_carried_workspace_bytes(2, 3, 100, 64, 1)
    assert 5 * 6 * 64 * 64 * 4 <= carried - base <= 5 * 6 * 64 * 64 * 4 + 512
    assert lib.lasad_backward_carried_workspace_bytes(0, 3, 100, 64, 1) == 0
    vp, cf = ctypes.c_void_p, ctypes.c_float
    dense = Layout(4 * 2 * 64, 2 * 64, 64)

    def call(**k):
        a = dict(q=0x1000, s0=0x20000, h=0x30000, ds0=0x40000, dq=0x5000, io=1, gd=1, d=64, n=4, qs=1.0, ws=0x100000, ws_bytes=0)
        a.update(k)
        return lib.lasad_backward_chunked_carried(
            vp(a["q"]), vp(0x2000), vp(0x3000), vp(0x4000), vp(a["s0"]), vp(a["h"]),
            vp(a["dq"]), vp(0x6000), vp(0x7000), vp(0x8000), vp(a["ds0"]),
            ctypes.byref(dense), ctypes.byref(dense), a["io"], a["gd"], 1, 2, a["d"], 2, 2, 0, a["n"],
            vp(0x9000), 0, cf(a["qs"]), vp(a["ws"]), ctypes.c_size_t(a["ws_bytes"]), None)

    assert call() == 3                                     # workspace too small
    assert call(s0=None, h=None, ds0=None) == 3            # every state is optional
    assert call(q=None) == 1 and call(d=48) == 2 and call(n=5) == 1 and call(io=0, gd=1) == 2
    assert call(s0=0x20004) == 1 and call(h=0x30008) == 1 and call(ds0=0x4000c) == 1      # misaligned states
    assert call(ds0=0x20000) == 1 and call(ds0=0x30000) == 1                               # d_state_in aliases an input
    assert call(qs=0.0) == 2 and call(qs=0.0, h=None) == 3                                  # q_scale 0 needs no final-state gradient
    assert len(lib.lasad_last_error()) > 0


def test_backward_gated_carried_entry_validates_and_sizes_its_workspace(lib):
    lib.lasad_backward_gated_workspace_bytes.restype = ctypes.c_size_t
    lib.lasad_backward_gated_carried_workspace_bytes.restype = ctypes.c_size_t
    extra = lib.lasad_backward_gated_carried_workspace_bytes(2, 3, 100, 64) - lib.lasad_backward_gated_workspace_bytes(2, 3, 100, 64)
    assert extra == 3 * 6 * 64 * 64 * 4 + 6 * 64 * 4
    vp, cf = ctypes.c_void_p, ctypes.c_float
    dense = Layout(4 * 2 * 64, 2 * 64, 64)

    def call(**k):
        a = dict(q=0x1000, s0=0x20000, h=0x30000, ds0=0x40000, d=64, n=4, qs=1.0, kk=None, dk=None)
        a.update(k)
        return lib.lasad_backward_gated_carried(
            vp(a["q"]), vp(0x2000), vp(a["kk"]), vp(0x3000), vp(0x4000), vp(a["s0"]), vp(a["h"]),
            vp(0x5000), vp(0x6000), vp(a["dk"]), vp(0x7000), vp(a["ds0"]),
            ctypes.byref(dense), ctypes.byref(dense), 1, 1, 1, 2, a["d"], 2, 2, 0, a["n"], 0, cf(a["qs"]),
            vp(0x100000), ctypes.c_size_t(0), None)

    assert call() == 3 and call(s0=None, h=None, ds0=None) == 3
    assert call(q=None) == 1 and call(d=48) == 2 and call(n=5) == 1 and call(kk=0x8000) == 1     # dk must come with k
    assert call(s0=0x20004) == 1 and call(ds0=0x30000) == 1 and call(qs=0.0) == 2
