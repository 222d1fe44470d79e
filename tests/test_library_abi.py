"""CPU-only checks of the C-ABI library: it loads, exports what include/specgbv.h
declares, sizes its workspace sanely and rejects bad arguments before touching the GPU."""
import ctypes
import os
import re

import pytest

import paper_2604_25925_amd as sg
from paper_2604_25925_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "specgbv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(specgbv_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = sg.load_library()
    names = _declared_functions()
    assert "specgbv_verify" in names and "specgbv_workspace_bytes" in names and len(names) >= 6
    for n in names:
        assert hasattr(lib, n), "libspecgbv.so does not export %s" % n
    assert sorted(binding.EXPORTS) == names
    assert "gfx950" in sg.specgbv_version()


def test_binding_has_same_names_as_the_abi():
    for n in _declared_functions():
        assert hasattr(sg, n), "python binding lacks %s" % n


def test_workspace_bytes():
    small = sg.specgbv_workspace_bytes(1, 2, 4, 1000, 0)
    big = sg.specgbv_workspace_bytes(128, 16, 8, 152064, 1)
    assert 0 < small < big < 64 << 20
    assert small % 256 == 0
    assert sg.specgbv_workspace_bytes(1, 0, 4, 1000, 0) == 0
    assert sg.specgbv_workspace_bytes(1, 2, 4, 1000, 7) == 0
    assert sg.specgbv_workspace_bytes(1, 65, 4, 1000, 0) == 0       # beyond SPECGBV_MAX_K
    assert sg.specgbv_workspace_bytes(0, 2, 4, 1000, 0) > 0


def _call(lib, **kw):
    a = dict(t=1 << 20, d=1 << 20, tok=1 << 20, K=2, L=3, V=64, B=1, dt=0, T=1.0, out=1 << 20, ws=1 << 20,
             wsb=1 << 30)
    a.update(kw)
    return lib.specgbv_verify(a["t"], a["d"], a["tok"], a["K"], a["L"], a["V"], a["B"], a["dt"],
                              ctypes.c_float(a["T"]), 0, 0, a["out"], a["out"], a["out"], a["ws"], a["wsb"], None)


def test_argument_errors_are_caught_before_any_launch():
    # the pointers below are never dereferenced: every call must fail in the host checks
    lib = sg.load_library()
    assert _call(lib, K=0) == 1 and "K" in sg.specgbv_last_error()
    assert _call(lib, V=-5) == 1
    assert _call(lib, B=-1) == 1
    assert _call(lib, dt=3) == 1
    assert _call(lib, T=0.0) == 1 and "temperature" in sg.specgbv_last_error()
    assert _call(lib, T=float("inf")) == 1
    assert _call(lib, t=None) == 1
    assert _call(lib, out=None) == 1
    assert _call(lib, t=(1 << 20) + 2) == 1                 # misaligned float pointer
    assert _call(lib, K=65) == 2                            # over the limit: unsupported
    assert _call(lib, L=63) == 2
    assert _call(lib, K=64, L=32) == 2                      # K*L over 1024
    assert _call(lib, ws=None) == 3
    assert _call(lib, ws=(1 << 20) + 8) == 3                # misaligned workspace
    assert _call(lib, wsb=128) == 3 and "need" in sg.specgbv_last_error()
    assert _call(lib, B=0) == 0                             # empty batch: nothing to do


def test_comparison_and_static_entry_point_errors_are_caught_before_any_launch():
    lib = sg.load_library()
    P = 1 << 20

    def kseq(K=4, L=3, V=64, B=1, dt=0, T=1.0, nd=2, t=P, ws=P, wsb=1 << 30):
        return lib.specgbv_verify_kseq(t, P, P, K, L, V, B, dt, ctypes.c_float(T), 0, 0, nd, P, P, P, ws, wsb, None)
    assert kseq(nd=0) == 1 and "ndrafts" in sg.specgbv_last_error()
    assert kseq(nd=5) == 1                                   # more drafts than the tensors hold
    assert kseq(K=0) == 1 and kseq(T=-1.0) == 1 and kseq(dt=7) == 1 and kseq(t=None) == 1
    assert kseq(K=65, nd=1) == 2
    assert kseq(ws=None) == 3 and kseq(wsb=64) == 3 and "need" in sg.specgbv_last_error()
    assert kseq(B=0) == 0

    def static(K=8, L=8, V=128256, B=32, dt=1):
        return lib.specgbv_verify_static(P, P, P, K, L, V, B, dt, ctypes.c_float(1.0), 0, 0, P, P, P, None)
    assert static(K=0) == 1
    assert static(K=65) == 2
    # the built-in scratch buffer has a fixed size: larger shapes are refused with the size they would need
    assert static(K=16, L=8, V=152064, B=128) == 2 and "SPECGBV_STATIC_SCRATCH_BYTES" in sg.specgbv_last_error()
    assert sg.specgbv_workspace_bytes(128, 16, 8, 152064, 1) > sg.STATIC_SCRATCH_BYTES >= sg.specgbv_workspace_bytes(32, 8, 8, 128256, 1)


def test_pending_option_errors_are_caught_before_any_launch():
    from paper_2604_25925_amd.binding import _Options
    lib = sg.load_library()
    P = 1 << 20

    def call(algo, carry, count):
        opt = _Options(algo, 0, None, None, carry, count, None)
        return lib.specgbv_verify_ex(P, P, P, 2, 3, 64, 1, 0, ctypes.c_float(1.0), 0, 0, P, P, P, P, 1 << 30, None,
                                     ctypes.byref(opt))
    assert call(0, P, None) == 1 and "together" in sg.specgbv_last_error()      # one pointer without the other
    assert call(0, None, P) == 1
    assert call(0, P + 4, P) == 1                                               # misaligned float64 pointer
    assert call(2, P, P) == 2 and "on chip" in sg.specgbv_last_error()          # chain schedule: row too short for it

    def call2(levels, carry, count, state, L=3):
        opt = _Options(0, levels, None, None, carry, count, state)
        return lib.specgbv_verify_ex(P, P, P, 2, L, 64, 1, 0, ctypes.c_float(1.0), 0, 0, P, P, P, P, 1 << 30, None,
                                     ctypes.byref(opt))
    assert call2(17, P, P, None) == 2 and "SPECGBV_MAX_PENDING" in sg.specgbv_last_error()
    assert call2(2, None, None, None) == 1                                      # levels without the arrays
    assert call2(0, P, P, P) == 1 and "not both" in sg.specgbv_last_error()
    assert call2(0, None, None, P + 4) == 1                                     # misaligned state
    assert call2(0, None, None, P, L=18) == 2                                   # more levels than the state holds
    assert sg.specgbv_pending_state_bytes(32) >= 32 * sg.MAX_PENDING * 12 and sg.specgbv_pending_state_bytes(-1) == 0


def test_modify_target_argument_errors():
    lib = sg.load_library()
    P = 1 << 20

    def call(**kw):
        a = dict(t=P, d=P, tok=P, K=2, M=3, bonus=0, V=64, B=1, dt=0, T=1.0, carry=P, count=P, out=P, ws=P,
                 wsb=1 << 30)
        a.update(kw)
        return lib.specgbv_modify_target(a["t"], a["d"], a["tok"], a["K"], a["M"], a["bonus"], a["V"], a["B"], a["dt"],
                                         ctypes.c_float(a["T"]), a["carry"], a["count"], a["out"], None, None, None,
                                         a["ws"], a["wsb"], None)
    assert call(K=0) == 1 and call(M=0) == 1 and call(V=0) == 1 and call(B=-1) == 1
    assert call(dt=2) == 1 and call(T=-1.0) == 1 and call(bonus=2) == 1
    assert call(carry=None) == 1 and call(out=None) == 1 and call(t=None) == 1
    assert call(K=65) == 2 and call(M=63) == 2
    assert call(ws=None) == 3 and call(ws=P + 8) == 3 and call(wsb=64) == 3
    assert call(B=0) == 0
    assert 0 < sg.specgbv_modify_workspace_bytes(32, 8, 8, 1) < 1 << 20
    assert sg.specgbv_modify_workspace_bytes(32, 8, 0, 0) == 0
    a, b = ctypes.c_void_p(), ctypes.c_void_p()
    need = sg.specgbv_workspace_bytes(4, 2, 3, 64, 0)
    assert lib.specgbv_workspace_carry(P, need, 4, 2, 3, 64, ctypes.byref(a), ctypes.byref(b)) == 0
    assert P < a.value < b.value < P + need and a.value % 8 == 0 and b.value % 4 == 0
    assert lib.specgbv_workspace_carry(P, need - 1, 4, 2, 3, 64, ctypes.byref(a), ctypes.byref(b)) == 3
    assert lib.specgbv_workspace_carry(None, need, 4, 2, 3, 64, ctypes.byref(a), ctypes.byref(b)) == 1


def test_python_binding_validates_tensors():
    import torch
    t = torch.zeros((1, 2, 4, 64))
    d = torch.zeros((1, 2, 3, 64))
    tok = torch.zeros((1, 2, 3), dtype=torch.int32)
    with pytest.raises(ValueError):
        sg.specgbv_verify(t, d, tok, 1.0, 0, 0)             # CPU tensors: no silent fallback
    with pytest.raises(ValueError):
        sg.specgbv_verify(t, d[:, :, :2], tok, 1.0, 0, 0)


def test_ctypes_structures_match_the_c_header(tmp_path):
    """The binding's ctypes mirrors of specgbv_options and specgbv_intermediates have the layout the C compiler
    gives the header's structures (sizes and every field offset), so a field added on one side only is caught."""
    import ctypes
    import shutil
    import subprocess
    from paper_2604_25925_amd import binding
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    header = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "specgbv.h")
    lines = ['#include <stddef.h>', '#include <stdio.h>', '#include "%s"' % header, 'int main(void) {']
    for cname, cls in (("specgbv_options", binding._Options), ("specgbv_intermediates", binding._Intermediates)):
        lines.append('printf("%s %%zu\\n", sizeof(%s));' % (cname, cname))
        for field, _ in cls._fields_:
            lines.append('printf("%s.%s %%zu\\n", offsetof(%s, %s));' % (cname, field, cname, field))
    lines += ['return 0; }']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run([cc, "-std=c99", "-o", str(exe), str(src)], check=True)
    got = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for cname, cls in (("specgbv_options", binding._Options), ("specgbv_intermediates", binding._Intermediates)):
        assert int(got[cname]) == ctypes.sizeof(cls), cname
        for field, _ in cls._fields_:
            assert int(got["%s.%s" % (cname, field)]) == getattr(cls, field).offset, "%s.%s" % (cname, field)
