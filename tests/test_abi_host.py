"""Host-side checks of the C ABI that need no GPU: the library loads, exports what include/ll.h
declares, sizes workspaces, and rejects bad arguments before touching the device."""
import ctypes
import math
import os
import re

import pytest

from paper_2604_06483_amd import binding as LL

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ll.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ll_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert {"ll_project", "ll_steer_vector", "ll_steer_inject", "ll_workspace_bytes", "ll_error_string"} <= set(names)
    L = LL.lib()
    for n in names:
        assert hasattr(L, n), f"{n} is declared in ll.h but not exported"


def test_header_constants_match_binding():
    text = open(HEADER).read()
    for name in ("LL_OK", "LL_EINVAL", "LL_EWORKSPACE", "LL_EHIP", "LL_ESCRATCH", "LL_KMAX"):
        m = re.search(rf"#define\s+{name}\s+(-?\d+)", text)
        assert m and int(m.group(1)) == getattr(LL, name)
    m = re.search(r"#define\s+LL_STATIC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", text)
    assert m and int(m.group(1)) << int(m.group(2)) == LL.LL_STATIC_SCRATCH_BYTES


def test_error_strings():
    L = LL.lib()
    seen = {L.ll_error_string(c) for c in (0, -1, -2, -3, -4)}
    assert len(seen) == 5 and all(s for s in seen)
    assert L.ll_error_string(-99) == b"unknown error code"
    assert L.ll_last_hip_error() == 0


def test_workspace_arithmetic():
    # invalid shapes and k give 0
    assert LL.ll_workspace_bytes(10, 0, 100, 5) == 0
    assert LL.ll_workspace_bytes(10, 100, 100, 5) == 0          # d not a multiple of 8
    assert LL.ll_workspace_bytes(10, 64, 100, 0) == 0
    assert LL.ll_workspace_bytes(10, 64, 100, LL.LL_KMAX + 1) == 0
    assert LL.ll_workspace_bytes(10, 64, 4, 5) == 0             # k > V
    assert LL.ll_workspace_bytes(-1, 64, 100, 5) == 0
    assert LL.ll_workspace_bytes(0, 64, 100, 5) > 0
    assert LL.ll_workspace_bytes(10, 64, 2 ** 31 - 1, 5) == 0   # rounding V up to whole tiles would leave 32 bits
    assert LL.ll_workspace_bytes(10, 64, 2 ** 31 - 257, 5) > 0
    # grows with k, is bounded in N beyond one pass (only 4 bytes per extra row)
    a = LL.ll_workspace_bytes(8192, 8192, 128256, 20)
    b = LL.ll_workspace_bytes(121500, 8192, 128256, 20)
    assert a % 256 == 0 and b % 256 == 0
    assert 0 < b - a <= (121500 - 8192) * 4 + 256
    assert LL.ll_workspace_bytes(8192, 8192, 128256, 10) < a
    assert b < 256 * 2 ** 20                                      # "bounded workspace": tens of MB
    assert LL.ll_steer_workspace_bytes(4096) > 0 and LL.ll_steer_workspace_bytes(4097) == 0


def _fake(n=1 << 20):
    return ctypes.c_void_p(n)        # a non-null, 16-byte aligned address that is never dereferenced


def test_project_rejects_bad_arguments_without_touching_the_gpu():
    L = LL.lib()
    s = LL.ll_shape(16, 64, 300)
    ok = dict(shape=s, ws=_fake(4096 * 256), wsb=1 << 30, h=_fake(), g=_fake(), w=_fake(), eps=1e-5, k=4, t=_fake(),
              ids=_fake(), p=_fake(), lp=_fake(), e=_fake(), st=None)

    def call(**kw):
        a = dict(ok, **kw)
        return L.ll_project(a["shape"], a["ws"], a["wsb"], a["h"], a["g"], a["w"], a["eps"], a["k"], a["t"],
                            a["ids"], a["p"], a["lp"], a["e"], a["st"])

    assert call(shape=None) == LL.LL_EINVAL
    assert call(h=None) == LL.LL_EINVAL
    assert call(w=None) == LL.LL_EINVAL
    assert call(ids=None) == LL.LL_EINVAL
    assert call(p=None) == LL.LL_EINVAL
    assert call(e=None) == LL.LL_EINVAL
    assert call(lp=None) == LL.LL_EINVAL                        # target ids given but nowhere to write
    assert call(k=0) == LL.LL_EINVAL
    assert call(k=LL.LL_KMAX + 1) == LL.LL_EINVAL
    assert call(k=301 if 301 <= LL.LL_KMAX else 33) == LL.LL_EINVAL
    assert call(shape=LL.ll_shape(16, 60, 300)) == LL.LL_EINVAL   # d % 8
    assert call(shape=LL.ll_shape(-1, 64, 300)) == LL.LL_EINVAL
    assert call(shape=LL.ll_shape(16, 64, 3)) == LL.LL_EINVAL     # k > V
    assert call(eps=float("nan")) == LL.LL_EINVAL
    assert call(eps=-1.0) == LL.LL_EINVAL
    assert call(h=_fake((1 << 20) + 2)) == LL.LL_EINVAL           # misaligned
    assert call(ws=None) == LL.LL_EWORKSPACE
    assert call(wsb=1024) == LL.LL_EWORKSPACE
    assert call(ws=_fake((1 << 20) + 16)) == LL.LL_EWORKSPACE     # not 256-byte aligned
    # N == 0 succeeds with nothing else looked at
    assert call(shape=LL.ll_shape(0, 64, 300), h=None, w=None, ws=None, wsb=0) == LL.LL_OK
    ms = (ctypes.c_float * 3)()
    a = ok
    assert L.ll_project_timed(a["shape"], a["ws"], a["wsb"], a["h"], a["g"], a["w"], a["eps"], a["k"], a["t"],
                              a["ids"], a["p"], a["lp"], a["e"], a["st"], None) == LL.LL_EINVAL


def test_static_variant_sizes_its_passes_and_rejects_what_does_not_fit():
    """ll_project_static: pass size from host arithmetic; bad arguments and oversized shapes are refused before
    anything touches the device (fake pointers, no GPU)."""
    L = LL.lib()
    f = _fake()
    # the usual pass when the plan fits the static buffer
    assert LL.ll_project_static_pass_rows(700, 256, 5000, 10) == 8192
    assert LL.ll_workspace_bytes(8192, 256, 5000, 10) <= LL.LL_STATIC_SCRATCH_BYTES
    # d = 8192, k = 20: the 8192-row plan is larger than the buffer, a smaller multiple of 256 is used
    assert LL.ll_workspace_bytes(8192, 8192, 128256, 20) > LL.LL_STATIC_SCRATCH_BYTES
    rows = LL.ll_project_static_pass_rows(121500, 8192, 128256, 20)
    assert 256 <= rows < 8192 and rows % 256 == 0
    assert LL.ll_workspace_bytes(rows, 8192, 128256, 20) <= LL.LL_STATIC_SCRATCH_BYTES + 121500 * 4
    assert LL.ll_project_static_pass_rows(81, 8192, 128256, 20) > 0          # one decoding step's rows always fit
    # invalid shape or k: 0 rows, LL_EINVAL
    assert LL.ll_project_static_pass_rows(10, 60, 100, 5) == 0
    assert LL.ll_project_static_pass_rows(10, 64, 100, 0) == 0
    call = lambda shape, k=4, h=f, w=f, ids=f: L.ll_project_static(shape, h, f, w, 1e-5, k, f, ids, f, f, f, None)
    assert call(LL.ll_shape(16, 60, 300)) == LL.LL_EINVAL
    assert call(LL.ll_shape(16, 64, 300), k=0) == LL.LL_EINVAL
    assert call(None) == LL.LL_EINVAL
    assert call(LL.ll_shape(0, 64, 300), h=None, w=None, ids=None) == LL.LL_OK
    # not even one row block fits: refused with its own code
    big = LL.ll_shape(1000, 1 << 18, 300)
    assert LL.ll_project_static_pass_rows(1000, 1 << 18, 300, 4) == 0
    assert LL.ll_project_static_pass_rows(16, 1 << 18, 300, 4) > 0            # a handful of such rows does fit
    assert call(big) == LL.LL_ESCRATCH
    assert b"static" in L.ll_error_string(LL.LL_ESCRATCH)


def test_project_ex_rejects_unknown_flags_and_misaligned_bias():
    L = LL.lib()
    f = _fake()
    s = LL.ll_shape(16, 64, 300)
    args = lambda bias, flags: (s, _fake(4096 * 256), 1 << 30, f, f, f, bias, flags, 1e-5, 4, f, f, f, f, f, None)
    assert L.ll_project_ex(*args(None, 4)) == LL.LL_EINVAL
    assert L.ll_project_ex(*args(None, 0xFFFF)) == LL.LL_EINVAL
    assert LL.LL_FLAG_TOPK_SOFTMAX == 1 and LL.LL_FLAG_REGISTER_STAGED == 2      # the two bits that are defined
    assert L.ll_project_ex(*args(_fake((1 << 20) + 2), 0)) == LL.LL_EINVAL
    assert L.ll_project_ex(LL.ll_shape(0, 64, 300), None, 0, None, None, None, None, 1, 1e-5, 4, None, None, None, None,
                           None, None) == LL.LL_OK


def test_steer_calls_reject_bad_arguments():
    L = LL.lib()
    f = _fake()
    assert L.ll_steer_vector(None, 4, f, 4, 64, 1, f, None, 0, None) == LL.LL_EINVAL
    assert L.ll_steer_vector(f, 0, f, 4, 64, 1, f, None, 0, None) == LL.LL_EINVAL
    assert L.ll_steer_vector(f, 4, f, 4, 60, 1, f, None, 0, None) == LL.LL_EINVAL
    assert L.ll_steer_vector(f, 4, f, 4, 64, 1, None, None, 0, None) == LL.LL_EINVAL
    assert L.ll_steer_vector(f, 4, f, 4, 64, 1, f, f, 16, None) == LL.LL_EWORKSPACE
    s = LL.ll_shape(4, 64, 0)
    assert L.ll_steer_inject(None, f, f, 1e-5, f, 1.0, f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject(s, None, f, 1e-5, f, 1.0, f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject(s, f, None, 1e-5, f, 1.0, f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject(s, f, f, 1e-5, None, 1.0, f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject(s, f, f, 1e-5, f, 1.0, None, None) == LL.LL_EINVAL
    assert L.ll_steer_inject(LL.ll_shape(4, 63, 0), f, f, 1e-5, f, 1.0, f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject(LL.ll_shape(0, 64, 0), None, None, 1e-5, None, 1.0, None, None) == LL.LL_OK


def test_steer_sweep_rejects_bad_arguments_before_any_device_work():
    L = LL.lib()
    f = _fake()
    al = (ctypes.c_float * 9)(*range(-4, 5))
    s = LL.ll_shape(16, 64, 300)
    need = LL.ll_steer_sweep_workspace_bytes(16, 64, 300, 9)
    assert need > 0 and need % 256 == 0
    assert LL.ll_steer_sweep_workspace_bytes(16, 72, 300, 9) > 0         # any multiple of 8 (the register-staged kernel)
    assert LL.ll_steer_sweep_workspace_bytes(16, 76, 300, 9) == 0        # d not a multiple of 8
    assert LL.ll_steer_sweep_workspace_bytes(16, 40960, 300, 9) > 0      # the largest hidden size: v is held in LDS
    assert LL.ll_steer_sweep_workspace_bytes(16, 40968, 300, 9) == 0
    # lists of up to LL_SWEEP_KMAX tokens per alpha cost workspace; longer lists are refused
    assert LL.ll_steer_sweep_workspace_bytes(16, 64, 300, 9, 3) > need
    assert LL.ll_steer_sweep_workspace_bytes(16, 64, 300, 9, LL.LL_SWEEP_KMAX + 1) == 0
    assert LL.ll_steer_sweep_workspace_bytes(16, 64, 2, 9, 3) == 0       # k > V
    assert LL.ll_steer_sweep_workspace_bytes(16, 64, 300, 0) == 0
    assert LL.ll_steer_sweep_workspace_bytes(16, 64, 300, LL.LL_SWEEP_MAX + 1) == 0
    # the table of alpha * (W_U v) is part of the workspace: more alphas, more bytes
    assert LL.ll_steer_sweep_workspace_bytes(16, 64, 300, 9) > LL.ll_steer_sweep_workspace_bytes(16, 64, 300, 1)
    call = lambda **kw: L.ll_steer_sweep(*[{**dict(shape=s, ws=_fake(4096 * 256), wsb=1 << 30, h=f, g=f, w=f, eps=1e-5, v=f,
                                                   al=al, n=9, t=f, ids=f, p=f, lp=f, e=f, st=None), **kw}[k]
                                           for k in ("shape", "ws", "wsb", "h", "g", "w", "eps", "v", "al", "n", "t", "ids",
                                                     "p", "lp", "e", "st")])
    for bad in (dict(h=None), dict(w=None), dict(v=None), dict(al=None), dict(ids=None), dict(p=None), dict(e=None),
                dict(lp=None), dict(n=0), dict(n=10), dict(eps=-1.0), dict(shape=LL.ll_shape(16, 76, 300)),
                dict(shape=LL.ll_shape(16, 40968, 300)),
                dict(v=_fake((1 << 20) + 4))):
        assert call(**bad) == LL.LL_EINVAL, bad
    nan = (ctypes.c_float * 9)(*([0.0] * 8 + [float("nan")]))
    assert call(al=nan) == LL.LL_EINVAL
    assert call(ws=None) == LL.LL_EWORKSPACE
    assert call(wsb=1024) == LL.LL_EWORKSPACE
    assert call(shape=LL.ll_shape(0, 64, 300), h=None, w=None, ws=None, wsb=0) == LL.LL_OK
    # the variant with lists: k out of range
    topk = lambda k: L.ll_steer_sweep_topk(s, _fake(4096 * 256), 1 << 30, f, f, f, 1e-5, f, al, 9, k, f, f, f, f, f, None)
    assert topk(0) == LL.LL_EINVAL and topk(LL.LL_SWEEP_KMAX + 1) == LL.LL_EINVAL
    m = re.search(r"#define\s+LL_SWEEP_KMAX\s+(\d+)", open(HEADER).read())
    assert m and int(m.group(1)) == LL.LL_SWEEP_KMAX


def test_inject_raw_and_capture_append_reject_bad_arguments():
    L = LL.lib()
    f = _fake()
    s = LL.ll_shape(4, 64, 0)
    assert L.ll_steer_inject_raw(None, f, f, 1.0, 1.0, 0.1, f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject_raw(s, None, f, 1.0, 1.0, 0.1, f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject_raw(s, f, None, 1.0, 1.0, 0.1, f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject_raw(s, f, f, 1.0, 1.0, 0.1, None, None) == LL.LL_EINVAL
    assert L.ll_steer_inject_raw(s, f, f, float("inf"), 1.0, 0.1, f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject_raw(s, f, f, 1.0, 1.0, float("nan"), f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject_raw(LL.ll_shape(4, 60, 0), f, f, 1.0, 1.0, 0.1, f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject_raw(LL.ll_shape(0, 64, 0), None, None, 1.0, 1.0, 0.1, None, None) == LL.LL_OK
    too_many = LL.ll_shape(4 * (2 ** 31 - 1) + 1, 64, 0)                          # more rows than the grid can hold
    assert L.ll_steer_inject_raw(too_many, f, f, 1.0, 1.0, 0.1, f, None) == LL.LL_EINVAL
    assert L.ll_steer_inject(too_many, f, f, 1e-5, f, 1.0, f, None) == LL.LL_EINVAL
    cs = LL.ll_capture_shape(3, 2, 100, 64)
    assert L.ll_capture_append(None, f, f, 0, 1, None) == LL.LL_EINVAL
    assert L.ll_capture_append(cs, None, f, 0, 1, None) == LL.LL_EINVAL
    assert L.ll_capture_append(cs, f, None, 0, 1, None) == LL.LL_EINVAL
    assert L.ll_capture_append(cs, f, f, -1, 1, None) == LL.LL_EINVAL
    assert L.ll_capture_append(cs, f, f, 0, -1, None) == LL.LL_EINVAL
    assert L.ll_capture_append(cs, f, f, 100, 1, None) == LL.LL_EINVAL          # past the capacity
    assert L.ll_capture_append(cs, f, f, 60, 41, None) == LL.LL_EINVAL
    assert L.ll_capture_append(cs, _fake((1 << 20) + 8), f, 0, 1, None) == LL.LL_EINVAL
    assert L.ll_capture_append(LL.ll_capture_shape(3, 2, 100, 60), f, f, 0, 1, None) == LL.LL_EINVAL
    assert L.ll_capture_append(LL.ll_capture_shape(0, 2, 100, 64), f, f, 0, 1, None) == LL.LL_EINVAL
    assert L.ll_capture_append(cs, None, None, 100, 0, None) == LL.LL_OK         # nothing to append
    huge = LL.ll_capture_shape(2 ** 31 - 1, 2 ** 31 - 1, 2 ** 40, 64)           # L * C * T leaves 64 bits
    assert L.ll_capture_append(huge, f, f, 0, 1, None) == LL.LL_EINVAL


def test_binding_refuses_cpu_tensors():
    import torch
    h = torch.zeros(4, 64, dtype=torch.bfloat16)
    with pytest.raises(TypeError):
        LL.ll_project(h, h[0], torch.zeros(300, 64, dtype=torch.bfloat16), 1e-5, 3)
