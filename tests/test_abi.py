"""The C-ABI library: it loads, exports every symbol include/lookat.h declares, and turns
bad arguments into status codes before touching the GPU.  CPU only (no kernel is launched)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", f) for f in sorted(os.listdir(os.path.join(ROOT, "include")))
           if f.endswith(".h")]


@pytest.fixture(scope="module")
def lib():
    from paper_2601_10155_amd import binding
    if not os.path.exists(binding.lib_path()):
        from paper_2601_10155_amd import build
        build.build(verbose=False)
    return binding.load_library()


def declared_symbols():
    names = set()
    for h in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(lookat_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"lookat_encode_keys", "lookat_build_lut", "lookat_attend_decode", "lookat_kmeans_step",
            "lookat_probe_stream_read", "lookat_score_prefill", "lookat_decode_step",
            "lookat_attend_decode_gqa", "lookat_attend_decode_gqa_workspace_bytes", "lookat_decode_step_split",
            "lookat_decode_step_split_workspace_bytes", "lookat_decode_step_gqa",
            "lookat_decode_step_gqa_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in lookat.h but not exported"


def test_version_and_error_string(lib):
    assert lib.lookat_version() >= 100
    assert isinstance(lib.lookat_last_error(), bytes)


from paper_2601_10155_amd.binding import _Shape as Shape  # noqa: E402  (the struct lookat_shape)


OK, E_NULL, E_SHAPE, E_DTYPE, E_ALIGN, E_WS, E_UNSUP = 0, -1, -2, -3, -4, -5, -6
FAKE = 0x10000  # 16-byte aligned, never dereferenced: validation fails first


def test_encode_argument_errors(lib):
    s = Shape(1, 1, 64, 4, 256)
    f = lib.lookat_encode_keys
    assert f(None, 1, FAKE, 2, FAKE, FAKE, 4, None) == E_NULL
    assert f(ctypes.byref(s), 0, None, 2, None, None, 0, None) == OK          # N = 0: no-op
    assert f(ctypes.byref(s), -1, FAKE, 2, FAKE, FAKE, 4, None) == E_SHAPE
    assert f(ctypes.byref(s), 1, FAKE, 7, FAKE, FAKE, 4, None) == E_DTYPE
    assert f(ctypes.byref(s), 1, None, 2, FAKE, FAKE, 4, None) == E_NULL
    assert f(ctypes.byref(s), 2, FAKE, 2, FAKE, FAKE, 4, None) == E_SHAPE      # stride < N*m
    assert f(ctypes.byref(s), 1, FAKE + 4, 2, FAKE, FAKE, 4, None) == E_ALIGN
    assert b"aligned" in lib.lookat_last_error()
    for bad, code in ((Shape(1, 1, 64, 5, 256), E_SHAPE), (Shape(1, 1, 64, 4, 128), E_SHAPE),
                      (Shape(0, 1, 64, 4, 256), E_SHAPE), (Shape(1, 1, 60, 4, 256), E_UNSUP),
                      (Shape(1, 1, 512, 4, 256), E_UNSUP), (Shape(1, 1, 256, 64, 256), E_UNSUP)):
        assert f(ctypes.byref(bad), 1, FAKE, 2, FAKE, FAKE, 64, None) == code


def test_build_lut_argument_errors(lib):
    s = Shape(2, 3, 64, 4, 256)
    f = lib.lookat_build_lut
    assert f(ctypes.byref(s), 0, FAKE, 1, FAKE, FAKE, None) == E_SHAPE
    assert f(ctypes.byref(s), 1, FAKE, 0, FAKE, FAKE, None) == E_DTYPE
    assert f(ctypes.byref(s), 1, FAKE, 1, None, FAKE, None) == E_NULL
    assert f(ctypes.byref(s), 1, FAKE, 1, FAKE, FAKE + 8, None) == E_ALIGN


def test_attend_decode_argument_errors(lib):
    s = Shape(2, 3, 64, 4, 256)
    f = lib.lookat_attend_decode
    ws = lib.lookat_attend_decode_workspace_bytes
    L = 1000
    args = lambda **kw: [kw.get("shape", ctypes.byref(s)), kw.get("L", L), kw.get("lut", FAKE), kw.get("codes", FAKE),
                         kw.get("cs", L * 4), kw.get("values", FAKE), kw.get("vs", L * 64),
                         ctypes.c_float(0.125), kw.get("splits", 1), kw.get("ws", None), kw.get("wsb", 0),
                         kw.get("out", FAKE), None, None]
    assert f(*args(L=0)) == E_SHAPE
    assert f(*args(splits=-1)) == E_SHAPE
    assert f(*args(lut=None)) == E_NULL
    assert f(*args(cs=L * 4 - 16)) == E_SHAPE
    assert f(*args(cs=L * 4 + 2)) == E_ALIGN
    assert f(*args(vs=L * 64 + 4)) == E_ALIGN
    assert f(*args(codes=FAKE + 2)) == E_ALIGN
    need = ws(ctypes.byref(s), L, 4)
    assert need == 2 * 3 * 4 * (64 + 2) * 4
    assert ws(ctypes.byref(s), L, 1) == 0
    assert f(*args(splits=4)) == E_WS
    assert f(*args(splits=4, ws=FAKE, wsb=need - 1)) == E_WS
    assert b"workspace" in lib.lookat_last_error()
    auto = lib.lookat_attend_decode_auto_splits(ctypes.byref(s), L)
    assert auto >= 1 and ws(ctypes.byref(s), L, 0) == (0 if auto == 1 else 2 * 3 * auto * 66 * 4)


def test_binding_refuses_host_tensors():
    import torch
    from paper_2601_10155_amd import binding
    cb = torch.zeros((1, 4, 256, 16))
    with pytest.raises(ValueError):
        binding.lookat_encode_keys(torch.zeros((1, 1, 4, 64)), cb)


def test_kmeans_and_probe_argument_errors(lib):
    s = Shape(2, 3, 64, 4, 256)
    f = lib.lookat_kmeans_step
    assert f(ctypes.byref(s), 10, FAKE, FAKE, FAKE + 0x1000, FAKE, None) == E_SHAPE      # B must be 1
    s1 = Shape(1, 3, 64, 4, 256)
    assert f(ctypes.byref(s1), 0, FAKE, FAKE, FAKE + 0x1000, FAKE, None) == E_SHAPE
    assert f(ctypes.byref(s1), 10, FAKE, FAKE, FAKE, FAKE, None) == E_SHAPE              # in == out
    assert f(ctypes.byref(s1), 10, None, FAKE, FAKE + 0x1000, FAKE, None) == E_NULL
    p = lib.lookat_probe_stream_read
    assert p(None, 1024, FAKE, None) == E_NULL
    assert p(FAKE, 1000, FAKE, None) == E_SHAPE
    assert p(FAKE + 8, 1024, FAKE, None) == E_ALIGN
    w = lib.lookat_probe_stream_write
    assert w(None, 1024, 0, None) == E_NULL
    assert w(FAKE, 1000, 0, None) == E_SHAPE
    assert w(FAKE + 8, 1024, 0, None) == E_ALIGN


def test_score_prefill_argument_errors(lib):
    s = Shape(2, 3, 128, 16, 256)
    f = lib.lookat_score_prefill
    ok_args = [ctypes.byref(s), 64, 64, FAKE, 1, FAKE, FAKE, 64 * 16, FAKE, None]
    def call(**kw):
        a = list(ok_args)
        for k, v in kw.items():
            a[{"T": 1, "L": 2, "q": 3, "dt": 4, "cb": 5, "codes": 6, "cs": 7, "scores": 8}[k]] = v
        return f(*a)
    assert call(T=0) == E_SHAPE
    assert call(L=63) == E_SHAPE                 # fewer keys than queries
    assert call(dt=9) == E_DTYPE
    assert call(codes=None) == E_NULL
    assert call(cs=64 * 16 - 16) == E_SHAPE
    assert call(q=FAKE + 2) == E_ALIGN
    assert call(codes=FAKE + 8) == E_ALIGN
    assert call(L=(1 << 30) + 64, cs=((1 << 30) + 64) * 16) == E_UNSUP    # rows of scores beyond 32-bit byte offsets
    bad = Shape(2, 3, 96, 4, 256)
    a = list(ok_args); a[0] = ctypes.byref(bad); a[7] = 64 * 4
    assert f(*a) == E_UNSUP


def test_decode_step_argument_errors(lib):
    s = Shape(2, 3, 64, 4, 256)
    f = lib.lookat_decode_step
    L = 100
    base = [ctypes.byref(s), L, FAKE, FAKE, 1, FAKE, FAKE, L * 4, FAKE, L * 64, ctypes.c_float(0.125), FAKE, None]
    def call(**kw):
        a = list(base)
        for k, v in kw.items():
            a[{"L": 1, "q": 2, "k": 3, "dt": 4, "cb": 5, "codes": 6, "cs": 7, "values": 8, "vs": 9, "out": 11}[k]] = v
        return f(*a)
    assert call(L=0) == E_SHAPE
    assert call(dt=3) == E_DTYPE
    assert call(k=None) == E_NULL
    assert call(cs=L * 4 - 4) == E_SHAPE
    assert call(q=FAKE + 4) == E_ALIGN
    assert call(codes=FAKE + 2) == E_ALIGN
    bad = Shape(2, 3, 32, 4, 256)
    a = list(base); a[0] = ctypes.byref(bad); a[9] = L * 32
    assert f(*a) == E_UNSUP


def test_decode_step_entries_per_workgroup(lib):
    """Which fused-step instance a shape resolves to (host only): pairs of batch entries only for even B,
    257..512 (b,h) pairs, and d_k = 64 with m in {2, 4} from 768 keys or d_k = 128 with m = 4 from 512 keys / m = 8
    from 2048 keys."""
    f = lib.lookat_decode_step_entries_per_workgroup
    def n(B, H, d_k, m, L):
        s = Shape(B, H, d_k, m, 256)
        return f(ctypes.byref(s), L)
    assert n(32, 12, 64, 4, 1024) == 2 and n(32, 12, 64, 2, 1024) == 2 and n(22, 12, 64, 4, 768) == 2
    assert n(42, 12, 64, 4, 4096) == 2 and n(16, 32, 64, 4, 1024) == 2
    assert n(20, 12, 64, 4, 1024) == 1      # 240 (b,h): every workgroup has a compute unit to itself
    assert n(44, 12, 64, 4, 1024) == 1      # 528 (b,h): the pairs would need a second round
    assert n(31, 12, 64, 4, 1024) == 1      # odd batch
    assert n(32, 12, 64, 8, 1024) == 1 and n(32, 12, 64, 4, 767) == 1
    assert n(12, 32, 128, 4, 512) == 2 and n(12, 32, 128, 4, 511) == 1          # d_k = 128: m = 4 from 512 keys,
    assert n(12, 32, 128, 8, 2048) == 2 and n(12, 32, 128, 8, 2047) == 1        # m = 8 from 2048,
    assert n(12, 32, 128, 16, 4096) == 1 and n(12, 32, 128, 2, 4096) == 1       # m = 16 and m = 2 never
    assert n(8, 32, 128, 8, 32768) == 1                                         # 256 (b,h): one each
    assert n(32, 12, 32, 4, 1024) == 0 and n(32, 12, 64, 4, 0) == 0 and f(None, 5) == 0


def test_decode_step_split_argument_errors(lib):
    """No call here reaches a launch: every argument list fails a host-side check."""
    s = Shape(1, 4, 128, 8, 256)
    f = lib.lookat_decode_step_split
    ws = lib.lookat_decode_step_split_workspace_bytes
    L = 8192
    assert ws(ctypes.byref(s), L, 1) == 0
    assert ws(ctypes.byref(s), L, 4) == 1 * 4 * 4 * (128 + 2) * 4
    assert ws(ctypes.byref(s), L, 0) == ws(ctypes.byref(s), L, lib.lookat_attend_decode_auto_splits(ctypes.byref(s), L))
    base = [ctypes.byref(s), L, FAKE, FAKE, 1, FAKE, FAKE, L * 8, FAKE, L * 128, ctypes.c_float(0.1), 4, FAKE, 1 << 20,
            FAKE, None]
    def call(**kw):
        a = list(base)
        for k, v in kw.items():
            a[{"L": 1, "q": 2, "dt": 4, "splits": 11, "ws": 12, "wsb": 13, "out": 14}[k]] = v
        return f(*a)
    assert call(L=0) == E_SHAPE
    assert call(dt=7) == E_DTYPE
    assert call(splits=-1) == E_SHAPE
    assert call(ws=None) == E_WS
    assert call(wsb=100) == E_WS
    assert call(ws=FAKE + 4) == E_ALIGN
    assert call(out=None) == E_NULL


def test_decode_step_gqa_argument_errors(lib):
    """No call here reaches a launch: every argument list fails a host-side check."""
    s = Shape(1, 4, 128, 8, 256)      # H = key/value heads
    f = lib.lookat_decode_step_gqa
    ws = lib.lookat_decode_step_gqa_workspace_bytes
    L = 8192
    assert ws(ctypes.byref(s), 4, L, 1) == 0
    assert ws(ctypes.byref(s), 4, L, 3) == 1 * 4 * 4 * 3 * (128 + 2) * 4
    base = [ctypes.byref(s), 4, L, FAKE, FAKE, 1, FAKE, FAKE, L * 8, FAKE, L * 128, ctypes.c_float(0.1), 3, FAKE, 1 << 20,
            FAKE, None]
    def call(**kw):
        a = list(base)
        for k, v in kw.items():
            a[{"group": 1, "L": 2, "q": 3, "dt": 5, "splits": 12, "ws": 13, "wsb": 14, "out": 15}[k]] = v
        return f(*a)
    assert call(group=3) == E_UNSUP
    assert call(L=0) == E_SHAPE
    assert call(dt=0) == E_DTYPE
    assert call(splits=-2) == E_SHAPE
    assert call(ws=None) == E_WS
    assert call(wsb=64) == E_WS
    assert call(q=None) == E_NULL
    assert call(out=FAKE + 8) == E_ALIGN
    big = Shape(1, 4, 128, 16, 256)   # 8 x 16 KB of tables + the reduction buffer do not fit 160 KB of LDS
    a = list(base); a[0] = ctypes.byref(big); a[1] = 8; a[8] = L * 16
    assert f(*a) == E_UNSUP


def test_attend_decode_gqa_argument_errors(lib):
    s = Shape(2, 3, 128, 8, 256)      # H = key/value heads
    f = lib.lookat_attend_decode_gqa
    ws = lib.lookat_attend_decode_gqa_workspace_bytes
    L = 1000
    args = lambda **kw: [kw.get("shape", ctypes.byref(s)), kw.get("group", 4), kw.get("L", L), kw.get("lut", FAKE),
                         kw.get("codes", FAKE), kw.get("cs", L * 8), kw.get("values", FAKE), kw.get("vs", L * 128),
                         ctypes.c_float(0.125), kw.get("splits", 1), kw.get("ws", None), kw.get("wsb", 0),
                         kw.get("out", FAKE), None, None]
    assert f(*args(group=3)) == E_UNSUP
    assert f(*args(group=0)) == E_UNSUP
    assert f(*args(L=0)) == E_SHAPE
    assert f(*args(lut=None)) == E_NULL
    assert f(*args(cs=L * 8 - 8)) == E_SHAPE
    assert f(*args(codes=FAKE + 4)) == E_ALIGN
    assert f(*args(shape=ctypes.byref(Shape(2, 3, 32, 4, 256)))) == E_UNSUP       # d_k outside {64, 128}
    need = ws(ctypes.byref(s), 4, L, 3)
    assert need == 2 * 3 * 4 * 3 * (128 + 2) * 4
    assert ws(ctypes.byref(s), 4, L, 1) == 0
    assert f(*args(splits=3)) == E_WS
    assert f(*args(splits=3, ws=FAKE, wsb=need - 1)) == E_WS
