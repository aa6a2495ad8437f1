"""CPU oracle for LOOKAT — TEST INFRASTRUCTURE, NOT THE PRODUCT.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It wraps ``lookat_oracle.c`` (plain C,
fp64, one loop per step of the paper's method) with numpy-array marshalling and
adds nothing to its arithmetic.  It imports nothing from the HIP package.

Paper passages followed: Sec. 3.4 (prototype learning, encoding), Sec. 3.5
(lookup tables, lookup-and-sum), Algorithm 1 (softmax and weighted value sum).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lookat_oracle.c")
_LIB = os.path.join(_HERE, "liblookat_oracle.so")

F16 = 1
F32 = 2

_lib = None


def build(force: bool = False) -> str:
    """Compile lookat_oracle.c with gcc into liblookat_oracle.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32, i64, vp, dbl = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.c_double
        lib.oracle_encode_keys.argtypes = [i32, i32, i64, i32, i32, i32, vp, i32, vp, vp]
        lib.oracle_build_lut.argtypes = [i32, i32, i32, i32, i32, i32, vp, i32, vp, vp]
        lib.oracle_adc_scores.argtypes = [i32, i32, i64, i32, i32, vp, vp, vp]
        lib.oracle_attend_decode.argtypes = [i32, i32, i64, i32, i32, i32, vp, vp, vp, dbl, vp, vp, vp]
        lib.oracle_attend_decode_gqa.argtypes = [i32, i32, i32, i64, i32, i32, i32, vp, vp, vp, dbl, vp, vp]
        lib.oracle_score_prefill.argtypes = [i32, i32, i32, i64, i32, i32, vp, vp, vp]
        lib.oracle_decode_codes.argtypes = [i32, i32, i64, i32, i32, i32, vp, vp, vp]
        lib.oracle_dense_attention.argtypes = [i32, i32, i64, i32, vp, i32, vp, vp, dbl, vp]
        lib.oracle_kmeans_step.argtypes = [i32, i64, i32, i32, i32, vp, vp, vp, vp]
        lib.oracle_set_num_threads.argtypes = [i32]
        lib.oracle_set_num_threads.restype = None
        lib.oracle_num_threads.restype = i32
        _lib = lib
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _float_input(a):
    """fp16 arrays are passed as raw bit patterns, everything else as fp32."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return a, F16
    if a.dtype != np.float32:
        raise TypeError(f"expected float16 or float32, got {a.dtype}")
    return a, F32


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with status {rc}")


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(int(n))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def encode_keys(keys, codebooks):
    """keys [B,H,N,d_k] fp16|fp32, codebooks [H,m,K,d_sub] fp32 -> codes [B,H,N,m] u8."""
    keys, kd = _float_input(keys)
    cb = np.ascontiguousarray(codebooks, dtype=np.float32)
    B, H, N, d_k = keys.shape
    Hc, m, K, d_sub = cb.shape
    assert Hc == H and m * d_sub == d_k
    codes = np.empty((B, H, N, m), dtype=np.uint8)
    _check(_load().oracle_encode_keys(B, H, N, d_k, m, K, _ptr(keys), kd, _ptr(cb), _ptr(codes)), "encode_keys")
    return codes


def build_lut(q, codebooks):
    """q [B,H,T,d_k] fp16|fp32 -> lut [B,H,T,m,K] fp32."""
    q, qd = _float_input(q)
    cb = np.ascontiguousarray(codebooks, dtype=np.float32)
    B, H, T, d_k = q.shape
    Hc, m, K, d_sub = cb.shape
    assert Hc == H and m * d_sub == d_k
    lut = np.empty((B, H, T, m, K), dtype=np.float32)
    _check(_load().oracle_build_lut(B, H, T, d_k, m, K, _ptr(q), qd, _ptr(cb), _ptr(lut)), "build_lut")
    return lut


def adc_scores(lut, codes):
    """lut [B,H,m,K] fp32, codes [B,H,L,m] u8 -> scores [B,H,L] fp32 (unscaled)."""
    lut = np.ascontiguousarray(lut, dtype=np.float32)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    B, H, m, K = lut.shape
    L = codes.shape[2]
    assert codes.shape == (B, H, L, m)
    s = np.empty((B, H, L), dtype=np.float32)
    _check(_load().oracle_adc_scores(B, H, L, m, K, _ptr(lut), _ptr(codes), _ptr(s)), "adc_scores")
    return s


def attend_decode(lut, codes, values, scale, want_scores=False, want_alpha=False):
    """Algorithm 1 after the table build.  Returns out [B,H,d_k] fp32, plus the
    unscaled scores [B,H,L] fp32 and/or the softmax weights [B,H,L] fp64 on request."""
    lut = np.ascontiguousarray(lut, dtype=np.float32)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    values = np.ascontiguousarray(values)
    assert values.dtype == np.float16
    B, H, m, K = lut.shape
    L, d_k = values.shape[2], values.shape[3]
    assert codes.shape == (B, H, L, m) and values.shape[:2] == (B, H)
    out = np.empty((B, H, d_k), dtype=np.float32)
    s = np.empty((B, H, L), dtype=np.float32) if want_scores else None
    a = np.empty((B, H, L), dtype=np.float64) if want_alpha else None
    _check(_load().oracle_attend_decode(B, H, L, d_k, m, K, _ptr(lut), _ptr(codes), _ptr(values),
                                        float(scale), _ptr(out), _ptr(s), _ptr(a)), "attend_decode")
    res = [out]
    if want_scores:
        res.append(s)
    if want_alpha:
        res.append(a)
    return res[0] if len(res) == 1 else tuple(res)


def attend_decode_gqa(lut, codes, values, scale, want_scores=False):
    """Grouped queries: lut [B,H*g,m,K], codes [B,H,L,m], values [B,H,L,d_k] fp16 -> out [B,H*g,d_k]
    fp32 (and the unscaled scores [B,H*g,L]); query head hq reads key/value head hq // g."""
    lut = np.ascontiguousarray(lut, dtype=np.float32)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    values = np.ascontiguousarray(values)
    assert values.dtype == np.float16
    B, HQ, m, K = lut.shape
    H, L, d_k = values.shape[1], values.shape[2], values.shape[3]
    assert HQ % H == 0 and codes.shape == (B, H, L, m) and values.shape[0] == B
    g = HQ // H
    out = np.empty((B, HQ, d_k), dtype=np.float32)
    s = np.empty((B, HQ, L), dtype=np.float32) if want_scores else None
    _check(_load().oracle_attend_decode_gqa(B, H, g, L, d_k, m, K, _ptr(lut), _ptr(codes), _ptr(values),
                                            float(scale), _ptr(out), _ptr(s)), "attend_decode_gqa")
    return (out, s) if want_scores else out


def score_prefill(lut, codes):
    """lut [B,H,T,m,K], codes [B,H,L,m], L >= T -> causal scores [B,H,T,L] fp32; the queries are
    the last T positions, entries with l > t + (L - T) are -inf."""
    lut = np.ascontiguousarray(lut, dtype=np.float32)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    B, H, T, m, K = lut.shape
    L = codes.shape[2]
    s = np.empty((B, H, T, L), dtype=np.float32)
    _check(_load().oracle_score_prefill(B, H, T, L, m, K, _ptr(lut), _ptr(codes), _ptr(s)), "score_prefill")
    return s


def decode_codes(codes, codebooks):
    """codes [B,H,N,m] -> reconstructed keys [B,H,N,d_k] fp32 (pins only)."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    cb = np.ascontiguousarray(codebooks, dtype=np.float32)
    B, H, N, m = codes.shape
    _, _, K, d_sub = cb.shape
    out = np.empty((B, H, N, m * d_sub), dtype=np.float32)
    _check(_load().oracle_decode_codes(B, H, N, m * d_sub, m, K, _ptr(codes), _ptr(cb), _ptr(out)), "decode_codes")
    return out


def dense_attention(q, keys, values, scale):
    """Textbook attention for one query per (b,h): q [B,H,d_k], keys [B,H,L,d_k] fp32,
    values fp16 -> out [B,H,d_k] fp32 (pins only)."""
    q, qd = _float_input(q)
    keys = np.ascontiguousarray(keys, dtype=np.float32)
    values = np.ascontiguousarray(values)
    assert values.dtype == np.float16
    B, H, L, d_k = keys.shape
    out = np.empty((B, H, d_k), dtype=np.float32)
    _check(_load().oracle_dense_attention(B, H, L, d_k, _ptr(q), qd, _ptr(keys), _ptr(values),
                                          float(scale), _ptr(out)), "dense_attention")
    return out


def kmeans_step(calib, codebooks):
    """One Lloyd iteration. calib [H,Nc,d_k] fp32, codebooks [H,m,K,d_sub] fp32 ->
    (new codebooks, objective [H,m] fp64 of the input codebooks)."""
    calib = np.ascontiguousarray(calib, dtype=np.float32)
    cb = np.ascontiguousarray(codebooks, dtype=np.float32)
    H, Nc, d_k = calib.shape
    Hc, m, K, d_sub = cb.shape
    assert Hc == H and m * d_sub == d_k
    out = np.empty_like(cb)
    obj = np.empty((H, m), dtype=np.float64)
    _check(_load().oracle_kmeans_step(H, Nc, d_k, m, K, _ptr(calib), _ptr(cb), _ptr(out), _ptr(obj)), "kmeans_step")
    return out, obj


def kmeans(calib, init_codebooks, iters):
    """`iters` Lloyd iterations from the given initial codebooks.
    Returns (codebooks, objectives [iters,H,m])."""
    cb = np.ascontiguousarray(init_codebooks, dtype=np.float32)
    objs = []
    for _ in range(int(iters)):
        cb, obj = kmeans_step(calib, cb)
        objs.append(obj)
    return cb, np.stack(objs) if objs else np.zeros((0,) + cb.shape[:2])
