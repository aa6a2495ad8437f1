"""ctypes binding of liblookat.so: torch tensors in, C-ABI calls out.

Marshalling only — shapes, pointers, strides, the current HIP stream.  Every step of
the method runs in the library's kernels.  If the library is missing the calls raise
(the product has no CPU path).
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "liblookat.so")

LOOKAT_F16 = 1
LOOKAT_F32 = 2

_lib = None


class LookatError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"lookat status {status}: {message}")
        self.status = status


class _Shape(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("d_k", ctypes.c_int32),
                ("m", ctypes.c_int32), ("K", ctypes.c_int32)]


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads the built library; raises if it has not been built (python -m paper_2601_10155_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise LookatError(-100, f"{_LIB_PATH} is not built; run `python -m paper_2601_10155_amd.build`")
        lib = ctypes.CDLL(_LIB_PATH)
        i32, i64, vp, sz, f32 = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float
        sp = ctypes.POINTER(_Shape)
        lib.lookat_encode_keys.argtypes = [sp, i64, vp, ctypes.c_int, vp, vp, i64, vp]
        lib.lookat_encode_keys.restype = ctypes.c_int
        lib.lookat_build_lut.argtypes = [sp, i32, vp, ctypes.c_int, vp, vp, vp]
        lib.lookat_build_lut.restype = ctypes.c_int
        lib.lookat_attend_decode_workspace_bytes.argtypes = [sp, i64, i32]
        lib.lookat_attend_decode_workspace_bytes.restype = sz
        lib.lookat_attend_decode_auto_splits.argtypes = [sp, i64]
        lib.lookat_attend_decode_auto_splits.restype = i32
        lib.lookat_attend_decode_launch_shape.argtypes = [sp, i64, i32, ctypes.POINTER(i32), ctypes.POINTER(i32)]
        lib.lookat_attend_decode_launch_shape.restype = ctypes.c_int
        lib.lookat_attend_decode.argtypes = [sp, i64, vp, vp, i64, vp, i64, f32, i32, vp, sz, vp, vp, vp]
        lib.lookat_attend_decode.restype = ctypes.c_int
        lib.lookat_attend_decode_noalloc.argtypes = [sp, i64, vp, vp, i64, vp, i64, f32, i32, vp, vp, vp]
        lib.lookat_attend_decode_noalloc.restype = ctypes.c_int
        lib.lookat_attend_decode_gqa_workspace_bytes.argtypes = [sp, i32, i64, i32]
        lib.lookat_attend_decode_gqa_workspace_bytes.restype = sz
        lib.lookat_attend_decode_gqa.argtypes = [sp, i32, i64, vp, vp, i64, vp, i64, f32, i32, vp, sz, vp, vp, vp]
        lib.lookat_attend_decode_gqa.restype = ctypes.c_int
        lib.lookat_decode_step.argtypes = [sp, i64, vp, vp, ctypes.c_int, vp, vp, i64, vp, i64, f32, vp, vp]
        lib.lookat_decode_step.restype = ctypes.c_int
        lib.lookat_decode_step_entries_per_workgroup.argtypes = [sp, i64]
        lib.lookat_decode_step_entries_per_workgroup.restype = i32
        lib.lookat_probe_decode_step_entries.argtypes = [sp, i32, i64, vp, vp, ctypes.c_int, vp, vp, i64, vp, i64, f32, vp, vp]
        lib.lookat_probe_decode_step_entries.restype = ctypes.c_int
        lib.lookat_decode_step_split_workspace_bytes.argtypes = [sp, i64, i32]
        lib.lookat_decode_step_split_workspace_bytes.restype = sz
        lib.lookat_decode_step_split.argtypes = [sp, i64, vp, vp, ctypes.c_int, vp, vp, i64, vp, i64, f32, i32, vp, sz, vp, vp]
        lib.lookat_decode_step_split.restype = ctypes.c_int
        lib.lookat_decode_step_gqa_workspace_bytes.argtypes = [sp, i32, i64, i32]
        lib.lookat_decode_step_gqa_workspace_bytes.restype = sz
        lib.lookat_decode_step_gqa.argtypes = [sp, i32, i64, vp, vp, ctypes.c_int, vp, vp, i64, vp, i64, f32, i32, vp, sz, vp, vp]
        lib.lookat_decode_step_gqa.restype = ctypes.c_int
        lib.lookat_score_prefill.argtypes = [sp, i32, i64, vp, ctypes.c_int, vp, vp, i64, vp, vp]
        lib.lookat_score_prefill.restype = ctypes.c_int
        lib.lookat_probe_score_prefill_lookup.argtypes = lib.lookat_score_prefill.argtypes
        lib.lookat_probe_score_prefill_lookup.restype = ctypes.c_int
        lib.lookat_kmeans_step.argtypes = [sp, i64, vp, vp, vp, vp, vp]
        lib.lookat_kmeans_step.restype = ctypes.c_int
        lib.lookat_probe_stream_read.argtypes = [vp, sz, vp, vp]
        lib.lookat_probe_stream_read.restype = ctypes.c_int
        lib.lookat_probe_stream_write.argtypes = [vp, sz, ctypes.c_uint32, vp]
        lib.lookat_probe_stream_write.restype = ctypes.c_int
        lib.lookat_probe_stream_read_shaped.argtypes = [vp, sz, vp, i32, i32, i32, i32, i32, vp]
        lib.lookat_probe_stream_read_shaped.restype = ctypes.c_int
        lib.lookat_probe_empty_launch.argtypes = [i32, i32, vp]
        lib.lookat_probe_empty_launch.restype = ctypes.c_int
        lib.lookat_probe_attend_decode_ticket_workspace_bytes.argtypes = [sp, i64, i32]
        lib.lookat_probe_attend_decode_ticket_workspace_bytes.restype = sz
        lib.lookat_probe_attend_decode_ticket.argtypes = [sp, i64, vp, vp, i64, vp, i64, f32, i32, vp, sz, vp, vp,
                                                          ctypes.POINTER(i32), vp]
        lib.lookat_probe_attend_decode_ticket.restype = ctypes.c_int
        lib.lookat_last_error.restype = ctypes.c_char_p
        lib.lookat_version.restype = ctypes.c_int
        _lib = lib
    return _lib


def last_error() -> str:
    return load_library().lookat_last_error().decode()


def version() -> int:
    return int(load_library().lookat_version())


def _check(status: int):
    if status != 0:
        raise LookatError(status, last_error())


def _dtype_tag(t: torch.Tensor) -> int:
    if t.dtype == torch.float16:
        return LOOKAT_F16
    if t.dtype == torch.float32:
        return LOOKAT_F32
    raise TypeError(f"expected float16 or float32 tensor, got {t.dtype}")


def _dev(t: torch.Tensor, name: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    return t


def _stream(t: torch.Tensor) -> int:
    return torch.cuda.current_stream(t.device).cuda_stream


def _bh_stride(t: torch.Tensor, name: str) -> int:
    """Element stride between consecutive (b,h) slabs of a [B,H,L,x] tensor whose slabs are dense."""
    B, H, L, X = t.shape
    if t.stride(3) != 1 or (L > 1 and t.stride(2) != X):
        raise ValueError(f"{name}: each (b,h) slab must be dense [L,{X}]")
    sh = t.stride(1) if H > 1 else max(t.stride(0), L * X)
    if B > 1 and t.stride(0) != H * sh:
        raise ValueError(f"{name}: batch stride must be H times the head stride")
    return sh


def lookat_encode_keys(keys: torch.Tensor, codebooks: torch.Tensor, codes_out: torch.Tensor | None = None,
                       cache: torch.Tensor | None = None, position: int = 0) -> torch.Tensor:
    """keys [B,H,N,d_k] fp16|fp32, codebooks [H,m,256,d_sub] fp32 -> codes [B,H,N,m] uint8.

    With `cache` ([B,H,Lmax,m] uint8) the codes are written in place at rows
    position .. position+N-1 and the cache is returned."""
    lib = load_library()
    keys = _dev(keys, "keys").contiguous()
    cb = _dev(codebooks, "codebooks").contiguous()
    B, H, N, d_k = keys.shape
    Hc, m, K, d_sub = cb.shape
    if Hc != H or m * d_sub != d_k or cb.dtype != torch.float32:
        raise ValueError("codebooks must be fp32 [H,m,K,d_k/m]")
    shape = _Shape(B, H, d_k, m, K)
    if cache is not None:
        if cache.dtype != torch.uint8 or cache.shape[:2] != (B, H) or cache.shape[3] != m:
            raise ValueError("cache must be uint8 [B,H,Lmax,m]")
        if position < 0 or position + N > cache.shape[2]:
            raise ValueError("position + N exceeds the cache length")
        stride = _bh_stride(cache, "cache")
        ptr = cache.data_ptr() + position * m
        ret = cache
    else:
        if codes_out is None:
            codes_out = torch.empty((B, H, N, m), dtype=torch.uint8, device=keys.device)
        if codes_out.dtype != torch.uint8 or tuple(codes_out.shape) != (B, H, N, m) or not codes_out.is_contiguous():
            raise ValueError("codes_out must be a contiguous uint8 [B,H,N,m] tensor")
        stride = N * m
        ptr = codes_out.data_ptr()
        ret = codes_out
    _check(lib.lookat_encode_keys(ctypes.byref(shape), N, keys.data_ptr(), _dtype_tag(keys), cb.data_ptr(),
                                  ptr, stride, _stream(keys)))
    return ret


def lookat_build_lut(q: torch.Tensor, codebooks: torch.Tensor, lut_out: torch.Tensor | None = None) -> torch.Tensor:
    """q [B,H,T,d_k] fp16|fp32 -> lut [B,H,T,m,256] fp32."""
    lib = load_library()
    q = _dev(q, "q").contiguous()
    cb = _dev(codebooks, "codebooks").contiguous()
    B, H, T, d_k = q.shape
    Hc, m, K, d_sub = cb.shape
    if Hc != H or m * d_sub != d_k or cb.dtype != torch.float32:
        raise ValueError("codebooks must be fp32 [H,m,K,d_k/m]")
    shape = _Shape(B, H, d_k, m, K)
    if lut_out is None:
        lut_out = torch.empty((B, H, T, m, K), dtype=torch.float32, device=q.device)
    if lut_out.dtype != torch.float32 or lut_out.numel() != B * H * T * m * K or not lut_out.is_contiguous():
        raise ValueError("lut_out must be a contiguous fp32 tensor of B*H*T*m*K elements")
    _check(lib.lookat_build_lut(ctypes.byref(shape), T, q.data_ptr(), _dtype_tag(q), cb.data_ptr(),
                                lut_out.data_ptr(), _stream(q)))
    return lut_out


def _decode_shape(lut, codes, values):
    B, H, L, m = codes.shape
    d_k = values.shape[3]
    if lut.numel() != B * H * m * 256 or lut.dtype != torch.float32 or not lut.is_contiguous():
        raise ValueError("lut must be contiguous fp32 [B,H,m,256]")
    if codes.dtype != torch.uint8 or values.dtype != torch.float16:
        raise ValueError("codes must be uint8 and values fp16")
    if tuple(values.shape[:3]) != (B, H, L):
        raise ValueError("values must be [B,H,L,d_k] matching codes [B,H,L,m]")
    return _Shape(B, H, d_k, m, 256), L


def attend_decode_workspace_bytes(B: int, H: int, d_k: int, m: int, L: int, num_splits: int = 0) -> int:
    shape = _Shape(B, H, d_k, m, 256)
    return int(load_library().lookat_attend_decode_workspace_bytes(ctypes.byref(shape), L, num_splits))


def attend_decode_gqa_workspace_bytes(B: int, H: int, group: int, d_k: int, m: int, L: int, num_splits: int = 0) -> int:
    """Workspace of lookat_attend_decode_gqa (H = key/value heads; num_splits 0 = the library's choice)."""
    shape = _Shape(B, H, d_k, m, 256)
    return int(load_library().lookat_attend_decode_gqa_workspace_bytes(ctypes.byref(shape), group, L, num_splits))


def attend_decode_auto_splits(B: int, H: int, d_k: int, m: int, L: int) -> int:
    shape = _Shape(B, H, d_k, m, 256)
    return int(load_library().lookat_attend_decode_auto_splits(ctypes.byref(shape), L))


def attend_decode_launch_shape(B: int, H: int, d_k: int, m: int, L: int, num_splits: int = 0) -> tuple[int, int]:
    """(ranges per (b,h), wavefronts per workgroup) of the launch lookat_attend_decode makes for this problem."""
    shape = _Shape(B, H, d_k, m, 256)
    ranges, waves = ctypes.c_int32(0), ctypes.c_int32(0)
    _check(load_library().lookat_attend_decode_launch_shape(ctypes.byref(shape), L, num_splits, ctypes.byref(ranges),
                                                            ctypes.byref(waves)))
    return int(ranges.value), int(waves.value)


def lookat_attend_decode(lut: torch.Tensor, codes: torch.Tensor, values: torch.Tensor, scale: float,
                         num_splits: int = 0, workspace: torch.Tensor | None = None,
                         out: torch.Tensor | None = None, scores_out: torch.Tensor | None = None) -> torch.Tensor:
    """lut [B,H,m,256] fp32, codes [B,H,L,m] u8, values [B,H,L,d_k] fp16 -> out [B,H,d_k] fp32.

    codes / values may be views of longer caches ([B,H,Lmax,*] sliced to L rows)."""
    lib = load_library()
    _dev(lut, "lut"), _dev(codes, "codes"), _dev(values, "values")
    shape, L = _decode_shape(lut, codes, values)
    B, H, d_k = shape.B, shape.H, shape.d_k
    cs = _bh_stride(codes, "codes")
    vs = _bh_stride(values, "values")
    need = int(lib.lookat_attend_decode_workspace_bytes(ctypes.byref(shape), L, num_splits))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=values.device)
    if out is None:
        out = torch.empty((B, H, d_k), dtype=torch.float32, device=values.device)
    if out.dtype != torch.float32 or out.numel() != B * H * d_k or not out.is_contiguous():
        raise ValueError("out must be contiguous fp32 [B,H,d_k]")
    if scores_out is not None and (scores_out.dtype != torch.float32 or scores_out.numel() != B * H * L
                                   or not scores_out.is_contiguous()):
        raise ValueError("scores_out must be contiguous fp32 [B,H,L]")
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.lookat_attend_decode(ctypes.byref(shape), L, lut.data_ptr(), codes.data_ptr(), cs,
                                    values.data_ptr(), vs, float(scale), int(num_splits), ws_ptr, ws_bytes,
                                    out.data_ptr(), scores_out.data_ptr() if scores_out is not None else None,
                                    _stream(values)))
    return out


def lookat_attend_decode_noalloc(lut: torch.Tensor, codes: torch.Tensor, values: torch.Tensor, scale: float,
                                 out: torch.Tensor, num_splits: int = 0,
                                 scores_out: torch.Tensor | None = None) -> torch.Tensor:
    """lookat_attend_decode without a workspace (the library's own scratch memory): for callers that
    cannot allocate.  `out` [B,H,d_k] fp32 must be given; nothing is allocated here or in the library."""
    lib = load_library()
    _dev(lut, "lut"), _dev(codes, "codes"), _dev(values, "values"), _dev(out, "out")
    shape, L = _decode_shape(lut, codes, values)
    if out.dtype != torch.float32 or out.numel() != shape.B * shape.H * shape.d_k or not out.is_contiguous():
        raise ValueError("out must be contiguous fp32 [B,H,d_k]")
    if scores_out is not None and (scores_out.dtype != torch.float32 or scores_out.numel() != shape.B * shape.H * L
                                   or not scores_out.is_contiguous()):
        raise ValueError("scores_out must be contiguous fp32 [B,H,L]")
    _check(lib.lookat_attend_decode_noalloc(ctypes.byref(shape), L, lut.data_ptr(), codes.data_ptr(),
                                            _bh_stride(codes, "codes"), values.data_ptr(), _bh_stride(values, "values"),
                                            float(scale), int(num_splits), out.data_ptr(),
                                            scores_out.data_ptr() if scores_out is not None else None, _stream(values)))
    return out


def lookat_attend_decode_gqa(lut: torch.Tensor, codes: torch.Tensor, values: torch.Tensor, scale: float,
                             num_splits: int = 0, workspace: torch.Tensor | None = None,
                             out: torch.Tensor | None = None, scores_out: torch.Tensor | None = None) -> torch.Tensor:
    """Grouped queries: lut [B,H*g,m,256] fp32, codes [B,H,L,m] u8, values [B,H,L,d_k] fp16
    -> out [B,H*g,d_k] fp32; H counts key/value heads, g = lut.shape[1] // H query heads share each."""
    lib = load_library()
    _dev(lut, "lut"), _dev(codes, "codes"), _dev(values, "values")
    B, H, L, m = codes.shape
    d_k = values.shape[3]
    if lut.dim() != 4 or lut.shape[0] != B or lut.shape[1] % H or tuple(lut.shape[2:]) != (m, 256) \
            or lut.dtype != torch.float32 or not lut.is_contiguous():
        raise ValueError("lut must be contiguous fp32 [B,H*g,m,256]")
    g = lut.shape[1] // H
    if codes.dtype != torch.uint8 or values.dtype != torch.float16 or tuple(values.shape[:3]) != (B, H, L):
        raise ValueError("codes must be uint8 [B,H,L,m] and values fp16 [B,H,L,d_k]")
    shape = _Shape(B, H, d_k, m, 256)
    cs = _bh_stride(codes, "codes")
    vs = _bh_stride(values, "values")
    need = int(lib.lookat_attend_decode_gqa_workspace_bytes(ctypes.byref(shape), g, L, num_splits))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=values.device)
    if out is None:
        out = torch.empty((B, H * g, d_k), dtype=torch.float32, device=values.device)
    if out.dtype != torch.float32 or out.numel() != B * H * g * d_k or not out.is_contiguous():
        raise ValueError("out must be contiguous fp32 [B,H*g,d_k]")
    if scores_out is not None and (scores_out.dtype != torch.float32 or scores_out.numel() != B * H * g * L
                                   or not scores_out.is_contiguous()):
        raise ValueError("scores_out must be contiguous fp32 [B,H*g,L]")
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.lookat_attend_decode_gqa(ctypes.byref(shape), g, L, lut.data_ptr(), codes.data_ptr(), cs,
                                        values.data_ptr(), vs, float(scale), int(num_splits), ws_ptr, ws_bytes,
                                        out.data_ptr(), scores_out.data_ptr() if scores_out is not None else None,
                                        _stream(values)))
    return out


def lookat_decode_step(q: torch.Tensor, k_new: torch.Tensor, codebooks: torch.Tensor, codes: torch.Tensor,
                       values: torch.Tensor, scale: float, out: torch.Tensor | None = None) -> torch.Tensor:
    """Fused decode step.  q, k_new [B,H,d_k] (same dtype), codes [B,H,L,m] u8 (row L-1 is written),
    values [B,H,L,d_k] fp16 (row L-1 already holds the new value) -> out [B,H,d_k] fp32.
    codes / values may be views of longer caches sliced to L rows."""
    return _decode_step(q, k_new, codebooks, codes, values, scale, out, None, None)


def decode_step_entries_per_workgroup(B: int, H: int, d_k: int, m: int, L: int) -> int:
    """Batch entries one workgroup of lookat_decode_step serves for this problem (1 or 2; 0: no kernel)."""
    shape = _Shape(B, H, d_k, m, 256)
    return int(load_library().lookat_decode_step_entries_per_workgroup(ctypes.byref(shape), L))


def lookat_probe_decode_step_entries(entries_per_workgroup: int, q: torch.Tensor, k_new: torch.Tensor,
                                     codebooks: torch.Tensor, codes: torch.Tensor, values: torch.Tensor, scale: float,
                                     out: torch.Tensor | None = None) -> torch.Tensor:
    """lookat_decode_step on the kernel instance that serves `entries_per_workgroup` (1 or 2) batch entries of
    a head per workgroup (2: even B, d_k = 64; measurement aid)."""
    return _decode_step(q, k_new, codebooks, codes, values, scale, out, None, None,
                        _entries=int(entries_per_workgroup))


def lookat_decode_step_split(q: torch.Tensor, k_new: torch.Tensor, codebooks: torch.Tensor, codes: torch.Tensor,
                             values: torch.Tensor, scale: float, num_splits: int = 0,
                             workspace: torch.Tensor | None = None, out: torch.Tensor | None = None) -> torch.Tensor:
    """The fused decode step with every (b,h)'s sequence cut into num_splits ranges (0 = the library's
    choice): for few (b,h) pairs and long contexts.  Arguments as lookat_decode_step."""
    return _decode_step(q, k_new, codebooks, codes, values, scale, out, int(num_splits), workspace)


def lookat_decode_step_gqa(q: torch.Tensor, k_new: torch.Tensor, codebooks: torch.Tensor, codes: torch.Tensor,
                           values: torch.Tensor, scale: float, num_splits: int = 0,
                           workspace: torch.Tensor | None = None, out: torch.Tensor | None = None) -> torch.Tensor:
    """Fused decode step with grouped queries: q [B,H*g,d_k], k_new [B,H,d_k] (same dtype), codebooks
    [H,m,256,d_k/m], codes [B,H,L,m] u8 (row L-1 is written), values [B,H,L,d_k] fp16 -> out [B,H*g,d_k] fp32;
    H counts key/value heads, g = q.shape[1] // H."""
    lib = load_library()
    q = _dev(q, "q").contiguous()
    k_new = _dev(k_new, "k_new").contiguous()
    cb = _dev(codebooks, "codebooks").contiguous()
    _dev(codes, "codes"), _dev(values, "values")
    B, H, L, m = codes.shape
    d_k = values.shape[3]
    if q.dim() != 3 or q.shape[0] != B or q.shape[1] % H or q.shape[2] != d_k or q.dtype != k_new.dtype \
            or k_new.numel() != B * H * d_k:
        raise ValueError("q must be [B,H*g,d_k] and k_new [B,H,d_k], of one dtype")
    g = q.shape[1] // H
    if cb.dtype != torch.float32 or tuple(cb.shape) != (H, m, 256, d_k // m):
        raise ValueError("codebooks must be fp32 [H,m,256,d_k/m]")
    if codes.dtype != torch.uint8 or values.dtype != torch.float16 or tuple(values.shape[:3]) != (B, H, L):
        raise ValueError("codes must be uint8 [B,H,L,m] and values fp16 [B,H,L,d_k]")
    cs = _bh_stride(codes, "codes")
    vs = _bh_stride(values, "values")
    if out is None:
        out = torch.empty((B, H * g, d_k), dtype=torch.float32, device=values.device)
    if out.dtype != torch.float32 or out.numel() != B * H * g * d_k or not out.is_contiguous():
        raise ValueError("out must be contiguous fp32 [B,H*g,d_k]")
    shape = _Shape(B, H, d_k, m, 256)
    need = int(lib.lookat_decode_step_gqa_workspace_bytes(ctypes.byref(shape), g, L, num_splits))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=values.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.lookat_decode_step_gqa(ctypes.byref(shape), g, L, q.data_ptr(), k_new.data_ptr(), _dtype_tag(q),
                                      cb.data_ptr(), codes.data_ptr(), cs, values.data_ptr(), vs, float(scale),
                                      int(num_splits), ws_ptr, ws_bytes, out.data_ptr(), _stream(values)))
    return out


def decode_step_split_workspace_bytes(B: int, H: int, d_k: int, m: int, L: int, num_splits: int = 0) -> int:
    shape = _Shape(B, H, d_k, m, 256)
    return int(load_library().lookat_decode_step_split_workspace_bytes(ctypes.byref(shape), L, num_splits))


def _decode_step(q, k_new, codebooks, codes, values, scale, out, num_splits, workspace, _entries=None):
    lib = load_library()
    q = _dev(q, "q").contiguous()
    k_new = _dev(k_new, "k_new").contiguous()
    cb = _dev(codebooks, "codebooks").contiguous()
    _dev(codes, "codes"), _dev(values, "values")
    B, H, L, m = codes.shape
    d_k = values.shape[3]
    if q.dtype != k_new.dtype or q.numel() != B * H * d_k or k_new.numel() != B * H * d_k:
        raise ValueError("q and k_new must both be [B,H,d_k] of one dtype")
    if cb.dtype != torch.float32 or tuple(cb.shape) != (H, m, 256, d_k // m):
        raise ValueError("codebooks must be fp32 [H,m,256,d_k/m]")
    if codes.dtype != torch.uint8 or values.dtype != torch.float16 or tuple(values.shape[:3]) != (B, H, L):
        raise ValueError("codes must be uint8 [B,H,L,m] and values fp16 [B,H,L,d_k]")
    cs = _bh_stride(codes, "codes")
    vs = _bh_stride(values, "values")
    if out is None:
        out = torch.empty((B, H, d_k), dtype=torch.float32, device=values.device)
    if out.dtype != torch.float32 or out.numel() != B * H * d_k or not out.is_contiguous():
        raise ValueError("out must be contiguous fp32 [B,H,d_k]")
    shape = _Shape(B, H, d_k, m, 256)
    if num_splits is None:
        if _entries is not None:
            _check(lib.lookat_probe_decode_step_entries(ctypes.byref(shape), _entries, L, q.data_ptr(), k_new.data_ptr(),
                                                        _dtype_tag(q), cb.data_ptr(), codes.data_ptr(), cs,
                                                        values.data_ptr(), vs, float(scale), out.data_ptr(),
                                                        _stream(values)))
            return out
        _check(lib.lookat_decode_step(ctypes.byref(shape), L, q.data_ptr(), k_new.data_ptr(), _dtype_tag(q),
                                      cb.data_ptr(), codes.data_ptr(), cs, values.data_ptr(), vs, float(scale),
                                      out.data_ptr(), _stream(values)))
        return out
    need = int(lib.lookat_decode_step_split_workspace_bytes(ctypes.byref(shape), L, num_splits))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty(need, dtype=torch.uint8, device=values.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.lookat_decode_step_split(ctypes.byref(shape), L, q.data_ptr(), k_new.data_ptr(), _dtype_tag(q),
                                        cb.data_ptr(), codes.data_ptr(), cs, values.data_ptr(), vs, float(scale),
                                        num_splits, ws_ptr, ws_bytes, out.data_ptr(), _stream(values)))
    return out


def lookat_score_prefill(q: torch.Tensor, codebooks: torch.Tensor, codes: torch.Tensor,
                         scores_out: torch.Tensor | None = None, _entry: str = "lookat_score_prefill") -> torch.Tensor:
    """q [B,H,T,d_k] fp16|fp32, codes [B,H,L,m] u8 (L >= T) -> causal scores [B,H,T,L] fp32
    (-inf where key l is later than query t's position t + L - T)."""
    lib = load_library()
    q = _dev(q, "q").contiguous()
    cb = _dev(codebooks, "codebooks").contiguous()
    _dev(codes, "codes")
    B, H, T, d_k = q.shape
    Hc, m, K, d_sub = cb.shape
    L = codes.shape[2]
    if Hc != H or m * d_sub != d_k or cb.dtype != torch.float32:
        raise ValueError("codebooks must be fp32 [H,m,K,d_k/m]")
    if codes.dtype != torch.uint8 or codes.shape[:2] != (B, H) or codes.shape[3] != m:
        raise ValueError("codes must be uint8 [B,H,L,m]")
    cs = _bh_stride(codes, "codes")
    if scores_out is None:
        scores_out = torch.empty((B, H, T, L), dtype=torch.float32, device=q.device)
    if scores_out.dtype != torch.float32 or scores_out.numel() != B * H * T * L or not scores_out.is_contiguous():
        raise ValueError("scores_out must be contiguous fp32 [B,H,T,L]")
    shape = _Shape(B, H, d_k, m, K)
    _check(getattr(lib, _entry)(ctypes.byref(shape), T, L, q.data_ptr(), _dtype_tag(q), cb.data_ptr(),
                                codes.data_ptr(), cs, scores_out.data_ptr(), _stream(q)))
    return scores_out


def lookat_probe_score_prefill_lookup(q: torch.Tensor, codebooks: torch.Tensor, codes: torch.Tensor,
                                      scores_out: torch.Tensor | None = None) -> torch.Tensor:
    """lookat_score_prefill forced onto its lookup-and-sum kernel (measurement aid)."""
    return lookat_score_prefill(q, codebooks, codes, scores_out, _entry="lookat_probe_score_prefill_lookup")


def lookat_kmeans_step(calib: torch.Tensor, codebooks: torch.Tensor, codebooks_out: torch.Tensor | None = None,
                       assign_out: torch.Tensor | None = None):
    """One Lloyd iteration. calib [H,Nc,d_k] fp32, codebooks [H,m,256,d_sub] fp32 ->
    (new codebooks, assignment [H,Nc,m] uint8 against the input codebooks)."""
    lib = load_library()
    calib = _dev(calib, "calib").contiguous()
    cb = _dev(codebooks, "codebooks").contiguous()
    H, Nc, d_k = calib.shape
    Hc, m, K, d_sub = cb.shape
    if Hc != H or m * d_sub != d_k or cb.dtype != torch.float32 or calib.dtype != torch.float32:
        raise ValueError("calib must be fp32 [H,Nc,d_k] and codebooks fp32 [H,m,K,d_k/m]")
    if codebooks_out is None:
        codebooks_out = torch.empty_like(cb)
    if assign_out is None:
        assign_out = torch.empty((H, Nc, m), dtype=torch.uint8, device=calib.device)
    shape = _Shape(1, H, d_k, m, K)
    _check(lib.lookat_kmeans_step(ctypes.byref(shape), Nc, calib.data_ptr(), cb.data_ptr(), codebooks_out.data_ptr(),
                                  assign_out.data_ptr(), _stream(calib)))
    return codebooks_out, assign_out


def lookat_kmeans(calib: torch.Tensor, codebooks: torch.Tensor, iters: int) -> torch.Tensor:
    """`iters` Lloyd iterations from the given initial codebooks (ping-pong between two buffers)."""
    cur = codebooks.contiguous().clone()
    nxt = torch.empty_like(cur)
    assign = torch.empty((calib.shape[0], calib.shape[1], cur.shape[1]), dtype=torch.uint8, device=calib.device)
    for _ in range(int(iters)):
        lookat_kmeans_step(calib, cur, nxt, assign)
        cur, nxt = nxt, cur
    return cur


def lookat_probe_stream_read(src: torch.Tensor, sink: torch.Tensor) -> None:
    """Measurement aid: streams all bytes of `src` once through a plain read kernel."""
    lib = load_library()
    _dev(src, "src"), _dev(sink, "sink")
    if not src.is_contiguous():
        raise ValueError("src must be contiguous")
    _check(lib.lookat_probe_stream_read(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(),
                                        _stream(src)))


def lookat_probe_stream_write(dst: torch.Tensor, word: int = 0) -> None:
    """Measurement aid: overwrites all bytes of `dst` once with a 32-bit pattern through a plain write kernel."""
    lib = load_library()
    _dev(dst, "dst")
    if not dst.is_contiguous():
        raise ValueError("dst must be contiguous")
    _check(lib.lookat_probe_stream_write(dst.data_ptr(), dst.numel() * dst.element_size(), int(word) & 0xffffffff,
                                         _stream(dst)))


def lookat_probe_stream_read_shaped(src: torch.Tensor, sink: torch.Tensor, threads: int, loads_per_thread: int,
                                    workgroups: int = 0, contiguous: bool = False, nontemporal: bool = True) -> None:
    """Measurement aid: the read stream in a chosen launch shape (see include/lookat_probe.h)."""
    lib = load_library()
    _dev(src, "src"), _dev(sink, "sink")
    if not src.is_contiguous():
        raise ValueError("src must be contiguous")
    _check(lib.lookat_probe_stream_read_shaped(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(),
                                               int(threads), int(loads_per_thread), int(workgroups), int(bool(contiguous)),
                                               int(bool(nontemporal)), _stream(src)))


def lookat_probe_empty_launch(workgroups: int, threads: int) -> None:
    """Measurement aid: launches a kernel that does nothing on the current stream."""
    _check(load_library().lookat_probe_empty_launch(int(workgroups), int(threads),
                                                    torch.cuda.current_stream().cuda_stream))


def probe_attend_decode_ticket_workspace_bytes(B: int, H: int, d_k: int, m: int, L: int, num_splits: int = 0) -> int:
    shape = _Shape(B, H, d_k, m, 256)
    return int(load_library().lookat_probe_attend_decode_ticket_workspace_bytes(ctypes.byref(shape), L, num_splits))


def lookat_probe_attend_decode_ticket(lut: torch.Tensor, codes: torch.Tensor, values: torch.Tensor, scale: float,
                                      num_splits: int = 0, workspace: torch.Tensor | None = None,
                                      out: torch.Tensor | None = None, scores_out: torch.Tensor | None = None):
    """Measurement aid: lookat_attend_decode on the flat geometry with the in-kernel ticket merge.
    Returns (out, pieces per (b,h)).  A workspace allocated here is zeroed (its ticket counters must be)."""
    lib = load_library()
    _dev(lut, "lut"), _dev(codes, "codes"), _dev(values, "values")
    shape, L = _decode_shape(lut, codes, values)
    B, H, d_k = shape.B, shape.H, shape.d_k
    need = int(lib.lookat_probe_attend_decode_ticket_workspace_bytes(ctypes.byref(shape), L, num_splits))
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.zeros(need, dtype=torch.uint8, device=values.device)
    if out is None:
        out = torch.empty((B, H, d_k), dtype=torch.float32, device=values.device)
    pieces = ctypes.c_int32(0)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.lookat_probe_attend_decode_ticket(ctypes.byref(shape), L, lut.data_ptr(), codes.data_ptr(),
                                                 _bh_stride(codes, "codes"), values.data_ptr(), _bh_stride(values, "values"),
                                                 float(scale), int(num_splits), ws_ptr, ws_bytes, out.data_ptr(),
                                                 scores_out.data_ptr() if scores_out is not None else None,
                                                 ctypes.byref(pieces), _stream(values)))
    return out, int(pieces.value)


# short aliases
encode_keys = lookat_encode_keys
build_lut = lookat_build_lut
attend_decode = lookat_attend_decode
