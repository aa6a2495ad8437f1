"""lookat_attend_decode_noalloc (the entry point for callers that cannot allocate: its per-range partial
results live in the library's own device memory) against lookat_attend_decode, through the C ABI, on two
calls in a row, the second on a smaller problem, and against the oracle at the bars of tests/bars.py."""
import ctypes
import math

import numpy as np
import pytest
import torch

import oracle
from bars import assert_out_close, assert_scores_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lk():
    import paper_2601_10155_amd as pkg
    pkg.load_library()
    return pkg


def _case(seed, B, H, L, d_k, m):
    rng = np.random.default_rng(seed)
    lut = (rng.standard_normal((B, H, m, 256)) * 6.0).astype(np.float32)
    codes = rng.integers(0, 256, size=(B, H, L, m), dtype=np.uint8)
    v = rng.standard_normal((B, H, L, d_k)).astype(np.float16)
    return lut, codes, v


def _both(lk, lut, codes, v, scale, splits):
    """One call of each entry point on the same device arrays; returns (noalloc out, scores, workspace-call out)."""
    d = lambda a: torch.from_numpy(a).cuda()
    lut_d, codes_d, v_d = d(lut), d(codes), d(v)
    B, H, L, _ = codes.shape
    out = torch.full((B, H, v.shape[3]), float("nan"), dtype=torch.float32, device="cuda")
    scores = torch.empty((B, H, L), dtype=torch.float32, device="cuda")
    lk.lookat_attend_decode_noalloc(lut_d, codes_d, v_d, scale, out, num_splits=splits, scores_out=scores)
    ref = lk.lookat_attend_decode(lut_d, codes_d, v_d, scale, num_splits=splits)
    torch.cuda.synchronize()
    return out.cpu().numpy(), scores.cpu().numpy(), ref.cpu().numpy()


@pytest.mark.parametrize("d_k,m", [(64, 4), (128, 8)])
def test_noalloc_equals_workspace_call_twice_in_a_row(lk, d_k, m):
    scale = 1.0 / math.sqrt(d_k)
    # first call: 7 ranges over a ragged context; second call: fewer (b,h) pairs, shorter context, 3 ranges
    # (its partial results land on memory the first call left full); third: one range (no scratch memory used)
    for seed, (B, H, L, splits) in enumerate([(3, 5, 2500, 7), (2, 3, 700, 3), (1, 2, 333, 1), (2, 9, 5000, 0)]):
        lut, codes, v = _case(40 + seed + d_k, B, H, L, d_k, m)
        out, scores, ws_out = _both(lk, lut, codes, v, scale, splits)
        ref, s_ref = oracle.attend_decode(lut, codes, v, scale, want_scores=True)
        assert np.array_equal(out, ws_out), f"call {seed}: differs from lookat_attend_decode by {np.abs(out - ws_out).max()}"
        assert_out_close(out, ref, "attend_decode_noalloc", s_ref, scale)
        assert_scores_close(scores, lut, codes, s_ref)


def test_noalloc_rejects_what_does_not_fit(lk):
    """More partial results than the library's scratch memory holds: an error, nothing enqueued."""
    from paper_2601_10155_amd.binding import _Shape, load_library
    lib = load_library()
    shape = _Shape(64, 64, 128, 8, 256)                    # 4096 (b,h) x 16 ranges x 130 floats = 34 MB
    fake = ctypes.c_void_p(0x10000)
    rc = lib.lookat_attend_decode_noalloc(ctypes.byref(shape), 65536, fake, fake, 65536 * 8, fake, 65536 * 128, 0.1, 16,
                                          fake, None, None)
    assert rc == -5 and b"scratch" in lib.lookat_last_error()
    assert lib.lookat_attend_decode_workspace_bytes(ctypes.byref(shape), 65536, 16) > 4 * 1024 * 1024
