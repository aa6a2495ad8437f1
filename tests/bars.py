"""Parity bars shared by the GPU tests, and a record of the largest errors seen (printed at the end
of the run by conftest.py).

  * codes: bit-exact;
  * table entries and scores: |gpu - oracle| <= REL * (sum of the magnitudes of the summed terms);
  * outputs: |gpu - oracle| <= OUT_ATOL absolute (the contract: fp16 values, fp32 accumulation), and a
    second, tighter bar OUT_TIGHT that follows from the kernel's arithmetic: a weight is
    2^(x - max) with x = fl(fl(s) * scale*log2(e)), so its relative error is at most about
    2*X*2^-24*ln 2 + 2^-23 (two roundings at magnitude X = max |x|, one ulp of the hardware exponential);
    the output moves by at most that times the weighted mean of |v - o| (about 1 for N(0,1) values):
    2.6e-6 at X = 30.  fp32 accumulation of L terms adds about sqrt(L)*2^-24*|o|.  OUT_TIGHT = 2e-5 leaves
    a factor of 8 over that estimate for X <= 64 and scales with X beyond.  Unlike OUT_ATOL it is small
    enough to see one lost 64-key tile in a 16K-key context, or one lost key that carries weight.
"""
import numpy as np

OUT_ATOL = 2e-3
OUT_TIGHT = 2e-5
REL = 1e-4
LOG2E = 1.4426950408889634

observed = {}   # label -> largest |gpu - oracle| seen under that label


def record(label, value):
    value = float(value)
    if value > observed.get(label, -1.0):
        observed[label] = value


def assert_out_close(out, ref, label, scores=None, scale=None):
    """out, ref: arrays of one shape.  scores (unscaled, oracle's) and scale, when given, set X."""
    out = np.asarray(out, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert out.shape == ref.shape
    assert np.isfinite(out).all(), f"{label}: non-finite output"
    err = float(np.max(np.abs(out - ref))) if out.size else 0.0
    x = 0.0 if scores is None else float(np.max(np.abs(np.asarray(scores, dtype=np.float64)))) * abs(scale) * LOG2E
    tight = OUT_TIGHT * max(1.0, x / 64.0)
    record(label, err)
    print(f"[parity] {label}: max |gpu - oracle| = {err:.3e} (bars {tight:.1e} / {OUT_ATOL:.0e})")
    assert err <= OUT_ATOL, f"{label}: {err} > contract bar {OUT_ATOL}"
    assert err <= tight, f"{label}: {err} > arithmetic bar {tight}"
    return err


def assert_scores_close(s_gpu, lut, codes, s_ref, label="scores"):
    """lut [B,H,m,K], codes [B,H,L,m]: tolerance relative to sum_i |lut[i][c_i]|."""
    B, H, L, m = codes.shape
    mag = np.zeros((B, H, L))
    for i in range(m):
        mag += np.abs(np.take_along_axis(lut[:, :, i, :].astype(np.float64), codes[..., i].astype(np.int64), axis=-1))
    err = np.abs(s_gpu.astype(np.float64) - s_ref.astype(np.float64))
    record(label + " (relative to the summands)", float(np.max(err / np.maximum(mag, 1e-6))) if err.size else 0.0)
    assert np.all(err <= REL * np.maximum(mag, 1e-6)), f"max score err {err.max()}"


def assert_lut_close(lut_gpu, q, cb, lut_ref):
    """q [B,H,T,d_k], cb [H,m,K,d_sub], lut [B,H,T,m,K]: tolerance relative to sum_j |q_j c_j|."""
    B, H, T, d_k = q.shape
    _, m, K, d_sub = cb.shape
    qa = np.abs(q.astype(np.float64)).reshape(B, H, T, m, d_sub)
    mag = np.einsum("bhtij,hicj->bhtic", qa, np.abs(cb.astype(np.float64)))
    err = np.abs(lut_gpu.astype(np.float64) - lut_ref.astype(np.float64))
    record("table entries (relative to the summands)", float(np.max(err / np.maximum(mag, 1e-6))))
    assert np.all(err <= REL * np.maximum(mag, 1e-6)), f"max lut err {err.max()}"
