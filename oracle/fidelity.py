"""Fidelity metrics of LOOKAT attention against dense attention (paper Sec. "Evaluation Metrics"),
on the seeded synthetic caches of lookat_inputs.  Test infrastructure, like the rest of oracle/:
CPU only, numpy fp64, informational (the paper's own figures need GPT-2 caches that are not here).

    python -m oracle.fidelity            # table over m in {2,4,8,16} and L in {64..1024}

Metrics, per (batch, head) row and then averaged:
  cosine      cos(y_dense, y_lookat) of the attention outputs
  kl          KL(A_dense || A_lookat) = sum_l A_dense[l] log(A_dense[l] / A_lookat[l])
  spearman    rank correlation of the two attention distributions (average ranks on ties)
  top5        |Top5(A_dense) n Top5(A_lookat)| / 5
"""
from __future__ import annotations

import math

import numpy as np


def softmax_rows(scores, scale):
    s = np.asarray(scores, dtype=np.float64) * scale
    s = s - s.max(axis=-1, keepdims=True)
    a = np.exp(s)
    return a / a.sum(axis=-1, keepdims=True)


def cosine(y_ref, y_approx):
    y_ref = np.asarray(y_ref, dtype=np.float64)
    y_approx = np.asarray(y_approx, dtype=np.float64)
    num = (y_ref * y_approx).sum(-1)
    den = np.sqrt((y_ref * y_ref).sum(-1)) * np.sqrt((y_approx * y_approx).sum(-1))
    return num / den


def kl_divergence(a_ref, a_approx):
    a_ref = np.asarray(a_ref, dtype=np.float64)
    a_approx = np.asarray(a_approx, dtype=np.float64)
    with np.errstate(divide="ignore", invalid="ignore"):
        t = np.where(a_ref > 0, a_ref * (np.log(a_ref) - np.log(a_approx)), 0.0)
    return t.sum(-1)


def _average_ranks(x):
    """Ranks 1..n along the last axis, ties sharing the mean of their positions."""
    x = np.asarray(x, dtype=np.float64)
    flat = x.reshape(-1, x.shape[-1])
    out = np.empty_like(flat)
    for r, row in enumerate(flat):
        order = np.argsort(row, kind="stable")
        srt = row[order]
        ranks = np.empty(len(row))
        i = 0
        while i < len(row):
            j = i
            while j + 1 < len(row) and srt[j + 1] == srt[i]:
                j += 1
            ranks[order[i:j + 1]] = 0.5 * (i + j) + 1.0
            i = j + 1
        out[r] = ranks
    return out.reshape(x.shape)


def spearman(a_ref, a_approx):
    ra, rb = _average_ranks(a_ref), _average_ranks(a_approx)
    ra = ra - ra.mean(-1, keepdims=True)
    rb = rb - rb.mean(-1, keepdims=True)
    den = np.sqrt((ra * ra).sum(-1) * (rb * rb).sum(-1))
    with np.errstate(divide="ignore", invalid="ignore"):
        return np.where(den > 0, (ra * rb).sum(-1) / den, np.nan)


def topk_overlap(a_ref, a_approx, k=5):
    a_ref = np.asarray(a_ref)
    a_approx = np.asarray(a_approx)
    k = min(k, a_ref.shape[-1])
    ta = np.argsort(-a_ref, axis=-1, kind="stable")[..., :k]
    tb = np.argsort(-a_approx, axis=-1, kind="stable")[..., :k]
    hits = (ta[..., :, None] == tb[..., None, :]).any(-1).sum(-1)
    return hits / float(k)


def metrics(scores_dense, out_dense, scores_lookat, out_lookat, scale):
    """All four metrics, averaged over the leading axes.  scores_* are unscaled q.k (or table sums)."""
    a_d = softmax_rows(scores_dense, scale)
    a_l = softmax_rows(scores_lookat, scale)
    return {
        "cosine": float(np.mean(cosine(out_dense, out_lookat))),
        "kl": float(np.mean(kl_divergence(a_d, a_l))),
        "spearman": float(np.nanmean(spearman(a_d, a_l))),
        "top5": float(np.mean(topk_overlap(a_d, a_l, 5))),
    }


def evaluate(m, L, d_k=64, B=2, H=4, q_gain=1.0, seed=0, kmeans_iters=5, n_calib=2048):
    """One cell of the table: LOOKAT-m against dense attention on a synthetic cache of length L."""
    import lookat_inputs as li
    import oracle

    cfg = li.shrink(li.CONFIGS["C2"], B=B, H=H, L=L, d_k=d_k, m=m, n_calib=n_calib)
    case = li.make_case(cfg, seed=seed)
    cb, _ = oracle.kmeans(case["calib"], case["cb_init"], kmeans_iters)
    q = (case["q"].astype(np.float32) * q_gain).astype(np.float32)
    keys, values = case["keys"].astype(np.float32), case["values"]
    scale = 1.0 / math.sqrt(d_k)
    codes = oracle.encode_keys(keys, cb)
    lut = oracle.build_lut(q, cb)[:, :, 0]
    out_l, s_l = oracle.attend_decode(lut, codes, values, scale, want_scores=True)
    s_d = np.einsum("bhd,bhld->bhl", q[:, :, 0].astype(np.float64), keys.astype(np.float64))
    out_d = oracle.dense_attention(q[:, :, 0], keys, values, scale)
    return metrics(s_d, out_d, s_l, out_l, scale)


def table(ms=(2, 4, 8, 16), Ls=(64, 128, 256, 512, 1024), **kw):
    rows = []
    for m in ms:
        for L in Ls:
            r = evaluate(m, L, **kw)
            rows.append((m, L, r))
    return rows


def main():
    for gain in (1.0, 8.0):
        print(f"# query gain {gain:g} (queries N(0,1)/8 x gain), d_k=64, rank-8 keys + 0.1 noise, 5 Lloyd iterations")
        print("| m | bytes/key | L | cosine | KL | Spearman | top-5 |")
        print("|---|---:|---:|---:|---:|---:|---:|")
        for m, L, r in table(q_gain=gain):
            print(f"| {m} | {m} | {L} | {r['cosine']:.4f} | {r['kl']:.2e} | {r['spearman']:.4f} | {r['top5']:.3f} |")


if __name__ == "__main__":
    main()
