"""The fidelity metrics of oracle/fidelity.py (paper Sec. "Evaluation Metrics") against closed
forms and scipy; and, on the GPU, that the HIP path's scores and outputs give the same metric
values as the oracle's."""
import math

import numpy as np
import pytest
import scipy.stats

import lookat_inputs as li
import oracle
from oracle import fidelity as fd


def test_cosine_closed_forms():
    assert fd.cosine([1.0, 0.0], [0.0, 2.0]) == 0.0
    assert abs(fd.cosine([1.0, 2.0, 3.0], [2.0, 4.0, 6.0]) - 1.0) < 1e-15
    assert abs(fd.cosine([1.0, 0.0], [1.0, 1.0]) - 1 / math.sqrt(2)) < 1e-15
    assert abs(fd.cosine([1.0, 2.0], [-1.0, -2.0]) + 1.0) < 1e-15


def test_kl_closed_forms():
    p = np.array([0.5, 0.5])
    q = np.array([0.25, 0.75])
    assert abs(fd.kl_divergence(p, q) - (0.5 * math.log(2) + 0.5 * math.log(2 / 3))) < 1e-15
    assert fd.kl_divergence(q, q) == 0.0
    assert fd.kl_divergence(np.array([1.0, 0.0]), q) == pytest.approx(math.log(4))   # 0 log 0 = 0
    rng = np.random.default_rng(0)
    a = rng.random((7, 33))
    a /= a.sum(-1, keepdims=True)
    b = rng.random((7, 33))
    b /= b.sum(-1, keepdims=True)
    assert np.allclose(fd.kl_divergence(a, b), [scipy.stats.entropy(x, y) for x, y in zip(a, b)], rtol=1e-12)


def test_spearman_against_scipy_with_ties():
    rng = np.random.default_rng(1)
    a = rng.integers(0, 6, size=(9, 40)).astype(float)      # many ties
    b = rng.standard_normal((9, 40))
    got = fd.spearman(a, b)
    ref = [scipy.stats.spearmanr(x, y).statistic for x, y in zip(a, b)]
    assert np.allclose(got, ref, atol=1e-12)
    x = rng.standard_normal(50)
    assert fd.spearman(x, np.exp(x)) == pytest.approx(1.0)   # any increasing map keeps the ranks
    assert fd.spearman(x, -x) == pytest.approx(-1.0)


def test_topk_overlap():
    a = np.array([9.0, 8, 7, 6, 5, 1, 2, 3, 4, 0])
    assert fd.topk_overlap(a, a) == 1.0
    b = a.copy()
    b[0], b[9] = 0.0, 9.0                                    # one of the top five replaced
    assert fd.topk_overlap(a, b) == 0.8
    assert fd.topk_overlap(a, -a) == 0.0
    assert fd.topk_overlap(np.array([3.0, 1, 2]), np.array([1.0, 3, 2])) == 1.0   # fewer than five entries


def test_zero_distortion_gives_perfect_metrics():
    """256 keys that are their own centroids: LOOKAT is exact, so every metric is at its ideal."""
    rng = np.random.default_rng(2)
    B, H, L, d_k, m = 1, 2, 256, 16, 4
    d_sub = d_k // m
    keys = rng.standard_normal((B, H, L, d_k)).astype(np.float32)
    cb = np.stack([np.stack([keys[0, h, :, i * d_sub:(i + 1) * d_sub] for i in range(m)]) for h in range(H)])
    v = rng.standard_normal((B, H, L, d_k)).astype(np.float16)
    q = rng.standard_normal((B, H, 1, d_k)).astype(np.float32)
    scale = 1 / math.sqrt(d_k)
    lut = oracle.build_lut(q, cb)[:, :, 0]
    out_l, s_l = oracle.attend_decode(lut, oracle.encode_keys(keys, cb), v, scale, want_scores=True)
    s_d = np.einsum("bhd,bhld->bhl", q[:, :, 0].astype(np.float64), keys.astype(np.float64))
    r = fd.metrics(s_d, oracle.dense_attention(q[:, :, 0], keys, v, scale), s_l, out_l, scale)
    assert r["cosine"] > 1 - 1e-9 and r["kl"] < 1e-9 and r["spearman"] > 1 - 1e-9 and r["top5"] == 1.0


def test_table_cell_is_sane():
    r = fd.evaluate(m=4, L=128, B=1, H=2, n_calib=512, kmeans_iters=2)
    assert 0.5 < r["cosine"] <= 1.0 and r["kl"] >= 0.0 and -1.0 <= r["spearman"] <= 1.0 and 0.0 <= r["top5"] <= 1.0


@pytest.mark.gpu
def test_gpu_path_gives_the_oracles_fidelity():
    import torch

    import paper_2601_10155_amd as lk
    cfg = li.shrink(li.CONFIGS["C2"], B=2, H=4, L=700, n_calib=1024)
    case = li.make_case(cfg, seed=11)
    scale = 1 / math.sqrt(cfg.d_k)
    q = (case["q"].astype(np.float32) * 8).astype(np.float32)
    keys, v = case["keys"].astype(np.float32), case["values"]
    cb, _ = oracle.kmeans(case["calib"], case["cb_init"], 2)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    codes = lk.lookat_encode_keys(dev(keys), dev(cb))
    lut = lk.lookat_build_lut(dev(q), dev(cb))
    s_gpu = torch.empty((cfg.B, cfg.H, cfg.L), dtype=torch.float32, device="cuda")
    out_gpu = lk.lookat_attend_decode(lut.view(cfg.B, cfg.H, cfg.m, 256), codes, dev(v), scale, scores_out=s_gpu)
    lut_ref = oracle.build_lut(q, cb)[:, :, 0]
    out_ref, s_ref = oracle.attend_decode(lut_ref, oracle.encode_keys(keys, cb), v, scale, want_scores=True)
    s_d = np.einsum("bhd,bhld->bhl", q[:, :, 0].astype(np.float64), keys.astype(np.float64))
    out_d = oracle.dense_attention(q[:, :, 0], keys, v, scale)
    a = fd.metrics(s_d, out_d, s_gpu.cpu().numpy(), out_gpu.cpu().numpy(), scale)
    b = fd.metrics(s_d, out_d, s_ref, out_ref, scale)
    assert abs(a["cosine"] - b["cosine"]) < 1e-6 and abs(a["kl"] - b["kl"]) < 1e-6
    assert abs(a["spearman"] - b["spearman"]) < 1e-4 and abs(a["top5"] - b["top5"]) <= 0.2 / (cfg.B * cfg.H)
