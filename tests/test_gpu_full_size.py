"""Parity at the full sizes of the workload configurations, in the launch configuration bench.py
times (automatic split count, fused step where bench.py uses it).  Inputs are drawn in HBM with
the seeded device generator; the oracle recomputes SAMPLED (b,h) slabs, copied back to the host,
with the same bars as tests/test_gpu_parity.py (codes bit-exact, outputs abs <= 2e-3, scores
within 1e-4 of the summand magnitude)."""
import math

import numpy as np
import pytest
import torch

import lookat_inputs as li
import oracle

pytestmark = pytest.mark.gpu

OUT_ATOL = 2e-3
REL = 1e-4


@pytest.fixture(scope="module")
def lk():
    import paper_2601_10155_amd as pkg
    pkg.load_library()
    return pkg


def _slab(t, b, h):
    """Host copy of one (b,h) slab with the two leading axes kept (shape [1,1,...])."""
    return t[b:b + 1, h:h + 1].contiguous().cpu().numpy()


def _sample_bh(cfg, n, seed):
    rng = np.random.default_rng(seed)
    picks = {(0, 0), (cfg.B - 1, cfg.H - 1)}
    while len(picks) < n:
        picks.add((int(rng.integers(cfg.B)), int(rng.integers(cfg.H))))
    return sorted(picks)


def _lut_close(lut_gpu, q, cb, lut_ref):
    """|gpu - oracle| <= 1e-4 * sum_j |q_j c_j| per table entry."""
    B, H, T, d_k = q.shape
    _, m, K, d_sub = cb.shape
    qa = np.abs(q.astype(np.float64)).reshape(B, H, T, m, d_sub)
    mag = np.einsum("bhtij,hicj->bhtic", qa, np.abs(cb.astype(np.float64)))
    err = np.abs(lut_gpu.astype(np.float64) - lut_ref.astype(np.float64))
    assert np.all(err <= REL * np.maximum(mag, 1e-6)), f"max table err {err.max()}"


def _check_decode_slabs(cfg, case, cb, codes, lut, out, scale, picks):
    cbn = cb.cpu().numpy()
    for b, h in picks:
        keys = _slab(case["keys"], b, h)
        codes_ref = oracle.encode_keys(keys, cbn[h:h + 1])
        assert np.array_equal(_slab(codes, b, h), codes_ref), f"codes of slab {(b, h)}"
        lut_ref = oracle.build_lut(_slab(case["q"], b, h), cbn[h:h + 1])
        _lut_close(_slab(lut, b, h).reshape(lut_ref.shape), _slab(case["q"], b, h), cbn[h:h + 1], lut_ref)
        out_ref = oracle.attend_decode(lut_ref[:, :, 0], codes_ref, _slab(case["values"], b, h), scale)
        err = np.max(np.abs(_slab(out, b, h) - out_ref))
        assert err <= OUT_ATOL, f"slab {(b, h)}: {err}"


def test_config_c2_full_size_fused_step_and_three_calls(lk):
    """GPT-2-small shape, batch 32, context 1024, m=4: one layer at full size, both paths."""
    cfg = li.CONFIGS["C2"]
    case = li.torch_case(cfg, "cuda", layer=0)
    cb = lk.lookat_kmeans(case["calib"], case["cb_init"], 3)
    scale = 1.0 / math.sqrt(cfg.d_k)
    codes = lk.lookat_encode_keys(case["keys"], cb)
    lut = lk.lookat_build_lut(case["q"], cb)
    assert lk.attend_decode_auto_splits(cfg.B, cfg.H, cfg.d_k, cfg.m, cfg.L) == 1
    out = lk.lookat_attend_decode(lut.view(cfg.B, cfg.H, cfg.m, 256), codes, case["values"], scale)
    picks = _sample_bh(cfg, 6, 1)
    _check_decode_slabs(cfg, case, cb, codes, lut, out, scale, picks)
    # the fused step on a cache whose last row is stale must land on the same codes and outputs
    cache = codes.clone()
    cache[:, :, -1] = 0xEE
    out1 = lk.lookat_decode_step(case["q"][:, :, 0].float(), case["keys"][:, :, -1].contiguous(), cb, cache,
                                 case["values"], scale)
    assert torch.equal(cache, codes)
    assert float((out1 - out).abs().max()) <= 1e-5


def test_config_c1_full_size(lk):
    """GPT-2-small shape, batch 1, m=2 (64x key compression)."""
    cfg = li.CONFIGS["C1"]
    case = li.torch_case(cfg, "cuda", layer=3)
    cb = lk.lookat_kmeans(case["calib"], case["cb_init"], 3)
    scale = 1.0 / math.sqrt(cfg.d_k)
    codes = lk.lookat_encode_keys(case["keys"], cb)
    lut = lk.lookat_build_lut(case["q"], cb)
    out = lk.lookat_attend_decode(lut.view(cfg.B, cfg.H, cfg.m, 256), codes, case["values"], scale)
    _check_decode_slabs(cfg, case, cb, codes, lut, out, scale, _sample_bh(cfg, 4, 2))


def test_config_c3_full_size_long_context(lk):
    """Llama shape: 32 heads, d_k=128, m=8, batch 8, context 32768 (2.2 GB of codes + values): the
    automatic split count (one range: 256 (b,h) pairs fill the chip) and two ranges per (b,h) merged by the
    second kernel."""
    cfg = li.CONFIGS["C3"]
    case = li.torch_case(li.shrink(cfg, n_calib=2048), "cuda", layer=0)   # calibration set cut: set-up time only
    cb = lk.lookat_kmeans(case["calib"], case["cb_init"], 1)
    scale = 1.0 / math.sqrt(cfg.d_k)
    codes = lk.lookat_encode_keys(case["keys"], cb)
    lut = lk.lookat_build_lut(case["q"], cb)
    assert lk.attend_decode_auto_splits(cfg.B, cfg.H, cfg.d_k, cfg.m, cfg.L) == 1
    out = lk.lookat_attend_decode(lut.view(cfg.B, cfg.H, cfg.m, 256), codes, case["values"], scale)
    assert torch.isfinite(out).all()
    out2 = lk.lookat_attend_decode(lut.view(cfg.B, cfg.H, cfg.m, 256), codes, case["values"], scale, num_splits=2)
    assert float((out2 - out).abs().max()) <= 1e-5
    picks = _sample_bh(cfg, 3, 3)
    cbn = cb.cpu().numpy()
    for b, h in picks:
        # codes: the oracle encodes a sample of 4096 keys of the slab (275 GMAC for all of them)
        keys = _slab(case["keys"], b, h)
        idx = np.sort(np.random.default_rng(b * 100 + h).choice(cfg.L, 4096, replace=False))
        codes_ref = oracle.encode_keys(keys[:, :, idx], cbn[h:h + 1])
        got_codes = _slab(codes, b, h)
        assert np.array_equal(got_codes[:, :, idx], codes_ref)
        # attention over the whole slab, from the GPU's (sample-checked) codes
        lut_ref = oracle.build_lut(_slab(case["q"], b, h), cbn[h:h + 1])
        out_ref = oracle.attend_decode(lut_ref[:, :, 0], got_codes, _slab(case["values"], b, h), scale)
        assert np.max(np.abs(_slab(out, b, h) - out_ref)) <= OUT_ATOL
    # the fused step (what bench.py times at this shape: B*H = 256 workgroups, one range each) on a cache
    # whose last row is stale lands on the same codes and, up to the order of the partial sums, outputs
    cache = codes.clone()
    cache[:, :, -1] = 0xEE
    out1 = lk.lookat_decode_step(case["q"][:, :, 0].to(case["keys"].dtype).contiguous(),
                                 case["keys"][:, :, -1].contiguous(), cb, cache, case["values"], scale)
    assert torch.equal(cache, codes)
    assert float((out1 - out).abs().max()) <= 1e-5


def test_config_c3_full_size_grouped_queries(lk):
    """The long-context shape with 4 query heads per key/value head (32 query heads, 8 key/value heads),
    in the launch configuration `bench.py --workload C3 --group 4` times: sampled (b, key/value head)
    slabs, every query head of the group against the oracle, scores included."""
    g = 4
    cfg = li.CONFIGS["C3"]
    kv = li.shrink(cfg, H=cfg.H // g, n_calib=2048)
    case = li.torch_case(kv, "cuda", layer=1)
    cb = lk.lookat_kmeans(case["calib"], case["cb_init"], 1)
    scale = 1.0 / math.sqrt(cfg.d_k)
    codes = lk.lookat_encode_keys(case["keys"], cb)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(li.BASE_SEED + 4242)
    q = (torch.randn((cfg.B, cfg.H, 1, cfg.d_k), generator=gen, device="cuda") / 8).to(case["q"].dtype)
    lut = lk.lookat_build_lut(q, cb.repeat_interleave(g, dim=0).contiguous())
    scores = torch.empty((cfg.B, cfg.H, cfg.L), dtype=torch.float32, device="cuda")
    out = lk.lookat_attend_decode_gqa(lut.view(cfg.B, cfg.H, cfg.m, 256), codes, case["values"], scale,
                                      scores_out=scores)
    assert torch.isfinite(out).all()
    cbn = cb.cpu().numpy()
    for b, h in _sample_bh(kv, 3, 5):
        got_codes = _slab(codes, b, h)
        qs = q[b:b + 1, h * g:(h + 1) * g].contiguous().cpu().numpy()                    # [1,g,1,d_k]
        lut_ref = oracle.build_lut(qs, np.repeat(cbn[h:h + 1], g, axis=0))[:, :, 0]        # [1,g,m,256]
        out_ref, s_ref = oracle.attend_decode_gqa(lut_ref, got_codes, _slab(case["values"], b, h), scale,
                                                  want_scores=True)
        assert np.max(np.abs(out[b:b + 1, h * g:(h + 1) * g].cpu().numpy() - out_ref)) <= OUT_ATOL
        # |score error| <= 1e-4 of the summands' magnitude (sum over subspaces of the table entries picked)
        idx = got_codes[0, 0].astype(np.int64)                                             # [L,m]
        mag = np.abs(lut_ref[0])[:, np.arange(cfg.m)[None, :], idx].sum(-1)                # [g,L]
        err = np.abs(scores[b, h * g:(h + 1) * g].cpu().numpy().astype(np.float64) - s_ref[0])
        assert np.all(err <= REL * np.maximum(mag, 1e-6)), f"slab {(b, h)}: {err.max()}"


def test_config_c4_full_size_prefill(lk):
    """Prefill block: 32 heads, d_k=128, m=16, batch 4, 2048 fp16 keys and 2048 causal queries per head."""
    cfg = li.CONFIGS["C4"]
    case = li.torch_case(cfg, "cuda", layer=0)
    cb = lk.lookat_kmeans(case["calib"], case["cb_init"], 1)
    codes = lk.lookat_encode_keys(case["keys"], cb)
    scores = lk.lookat_score_prefill(case["q"], cb, codes)
    cbn = cb.cpu().numpy()
    for b, h in _sample_bh(cfg, 2, 4):
        keys = _slab(case["keys"], b, h)
        codes_ref = oracle.encode_keys(keys, cbn[h:h + 1])
        assert np.array_equal(_slab(codes, b, h), codes_ref)
        lut_ref = oracle.build_lut(_slab(case["q"], b, h), cbn[h:h + 1])          # [1,1,T,m,K]
        ref = oracle.score_prefill(lut_ref, codes_ref)
        got = _slab(scores, b, h)
        vis = np.isfinite(ref)
        assert np.array_equal(np.isneginf(got), ~vis)
        # summand magnitude sum_i sum_j |q_j| |C_i[c_i]_j| per (t, l): the tables are built in the kernel
        d_sub = cfg.d_k // cfg.m
        qa = np.abs(_slab(case["q"], b, h).astype(np.float64)).reshape(cfg.T, cfg.m, d_sub)
        picked = np.stack([np.abs(cbn[h, i].astype(np.float64))[codes_ref[0, 0, :, i].astype(np.int64)]
                           for i in range(cfg.m)], axis=1)                           # [L, m, d_sub]
        mag = np.einsum("tid,lid->tl", qa, picked)[None, None]
        err = np.abs(np.where(vis, got, 0.0) - np.where(vis, ref, 0.0))
        assert np.all(err <= REL * np.maximum(mag, 1e-6)), f"max err {err.max()}"
        # the materialised tables of the same queries (matrix-core path) agree with the oracle's
        lut_gpu = lk.lookat_build_lut(case["q"][b:b + 1, h:h + 1].contiguous(), cb[h:h + 1].contiguous())
        _lut_close(lut_gpu.cpu().numpy(), _slab(case["q"], b, h), cbn[h:h + 1], lut_ref)
