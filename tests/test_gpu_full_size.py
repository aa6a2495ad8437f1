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
from bars import OUT_ATOL, REL, assert_out_close, record

pytestmark = pytest.mark.gpu


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
        record(f"{cfg.name} full size, three calls", err)
        assert err <= OUT_ATOL, f"slab {(b, h)}: {err}"


def _plant_aligned(cfg, case, cb, seed):
    """The inputs of the fused step with the appended key planted on a far centroid and the query pointing at
    it (see tests/test_gpu_parity.py, fused decode step): centroid 255 of every subspace := u_h (+-8 per
    coordinate), k_new := u_h, q := beta * u_h with beta from the size of the context.  Returns (cb, k_new, q)
    as device tensors; `case["keys"]` row L-1 is overwritten so that the cache can be re-encoded."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    u = (torch.randint(0, 2, (cfg.H, cfg.d_k), generator=gen, device="cuda").float() * 16 - 8)
    cb = cb.clone()
    cb[:, :, 255] = u.view(cfg.H, cfg.m, cfg.d_k // cfg.m)
    kd = case["keys"].dtype
    case["keys"][:, :, -1] = u[None].to(kd)
    scale = 1.0 / math.sqrt(cfg.d_k)
    beta = math.log(cfg.L / 0.33) / (scale * 64.0 * cfg.d_k)      # row L-1 leads every other key by about |u|^2
    q = (beta * u)[None].expand(cfg.B, cfg.H, cfg.d_k).to(kd).contiguous()
    k_new = case["keys"][:, :, -1].contiguous()
    return cb, k_new, q


def _check_step_slabs(cfg, case, cb, cache, q, k_new, out, scale, picks, label, aligned=False):
    """The fused step's outputs on sampled (b,h) slabs against the oracle's three steps.  `cache` is the code
    cache after the step; its rows 0..L-2 were checked against the oracle elsewhere (or are checked by the
    caller), row L-1 is checked here."""
    cbn = cb.cpu().numpy()
    for b, h in picks:
        codes_slab = _slab(cache, b, h)
        new_ref = oracle.encode_keys(_slab(k_new[:, :, None], b, h), cbn[h:h + 1])
        assert np.array_equal(codes_slab[:, :, -1:], new_ref), f"appended code row of slab {(b, h)}"
        lut_ref = oracle.build_lut(_slab(q[:, :, None], b, h), cbn[h:h + 1])[:, :, 0]
        out_ref, s_ref, alpha = oracle.attend_decode(lut_ref, codes_slab, _slab(case["values"], b, h), scale,
                                                     want_scores=True, want_alpha=True)
        if aligned:
            assert 0.5 < alpha[0, 0, -1] < 0.99, f"weight of the appended key {alpha[0, 0, -1]}"
        assert_out_close(_slab(out, b, h), out_ref, label, s_ref, scale)


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
    q1, k1 = case["q"][:, :, 0].float(), case["keys"][:, :, -1].contiguous()
    # at this size the library serves two batch entries of a head per workgroup ...
    assert lk.decode_step_entries_per_workgroup(cfg.B, cfg.H, cfg.d_k, cfg.m, cfg.L) == 2
    out1 = lk.lookat_decode_step(q1, k1, cb, cache, case["values"], scale)
    assert torch.equal(cache, codes)
    assert float((out1 - out).abs().max()) <= 1e-5
    _check_step_slabs(cfg, case, cb, cache, q1, k1, out1, scale, picks, "C2 full size, fused step, recipe queries")
    # ... and on the first 20 batch entries (240 (b,h)) one: the same arithmetic per (b,h), so the same bits
    assert lk.decode_step_entries_per_workgroup(20, cfg.H, cfg.d_k, cfg.m, cfg.L) == 1
    cache[:20, :, -1] = 0xEE
    out20 = lk.lookat_decode_step(q1[:20].contiguous(), k1[:20].contiguous(), cb, cache[:20], case["values"][:20], scale)
    assert torch.equal(cache, codes)
    assert torch.equal(out20, out1[:20])
    # a peaked softmax (queries times 8), then the appended key carrying most of the weight
    cache[:, :, -1] = 0xEE
    out8 = lk.lookat_decode_step(q1 * 8, k1, cb, cache, case["values"], scale)
    assert torch.equal(cache, codes)
    _check_step_slabs(cfg, case, cb, cache, q1 * 8, k1, out8, scale, picks, "C2 full size, fused step, peaked queries")
    cb_a, k_a, q_a = _plant_aligned(cfg, case, cb, 77)
    codes_a = lk.lookat_encode_keys(case["keys"], cb_a)
    cache = codes_a.clone()
    cache[:, :, -1] = 0xEE
    out_a = lk.lookat_decode_step(q_a, k_a, cb_a, cache, case["values"], scale)
    assert torch.equal(cache, codes_a)
    cbn = cb_a.cpu().numpy()
    for b, h in picks:   # the re-encoded cache of the sampled slabs against the oracle
        assert np.array_equal(_slab(codes_a, b, h), oracle.encode_keys(_slab(case["keys"], b, h), cbn[h:h + 1]))
    _check_step_slabs(cfg, case, cb_a, cache, q_a, k_a, out_a, scale, picks, "C2 full size, fused step, aligned key",
                      aligned=True)


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
    assert lk.attend_decode_launch_shape(cfg.B, cfg.H, cfg.d_k, cfg.m, cfg.L, 0) == (1, 16)
    scores = torch.empty((cfg.B, cfg.H, cfg.L), dtype=torch.float32, device="cuda")
    out = lk.lookat_attend_decode(lut.view(cfg.B, cfg.H, cfg.m, 256), codes, case["values"], scale, scores_out=scores)
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
        out_ref, s_ref = oracle.attend_decode(lut_ref[:, :, 0], got_codes, _slab(case["values"], b, h), scale,
                                              want_scores=True)
        assert np.max(np.abs(_slab(out, b, h) - out_ref)) <= OUT_ATOL
        # both sides from ONE table (the GPU's, within 1e-4 of the oracle's by the check in _lut_close):
        # scores element by element and the output at the arithmetic bar, for the 16-wavefront instance
        lut_gpu = _slab(lut, b, h)[:, :, 0]
        _lut_close(_slab(lut, b, h), _slab(case["q"], b, h), cbn[h:h + 1], lut_ref)
        o_ref, sc_ref = oracle.attend_decode(lut_gpu, got_codes, _slab(case["values"], b, h), scale, want_scores=True)
        assert_out_close(_slab(out, b, h), o_ref, "C3 full size, attend_decode (16-wavefront instance)", sc_ref, scale)
        mag = np.abs(lut_gpu[0, 0])[np.arange(cfg.m)[None, :], got_codes[0, 0].astype(np.int64)].sum(-1)
        err = np.abs(scores[b, h].cpu().numpy().astype(np.float64) - sc_ref[0, 0])
        assert np.all(err <= REL * np.maximum(mag, 1e-6)), f"slab {(b, h)}: score err {err.max()}"
    # the fused step (what bench.py times at this shape: B*H = 256 workgroups, one range each) on a cache
    # whose last row is stale lands on the same codes and, up to the order of the partial sums, outputs
    cache = codes.clone()
    cache[:, :, -1] = 0xEE
    q1, k1 = case["q"][:, :, 0].to(case["keys"].dtype).contiguous(), case["keys"][:, :, -1].contiguous()
    out1 = lk.lookat_decode_step(q1, k1, cb, cache, case["values"], scale)
    assert torch.equal(cache, codes)
    assert float((out1 - out).abs().max()) <= 1e-5
    # peaked softmax, then the appended key carrying most of the weight, at the arithmetic bar
    cache[:, :, -1] = 0xEE
    out8 = lk.lookat_decode_step(q1 * 8, k1, cb, cache, case["values"], scale)
    assert torch.equal(cache, codes)
    _check_step_slabs(cfg, case, cb, cache, q1 * 8, k1, out8, scale, picks, "C3 full size, fused step, peaked queries")
    cb_a, k_a, q_a = _plant_aligned(cfg, case, cb, 78)
    cache[:, :, -1] = 0xEE          # (rows 0..L-2 keep the codes of the unplanted codebook: a valid cache all the same)
    out_a = lk.lookat_decode_step(q_a, k_a, cb_a, cache, case["values"], scale)
    _check_step_slabs(cfg, case, cb_a, cache, q_a, k_a, out_a, scale, picks, "C3 full size, fused step, aligned key",
                      aligned=True)


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
    # both scoring kernels at the full size: the library's choice for this shape (T >= 24: the
    # dense product against the keys' centroids on the matrix cores) and the lookup-and-sum kernel, forced
    scores = lk.lookat_score_prefill(case["q"], cb, codes)
    scores_lookup = lk.lookat_probe_score_prefill_lookup(case["q"], cb, codes)
    cbn = cb.cpu().numpy()
    for b, h in _sample_bh(cfg, 2, 4):
        keys = _slab(case["keys"], b, h)
        codes_ref = oracle.encode_keys(keys, cbn[h:h + 1])
        assert np.array_equal(_slab(codes, b, h), codes_ref)
        lut_ref = oracle.build_lut(_slab(case["q"], b, h), cbn[h:h + 1])          # [1,1,T,m,K]
        ref = oracle.score_prefill(lut_ref, codes_ref)
        vis = np.isfinite(ref)
        # summand magnitude sum_i sum_j |q_j| |C_i[c_i]_j| per (t, l): the tables are built in the kernel
        d_sub = cfg.d_k // cfg.m
        qa = np.abs(_slab(case["q"], b, h).astype(np.float64)).reshape(cfg.T, cfg.m, d_sub)
        picked = np.stack([np.abs(cbn[h, i].astype(np.float64))[codes_ref[0, 0, :, i].astype(np.int64)]
                           for i in range(cfg.m)], axis=1)                           # [L, m, d_sub]
        mag = np.einsum("tid,lid->tl", qa, picked)[None, None]
        for name, sc in (("library choice", scores), ("lookup-and-sum kernel", scores_lookup)):
            got = _slab(sc, b, h)
            assert np.array_equal(np.isneginf(got), ~vis), name
            err = np.abs(np.where(vis, got, 0.0) - np.where(vis, ref, 0.0))
            assert np.all(err <= REL * np.maximum(mag, 1e-6)), f"{name}: max err {err.max()}"
        # the materialised tables of the same queries (matrix-core path) agree with the oracle's
        lut_gpu = lk.lookat_build_lut(case["q"][b:b + 1, h:h + 1].contiguous(), cb[h:h + 1].contiguous())
        _lut_close(lut_gpu.cpu().numpy(), _slab(case["q"], b, h), cbn[h:h + 1], lut_ref)


@pytest.mark.parametrize("B,H,L,d_k,m,qk", [(12, 32, 1024, 128, 4, torch.float16), (10, 32, 2048, 128, 8, torch.float32),
                                            (22, 12, 768, 64, 2, torch.float16), (42, 12, 1024, 64, 4, torch.float32)])
def test_decode_step_where_the_library_pairs_batch_entries(lk, B, H, L, d_k, m, qk):
    """Shapes at which lookat_decode_step itself serves two batch entries of a head per workgroup (257..512
    (b,h)), other than C2: the whole launch bit-identical to the one-entry instance, sampled (b,h) against
    the oracle's three steps (queries scaled so that the softmax is peaked: a wrong code row would show)."""
    assert lk.decode_step_entries_per_workgroup(B, H, d_k, m, L) == 2
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4100 + B + L + m)
    cb = torch.randn((H, m, 256, d_k // m), generator=gen, device="cuda") * 0.5
    cache = torch.randint(0, 256, (B, H, L, m), generator=gen, device="cuda", dtype=torch.uint8)
    values = torch.randn((B, H, L, d_k), generator=gen, device="cuda").half()
    q = (torch.randn((B, H, d_k), generator=gen, device="cuda") * 1.5).to(qk)
    k_new = (torch.randn((B, H, d_k), generator=gen, device="cuda") * 0.5).to(qk)
    scale = 1.0 / math.sqrt(d_k)
    cache[:, :, -1] = 0xEE
    c2 = cache.clone()
    out = lk.lookat_decode_step(q, k_new, cb, cache, values, scale)
    out1 = lk.lookat_probe_decode_step_entries(1, q, k_new, cb, c2, values, scale)
    assert torch.equal(cache, c2) and torch.equal(out, out1)
    cbn = cb.cpu().numpy()
    rng = np.random.default_rng(B * 100 + H)
    picks = {(0, 0), (1, 0), (B - 1, H - 1), (B - 2, H - 1)} | {(int(rng.integers(B)), int(rng.integers(H))) for _ in range(4)}
    for b, h in sorted(picks):
        codes_slab = _slab(cache, b, h)
        new_ref = oracle.encode_keys(_slab(k_new[:, :, None], b, h), cbn[h:h + 1])
        assert np.array_equal(codes_slab[:, :, -1:], new_ref), f"appended code row of slab {(b, h)}"
        lut_ref = oracle.build_lut(_slab(q[:, :, None], b, h), cbn[h:h + 1])[:, :, 0]
        out_ref, s_ref = oracle.attend_decode(lut_ref, codes_slab, _slab(values, b, h), scale, want_scores=True)
        assert_out_close(_slab(out, b, h), out_ref, "fused step where the library pairs batch entries", s_ref, scale)
