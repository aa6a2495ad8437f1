"""Pins for the CPU oracle: what the paper and the mathematics fix, checked with
code that does not call the oracle routine under test (numpy broadcasts, closed
forms, hand-worked values).  CPU only."""
import math
import os

import numpy as np
import pytest

import lookat_inputs as li
import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _rand_case(rng, B=2, H=3, L=37, d_k=8, m=2, K=256, key_dtype=np.float32, q_dtype=np.float32):
    d_sub = d_k // m
    cb = rng.standard_normal((H, m, K, d_sub)).astype(np.float32)
    keys = rng.standard_normal((B, H, L, d_k)).astype(key_dtype)
    q = (rng.standard_normal((B, H, 1, d_k)) / 2).astype(q_dtype)
    v = rng.standard_normal((B, H, L, d_k)).astype(np.float16)
    return cb, keys, q, v


def _np_decode(codes, cb):
    """codes [B,H,N,m], cb [H,m,K,d_sub] -> [B,H,N,d_k] by fancy indexing."""
    B, H, N, m = codes.shape
    parts = []
    for i in range(m):
        sel = np.stack([cb[h, i][codes[:, h, :, i]] for h in range(H)], axis=1)  # [B,H,N,d_sub]
        parts.append(sel)
    return np.concatenate(parts, axis=-1)


def _np_softmax_attend(scores, v, scale):
    s = scores.astype(np.float64) * scale
    s = s - s.max(axis=-1, keepdims=True)
    a = np.exp(s)
    a /= a.sum(axis=-1, keepdims=True)
    return np.einsum("bhl,bhld->bhd", a, v.astype(np.float64)), a


# ---- fp16 input path ---------------------------------------------------------

def test_half_conversion_all_finite_patterns():
    """Every finite fp16 bit pattern must widen exactly: LUT of a 1-d codebook {1.0} is q itself."""
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16)
    fin = np.isfinite(h)
    q = h[fin].reshape(1, 1, -1, 1)
    cb = np.ones((1, 1, 1, 1), dtype=np.float32)
    lut = oracle.build_lut(q, cb)
    assert np.array_equal(lut.reshape(-1), q.reshape(-1).astype(np.float32))


# ---- P1: ADC identity (Sec. 3.5: LUT definition + lookup-and-sum) ----------------

@pytest.mark.parametrize("d_k,m,K", [(8, 2, 256), (8, 4, 5), (12, 3, 16), (64, 4, 256), (6, 1, 7), (16, 16, 256)])
@pytest.mark.parametrize("q_dtype", [np.float32, np.float16])
def test_adc_identity(d_k, m, K, q_dtype):
    rng = np.random.default_rng(11 + d_k + m + K)
    cb, keys, q, v = _rand_case(rng, d_k=d_k, m=m, K=K, q_dtype=q_dtype)
    B, H, L, _ = keys.shape
    codes = rng.integers(0, K, size=(B, H, L, m), dtype=np.uint8)
    lut = oracle.build_lut(q, cb)[:, :, 0]
    s = oracle.adc_scores(lut, codes).astype(np.float64)
    khat = _np_decode(codes, cb).astype(np.float64)
    ref = np.einsum("bhd,bhld->bhl", q[:, :, 0].astype(np.float64), khat)
    mag = np.einsum("bhd,bhld->bhl", np.abs(q[:, :, 0].astype(np.float64)), np.abs(khat))
    # the table is rounded to fp32 once per entry, the score once more
    assert np.all(np.abs(s - ref) <= 2.0 ** -22 * mag + 1e-30)
    # the oracle's own decode helper agrees with the numpy gather bit for bit
    assert np.array_equal(oracle.decode_codes(codes, cb), khat.astype(np.float32))


def test_lut_matches_numpy_einsum():
    rng = np.random.default_rng(5)
    cb, _, _, _ = _rand_case(rng, d_k=64, m=4)
    q = (rng.standard_normal((2, 3, 5, 64)) / 8).astype(np.float16)
    lut = oracle.build_lut(q, cb)
    qs = q.astype(np.float64).reshape(2, 3, 5, 4, 16)
    ref = np.einsum("bhtij,hicj->bhtic", qs, cb.astype(np.float64))
    assert lut.shape == (2, 3, 5, 4, 256)
    assert np.allclose(lut, ref, rtol=0, atol=2.0 ** -23 * np.abs(ref).max())
    # a transposed codebook or a shifted subspace slice would break the exact cases below
    e = np.zeros((1, 3, 1, 64), dtype=np.float32)
    e[..., 17] = 1.0   # unit query on coordinate 17 = subspace 1, local coordinate 1
    lut1 = oracle.build_lut(e, cb)[0, :, 0]
    assert np.array_equal(lut1[:, 1, :], cb[:, 1, :, 1])
    assert not lut1[:, 0].any() and not lut1[:, 2:].any()


# ---- P2: zero-distortion special case reduces to textbook attention (config C0) ----

def test_c0_zero_distortion_equals_dense_attention():
    cfg = li.CONFIGS["C0"]
    case = li.make_case(cfg, calib_is_cache=True)
    keys, v, q = case["keys"], case["values"], case["q"]
    # N = K = 256 and the codebooks start as the 256 keys themselves
    cb, objs = oracle.kmeans(case["calib"], case["cb_init"], 10)
    assert np.all(objs == 0.0)                      # every key is its own centroid
    assert np.array_equal(cb, case["cb_init"])      # singleton clusters never move
    codes = oracle.encode_keys(keys, cb)
    for i in range(cfg.m):
        assert sorted(codes[0, 0, :, i].tolist()) == list(range(256))
    assert np.array_equal(_np_decode(codes, cb), keys)
    scale = 1.0 / math.sqrt(cfg.d_k)
    lut = oracle.build_lut(q, cb)[:, :, 0]
    out, alpha = oracle.attend_decode(lut, codes, v, scale, want_alpha=True)
    s = np.einsum("bhd,bhld->bhl", q[:, :, 0].astype(np.float64), keys.astype(np.float64))
    ref, a_ref = _np_softmax_attend(s, v, scale)
    assert np.max(np.abs(out - ref)) <= 1e-6
    assert np.max(np.abs(alpha - a_ref)) <= 1e-7
    # the oracle's dense helper is the same textbook routine
    dense = oracle.dense_attention(q[:, :, 0], keys, v, scale)
    assert np.max(np.abs(dense - ref)) <= 1e-6


def test_scale_is_applied_inside_softmax():
    """Dropping the 1/sqrt(d_k) factor, or applying it after exp, must be visible."""
    rng = np.random.default_rng(3)
    lut = rng.standard_normal((1, 1, 2, 256)).astype(np.float32) * 3
    codes = rng.integers(0, 256, size=(1, 1, 50, 2), dtype=np.uint8)
    v = rng.standard_normal((1, 1, 50, 8)).astype(np.float16)
    s = lut[0, 0, 0][codes[0, 0, :, 0]].astype(np.float64) + lut[0, 0, 1][codes[0, 0, :, 1]].astype(np.float64)
    for scale in (1.0, 0.125, 0.37):
        ref, _ = _np_softmax_attend(s[None, None], v, scale)
        out = oracle.attend_decode(lut, codes, v, scale)
        assert np.max(np.abs(out - ref)) <= 1e-6
    a = oracle.attend_decode(lut, codes, v, 1.0)
    b = oracle.attend_decode(lut, codes, v, 0.125)
    assert np.max(np.abs(a - b)) > 1e-2


# ---- P3: argmin by brute force ---------------------------------------------------

@pytest.mark.parametrize("key_dtype", [np.float32, np.float16])
@pytest.mark.parametrize("d_k,m,K", [(8, 2, 256), (64, 4, 256), (16, 16, 256), (12, 3, 9)])
def test_encode_matches_numpy_bruteforce(d_k, m, K, key_dtype):
    rng = np.random.default_rng(100 + d_k + m)
    cb, keys, _, _ = _rand_case(rng, B=2, H=2, L=300, d_k=d_k, m=m, K=K, key_dtype=key_dtype)
    codes = oracle.encode_keys(keys, cb)
    d_sub = d_k // m
    x = keys.astype(np.float64).reshape(2, 2, 300, m, d_sub)
    n_checked = 0
    for h in range(2):
        for i in range(m):
            d = ((x[:, h, :, i, None, :] - cb[h, i].astype(np.float64)[None, None]) ** 2).sum(-1)  # [B,L,K]
            srt = np.sort(d, axis=-1)
            safe = (srt[..., 1] - srt[..., 0]) > 1e-9 * d_sub
            ref = d.argmin(-1)
            got = codes[:, h, :, i]
            assert np.array_equal(got[safe], ref[safe])
            n_checked += int(safe.sum())
    assert n_checked > 0.99 * codes.size


# ---- P4: ties -> lowest index ------------------------------------------------------

def test_encode_ties_lowest_index():
    d_sub, K = 4, 256
    rng = np.random.default_rng(9)
    cb = (rng.standard_normal((1, 1, K, d_sub)) * 10 + 100).astype(np.float32)
    cb[0, 0, 5] = 0.0
    cb[0, 0, 9] = 0.0          # duplicate of centroid 5
    cb[0, 0, 200] = 2.0        # key 1.0 is exactly midway between 0 and 2 on all coordinates
    keys = np.zeros((1, 1, 3, d_sub), dtype=np.float32)
    keys[0, 0, 0] = 0.0        # equal distance 0 to centroids 5 and 9
    keys[0, 0, 1] = 1.0        # equal distance d_sub to 5, 9 and 200
    keys[0, 0, 2] = 1.5        # strictly nearer to 200
    codes = oracle.encode_keys(keys, cb)
    assert codes.reshape(-1).tolist() == [5, 5, 200]
    same = np.full((1, 1, K, d_sub), 3.25, dtype=np.float32)
    assert oracle.encode_keys(keys, same).reshape(-1).tolist() == [0, 0, 0]
    # ties decided per subspace, independently
    cb2 = np.concatenate([cb, cb[:, :, ::-1]], axis=1)      # subspace 1 has the order reversed
    keys2 = np.concatenate([keys, keys], axis=-1)
    codes2 = oracle.encode_keys(keys2, cb2)
    assert codes2[0, 0, :, 0].tolist() == [5, 5, 200]
    assert codes2[0, 0, :, 1].tolist() == [255 - 9, 255 - 200, 255 - 200]


def test_encode_nan_never_wins():
    cb = np.zeros((1, 1, 4, 2), dtype=np.float32)
    cb[0, 0, 0] = np.nan
    cb[0, 0, 1] = 5.0
    cb[0, 0, 2] = 1.0
    cb[0, 0, 3] = 1.0
    keys = np.ones((1, 1, 1, 2), dtype=np.float32)
    # NaN at index 0 is the scan's starting value and no later distance compares below it
    assert oracle.encode_keys(keys, cb).item() == 0
    cb[0, 0, 0] = 7.0
    cb[0, 0, 1] = np.nan
    assert oracle.encode_keys(keys, cb).item() == 2


# ---- P5 / P6: softmax and convex combination ------------------------------------------

def test_softmax_rows_and_convex_hull():
    rng = np.random.default_rng(21)
    B, H, L, d_k, m = 2, 2, 333, 16, 4
    lut = (rng.standard_normal((B, H, m, 256)) * 4).astype(np.float32)
    codes = rng.integers(0, 256, size=(B, H, L, m), dtype=np.uint8)
    v = rng.standard_normal((B, H, L, d_k)).astype(np.float16)
    out, alpha = oracle.attend_decode(lut, codes, v, 0.25, want_alpha=True)
    assert np.all(alpha >= 0)
    assert np.max(np.abs(alpha.sum(-1) - 1.0)) <= 1e-12
    vf = v.astype(np.float64)
    assert np.all(out <= vf.max(axis=2) + 1e-6) and np.all(out >= vf.min(axis=2) - 1e-6)


def test_one_hot_and_uniform_closed_forms():
    rng = np.random.default_rng(22)
    L, d_k, m = 100, 8, 2
    v = rng.standard_normal((1, 1, L, d_k)).astype(np.float16)
    codes = np.zeros((1, 1, L, m), dtype=np.uint8)
    codes[0, 0, :, 1] = rng.integers(0, 256, size=L)
    codes[0, 0, 41, 0] = 7
    lut = np.zeros((1, 1, m, 256), dtype=np.float32)
    lut[0, 0, 0, 7] = 800.0      # only key 41 reaches this entry
    out = oracle.attend_decode(lut, codes, v, 1.0)
    assert np.array_equal(out[0, 0], v[0, 0, 41].astype(np.float32))
    flat = np.full((1, 1, m, 256), -3.5, dtype=np.float32)
    out = oracle.attend_decode(flat, codes, v, 0.3)
    assert np.max(np.abs(out[0, 0] - v[0, 0].astype(np.float64).mean(0))) <= 1e-6


def test_hand_worked_example():
    """d_k = 2, m = 2, K = 2, worked by hand.
    q = (ln 2, ln 3); C_1 = {0, 1}, C_2 = {0, 1}; LUT_1 = (0, ln 2), LUT_2 = (0, ln 3).
    Keys coded (0,0), (1,0), (0,1), (1,1) score 0, ln 2, ln 3, ln 6; with scale 1 the softmax
    weights are (1, 2, 3, 6)/12.  Values (12,0), (0,12), (12,12), (2,4) give
    o = (1*12 + 3*12 + 6*2, 2*12 + 3*12 + 6*4)/12 = (5, 7)."""
    q = np.array([math.log(2.0), math.log(3.0)], dtype=np.float32).reshape(1, 1, 1, 2)
    cb = np.array([[0.0], [1.0]], dtype=np.float32).reshape(1, 1, 2, 1).repeat(2, axis=1)
    lut = oracle.build_lut(q, cb)
    assert lut.shape == (1, 1, 1, 2, 2)
    assert np.array_equal(lut[0, 0, 0], np.array([[0, q[0, 0, 0, 0]], [0, q[0, 0, 0, 1]]], dtype=np.float32))
    codes = np.array([[0, 0], [1, 0], [0, 1], [1, 1]], dtype=np.uint8).reshape(1, 1, 4, 2)
    v = np.array([[12, 0], [0, 12], [12, 12], [2, 4]], dtype=np.float16).reshape(1, 1, 4, 2)
    out, s, a = oracle.attend_decode(lut[:, :, 0], codes, v, 1.0, want_scores=True, want_alpha=True)
    assert np.allclose(s[0, 0], [0.0, math.log(2), math.log(3), math.log(6)], atol=1e-6)
    assert np.allclose(a[0, 0], np.array([1, 2, 3, 6]) / 12.0, atol=1e-7)
    assert np.allclose(out[0, 0], [5.0, 7.0], atol=1e-5)
    # encoding of the matching keys: nearest of {0, 1} per coordinate
    keys = np.array([[0.2, 0.4], [0.9, 0.1], [0.3, 0.7], [0.6, 0.8]], dtype=np.float32).reshape(1, 1, 4, 2)
    assert np.array_equal(oracle.encode_keys(keys, cb), codes)


# ---- P7: invariances -------------------------------------------------------------

def test_permutation_and_lut_shift_invariance():
    rng = np.random.default_rng(23)
    B, H, L, d_k, m = 1, 2, 200, 8, 4
    lut = rng.standard_normal((B, H, m, 256)).astype(np.float32)
    codes = rng.integers(0, 256, size=(B, H, L, m), dtype=np.uint8)
    v = rng.standard_normal((B, H, L, d_k)).astype(np.float16)
    out = oracle.attend_decode(lut, codes, v, 0.5)
    p = rng.permutation(L)
    out_p = oracle.attend_decode(lut, codes[:, :, p], v[:, :, p], 0.5)
    assert np.max(np.abs(out - out_p)) <= 1e-6
    shifted = lut.copy()
    shifted[:, :, 2] += np.float32(1.75)
    out_s = oracle.attend_decode(shifted, codes, v, 0.5)
    assert np.max(np.abs(out - out_s)) <= 1e-5


# ---- causal prefill scoring ---------------------------------------------------------

def test_score_prefill_matches_numpy_gather():
    rng = np.random.default_rng(31)
    B, H, T, m = 1, 2, 9, 4
    lut = rng.standard_normal((B, H, T, m, 256)).astype(np.float32)
    codes = rng.integers(0, 256, size=(B, H, T, m), dtype=np.uint8)
    s = oracle.score_prefill(lut, codes)
    assert s.shape == (B, H, T, T)
    for h in range(H):
        for t in range(T):
            for l in range(T):
                if l > t:
                    assert s[0, h, t, l] == -np.inf
                else:
                    ref = sum(float(lut[0, h, t, i, codes[0, h, l, i]]) for i in range(m))
                    assert abs(s[0, h, t, l] - ref) <= 1e-6
    # queries that are the last T positions of a longer cache: query t sees l <= t + (L - T)
    L = T + 5
    codes2 = rng.integers(0, 256, size=(B, H, L, m), dtype=np.uint8)
    s2 = oracle.score_prefill(lut, codes2)
    assert s2.shape == (B, H, T, L)
    for h in range(H):
        for t in range(T):
            for l in range(L):
                if l > t + 5:
                    assert s2[0, h, t, l] == -np.inf
                else:
                    ref = sum(float(lut[0, h, t, i, codes2[0, h, l, i]]) for i in range(m))
                    assert abs(s2[0, h, t, l] - ref) <= 1e-6
    with pytest.raises(RuntimeError):
        oracle.score_prefill(lut, codes2[:, :, :T - 1])
    # row t of the causal scores equals decode scores of query t restricted to l <= t
    dec = oracle.adc_scores(lut[:, :, 5], codes)
    assert np.array_equal(dec[..., :6], s[:, :, 5, :6])


# ---- P8: Lloyd iterations (harness) ----------------------------------------------------

def test_kmeans_step_matches_numpy_and_is_monotone():
    cfg = li.shrink(li.CONFIGS["C1"], H=2, L=8, n_calib=700, m=4)
    case = li.make_case(cfg, seed=77)
    calib, cb = case["calib"], case["cb_init"]
    new, obj = oracle.kmeans_step(calib, cb)
    H, m, K, d_sub = cb.shape
    for h in range(H):
        for i in range(m):
            x = calib[h, :, i * d_sub:(i + 1) * d_sub].astype(np.float64)
            d = ((x[:, None, :] - cb[h, i].astype(np.float64)[None]) ** 2).sum(-1)
            a = d.argmin(-1)
            assert abs(obj[h, i] - d.min(-1).sum()) <= 1e-9 * max(1.0, obj[h, i])
            for c in range(K):
                mem = x[a == c]
                if len(mem):
                    assert np.allclose(new[h, i, c], mem.mean(0), rtol=0, atol=1e-6)
                else:
                    assert np.array_equal(new[h, i, c], cb[h, i, c])
    _, objs = oracle.kmeans(calib, cb, 10)
    tot = objs.sum(axis=(1, 2))
    assert np.all(np.diff(tot) <= 1e-9 * tot[0])
    assert tot[-1] < 0.9 * tot[0]


# ---- P9: the paper's printed accounting ---------------------------------------------

def _golden():
    vals = {}
    with open(os.path.join(HERE, "golden", "paper_accounting.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                vals[k.strip()] = int(v)
    return vals


def test_paper_accounting_matches_array_shapes():
    g = _golden()
    cfg = li.shrink(li.CONFIGS["C2"], B=1, H=1, L=512, n_calib=256)
    case = li.make_case(cfg)
    codes = oracle.encode_keys(case["keys"], case["cb_init"])
    lut = oracle.build_lut(case["q"], case["cb_init"])
    assert codes[0, 0, 0].nbytes == g["lookat4_key_bytes"]
    assert case["keys"][0, 0, 0].astype(np.float16).nbytes == g["fp16_key_bytes_dk64"]
    assert g["fp16_key_bytes_dk64"] // codes[0, 0, 0].nbytes == g["lookat4_compression"]
    assert lut.shape[-2:] == (g["lut_tables"], g["lut_entries_per_table"])
    assert lut[0, 0, 0].size * cfg.d_sub == g["lut_build_macs_dk64_m4"]
    assert cfg.m == g["lookups_per_key_m4"] and cfg.m - 1 == g["adds_per_key_m4"]
    assert cfg.L * cfg.d_k == g["standard_ops_L512_d64"]
    assert lut[0, 0, 0].size + codes[0, 0].size == g["lookat_ops_L512_m4"]
    for m_, name in ((2, "lookat2"), (8, "lookat8"), (16, "lookat16")):
        assert m_ == g[f"{name}_bytes_per_token"]
        assert 2 * 64 // m_ == g[f"{name}_compression"]


# ---------------------------------------------------------------- grouped queries ----

def _gqa_case(rng, B=2, H=3, g=4, L=41, d_k=8, m=2):
    d_sub = d_k // m
    cb = rng.standard_normal((H, m, 256, d_sub)).astype(np.float32)
    keys = rng.standard_normal((B, H, L, d_k)).astype(np.float32)
    v = rng.standard_normal((B, H, L, d_k)).astype(np.float16)
    q = (rng.standard_normal((B, H * g, 1, d_k)) / 2).astype(np.float32)
    codes = oracle.encode_keys(keys, cb)
    # tables of query head hq against the codebooks of key/value head hq // g
    lut = oracle.build_lut(q, np.repeat(cb, g, axis=0))[:, :, 0]
    return cb, keys, v, q, codes, lut


def test_gqa_equals_numpy_on_shared_heads():
    """Grouped queries against a numpy evaluation (gather, softmax, weighted sum) that maps query
    head hq to key/value head hq // g by explicit indexing."""
    rng = np.random.default_rng(31)
    for g in (1, 2, 4, 8):
        cb, keys, v, q, codes, lut = _gqa_case(rng, g=g)
        out, scores = oracle.attend_decode_gqa(lut, codes, v, 0.3, want_scores=True)
        B, HQ, m, K = lut.shape
        L = codes.shape[2]
        ref_s = np.zeros((B, HQ, L))
        for hq in range(HQ):
            for i in range(m):
                ref_s[:, hq] += np.take_along_axis(lut[:, hq, i].astype(np.float64), codes[:, hq // g, :, i].astype(np.int64), axis=-1)
        assert np.allclose(scores, ref_s, rtol=0, atol=1e-5)
        v_exp = np.stack([v[:, hq // g] for hq in range(HQ)], axis=1)
        ref_o, _ = _np_softmax_attend(ref_s.astype(np.float32), v_exp, 0.3)
        assert np.allclose(out, ref_o, rtol=0, atol=1e-5)


def test_gqa_group_one_is_plain_attention_and_heads_map_by_division():
    rng = np.random.default_rng(32)
    cb, keys, v, q, codes, lut = _gqa_case(rng, g=1)
    assert np.array_equal(oracle.attend_decode_gqa(lut, codes, v, 0.25), oracle.attend_decode(lut, codes, v, 0.25))
    # changing the values of key/value head 1 changes exactly the outputs of query heads 4..7 (g = 4):
    # a modulo instead of a division in the head mapping would touch heads 1, 4, 7, 10
    cb, keys, v, q, codes, lut = _gqa_case(rng, g=4)
    base = oracle.attend_decode_gqa(lut, codes, v, 0.25)
    v2 = v.copy()
    v2[:, 1] += np.float16(1.0)
    moved = np.abs(oracle.attend_decode_gqa(lut, codes, v2, 0.25) - base).max(axis=(0, 2)) > 0
    assert moved.tolist() == [False] * 4 + [True] * 4 + [False] * 4


def test_gqa_zero_distortion_equals_dense_grouped_attention():
    """256 keys that are their own centroids: LOOKAT with grouped queries equals dense grouped-query
    attention softmax(q K^T / sqrt(d_k)) V evaluated by numpy in fp64."""
    rng = np.random.default_rng(33)
    B, H, g, L, d_k, m = 1, 2, 4, 256, 16, 4
    d_sub = d_k // m
    keys = rng.standard_normal((B, H, L, d_k)).astype(np.float32)
    cb = np.stack([np.stack([keys[0, h, :, i * d_sub:(i + 1) * d_sub] for i in range(m)]) for h in range(H)])
    v = rng.standard_normal((B, H, L, d_k)).astype(np.float16)
    q = (rng.standard_normal((B, H * g, 1, d_k)) / 2).astype(np.float32)
    codes = oracle.encode_keys(keys, cb)
    lut = oracle.build_lut(q, np.repeat(cb, g, axis=0))[:, :, 0]
    out = oracle.attend_decode_gqa(lut, codes, v, 1.0 / math.sqrt(d_k))
    kx = np.repeat(keys.astype(np.float64), g, axis=1)
    vx = np.repeat(v.astype(np.float64), g, axis=1)
    s = np.einsum("bhd,bhld->bhl", q[:, :, 0].astype(np.float64), kx) / math.sqrt(d_k)
    a = np.exp(s - s.max(-1, keepdims=True))
    a /= a.sum(-1, keepdims=True)
    ref = np.einsum("bhl,bhld->bhd", a, vx)
    assert np.allclose(out, ref, rtol=0, atol=2e-6)
