"""HIP path vs CPU oracle, element by element on the same seeded inputs, through the C ABI.

Bars (tests/bars.py):
  * codes: bit-exact;
  * table entries and scores: |gpu - oracle| <= 1e-4 * (sum of the magnitudes of the summed terms)
    (fp32 accumulation; relative to the summands so that cancellation is not penalised);
  * outputs: |gpu - oracle| <= 2e-3 absolute (the contract: fp16 values, fp32 accumulation) AND
    <= 2e-5 (what the kernel's arithmetic gives; small enough to see a lost tile or a lost key
    that carries weight).
"""
import functools
import math

import numpy as np
import pytest
import torch

import lookat_inputs as li
import oracle
from bars import OUT_ATOL, REL, assert_lut_close, assert_out_close, assert_scores_close, record

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lk():
    import paper_2601_10155_amd as pkg
    pkg.load_library()
    return pkg


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# ---------------------------------------------------------------- encode --------------

@pytest.mark.parametrize("d_k,m", [(64, 4), (64, 2), (64, 16), (128, 8), (128, 16), (64, 64 // 64), (24, 2), (8, 8)])
@pytest.mark.parametrize("key_dtype", ["float32", "float16"])
def test_encode_bit_exact(lk, d_k, m, key_dtype):
    cfg = li.shrink(li.CONFIGS["C2"], B=3, H=2, L=300 + m, d_k=d_k, m=m, n_calib=600, key_dtype=key_dtype,
                    rank=min(8, d_k))
    case = li.make_case(cfg, seed=1000 + d_k + m)
    cb, _ = oracle.kmeans(case["calib"], case["cb_init"], 2)
    ref = oracle.encode_keys(case["keys"], cb)
    got = lk.lookat_encode_keys(dev(case["keys"]), dev(cb)).cpu().numpy()
    assert got.dtype == np.uint8 and got.shape == ref.shape
    assert np.array_equal(got, ref), f"{(got != ref).sum()} of {ref.size} codes differ"


@pytest.mark.parametrize("d_k,m,key_dtype", [(64, 4, "float32"), (128, 16, "float16"), (64, 2, "float16")])
def test_encode_bit_exact_many_keys(lk, d_k, m, key_dtype):
    """Enough keys per head that the one-thread-per-key kernel runs (the small cases above take
    the centroid-parallel kernel); ragged last block."""
    cfg = li.shrink(li.CONFIGS["C2"], B=4, H=4, L=4096 + 37, d_k=d_k, m=m, n_calib=512, key_dtype=key_dtype)
    case = li.make_case(cfg, seed=1500 + d_k + m)
    cb, _ = oracle.kmeans(case["calib"], case["cb_init"], 1)
    ref = oracle.encode_keys(case["keys"], cb)
    got = lk.lookat_encode_keys(dev(case["keys"]), dev(cb)).cpu().numpy()
    assert np.array_equal(got, ref), f"{(got != ref).sum()} of {ref.size} codes differ"


@pytest.mark.parametrize("N", [3, 5000])
def test_encode_nan_distances(lk, N):
    """A NaN distance never wins, unless it is centroid 0's (the scan starts there)."""
    rng = np.random.default_rng(6)
    cb = rng.standard_normal((2, 4, 256, 16)).astype(np.float32)
    cb[0, 0, 0, 3] = np.nan          # head 0, subspace 0: centroid 0 is NaN -> code 0 for every key
    cb[0, 1, 77, 0] = np.nan         # a NaN centroid elsewhere is never chosen
    cb[1, 2, 255] = np.nan
    keys = rng.standard_normal((2, 2, N, 64)).astype(np.float32)
    ref = oracle.encode_keys(keys, cb)
    got = lk.lookat_encode_keys(dev(keys), dev(cb)).cpu().numpy()
    assert np.array_equal(got, ref)
    assert (got[:, 0, :, 0] == 0).all() and not (got[:, 0, :, 1] == 77).any() and not (got[:, 1, :, 2] == 255).any()


@pytest.mark.parametrize("n_keys", [24, 70, 9000])   # 24: the few-key kernel (under 64 rows per head)
def test_encode_ties_and_duplicates(lk, n_keys):
    d_sub, K = 16, 256
    rng = np.random.default_rng(4)
    cb = (rng.standard_normal((2, 4, K, d_sub)) * 3).astype(np.float32)
    cb[:, :, 9] = cb[:, :, 5]               # duplicate centroid: 9 may never be chosen
    cb[0, 0, 100] = 0.0
    cb[0, 0, 200] = 2.0                     # keys of all-ones are exactly midway between 100 and 200
    cb[1] = 1.5                             # a head whose centroids are all equal -> code 0 everywhere
    keys = rng.standard_normal((2, 2, n_keys, 64)).astype(np.float32)
    keys[:, 0, :10, :16] = 1.0
    keys[:, 0, 10:20, 16:32] = cb[0, 1, 5]  # exactly on the duplicated centroid
    ref = oracle.encode_keys(keys, cb)
    got = lk.lookat_encode_keys(dev(keys), dev(cb)).cpu().numpy()
    assert np.array_equal(got, ref)
    assert not (got == 9).any()
    assert (got[:, 1] == 0).all()
    assert (got[:, 0, 10:20, 1] == 5).all()


@pytest.mark.parametrize("d_k,m", [(64, 4), (128, 16), (64, 16), (64, 2)])
@pytest.mark.parametrize("key_dtype", ["float32", "float16"])
def test_encode_near_ties_sweep(lk, d_k, m, key_dtype):
    """Keys placed on the bisector of two centroids and pushed off it by 1e-9 .. 1e-2 of the
    centroid distance, towards either side: the fp32 filter in front of the exact rule must hand
    every case it cannot decide to the exact rule, whatever the size of the push."""
    d_sub = d_k // m
    rng = np.random.default_rng(77 + d_k + m)
    H, B, N = 2, 2, 4096
    cb = (rng.standard_normal((H, m, 256, d_sub)) * 2).astype(np.float32)
    keys = (rng.standard_normal((B, H, N, d_k)) * 2).astype(np.float32)
    for b in range(B):
        for h in range(H):
            for n in range(0, N, 2):            # every other key is a constructed near tie
                i = int(rng.integers(m))
                ca, cc = rng.choice(256, 2, replace=False)
                mid = 0.5 * (cb[h, i, ca].astype(np.float64) + cb[h, i, cc])
                dirn = cb[h, i, ca].astype(np.float64) - cb[h, i, cc]
                eps = 10.0 ** rng.uniform(-9, -2) * rng.choice([-1.0, 1.0])
                keys[b, h, n, i * d_sub:(i + 1) * d_sub] = (mid + eps * dirn).astype(np.float32)
    keys = keys.astype(key_dtype)
    ref = oracle.encode_keys(keys, cb)
    got = lk.lookat_encode_keys(dev(keys), dev(cb)).cpu().numpy()
    assert np.array_equal(got, ref), f"{(got != ref).sum()} of {ref.size} codes differ"


def test_encode_filter_and_exact_kernels_agree(lk, monkeypatch):
    """The filter kernel and the plain exact kernels (forced through the environment switch) give
    the same codes, both equal to the oracle's."""
    cfg = li.shrink(li.CONFIGS["C4"], B=2, H=3, L=3000, T=1, n_calib=512)
    case = li.make_case(cfg, seed=1700)
    cb, _ = oracle.kmeans(case["calib"], case["cb_init"], 1)
    ref = oracle.encode_keys(case["keys"], cb)
    fast = lk.lookat_encode_keys(dev(case["keys"]), dev(cb)).cpu().numpy()
    monkeypatch.setenv("LOOKAT_ENCODE_EXACT", "1")
    slow = lk.lookat_encode_keys(dev(case["keys"]), dev(cb)).cpu().numpy()
    monkeypatch.delenv("LOOKAT_ENCODE_EXACT")
    assert np.array_equal(fast, ref) and np.array_equal(slow, ref)


def test_encode_append_into_cache(lk):
    cfg = li.shrink(li.CONFIGS["C2"], B=2, H=3, L=5, n_calib=300)
    case = li.make_case(cfg, seed=5)
    cb = case["cb_init"]
    ref = oracle.encode_keys(case["keys"], cb)
    cache = torch.full((2, 3, 40, 4), 255, dtype=torch.uint8, device="cuda")
    lk.lookat_encode_keys(dev(case["keys"]), dev(cb), cache=cache, position=16)
    c = cache.cpu().numpy()
    assert np.array_equal(c[:, :, 16:21], ref)
    assert (c[:, :, :16] == 255).all() and (c[:, :, 21:] == 255).all()
    # N = 0 is a no-op
    empty = torch.empty((2, 3, 0, 64), device="cuda")
    assert lk.lookat_encode_keys(empty, dev(cb)).shape == (2, 3, 0, 4)


# ---------------------------------------------------------------- LUT ------------------

@pytest.mark.parametrize("d_k,m", [(64, 4), (64, 2), (128, 8), (128, 16), (64, 1), (24, 2)])
@pytest.mark.parametrize("q_dtype", ["float16", "float32"])
@pytest.mark.parametrize("B,T", [(1, 1), (5, 1), (2, 37)])
def test_build_lut_parity(lk, d_k, m, q_dtype, B, T):
    cfg = li.shrink(li.CONFIGS["C2"], B=B, H=3, L=4, T=T, d_k=d_k, m=m, n_calib=300, q_dtype=q_dtype,
                    rank=min(8, d_k))
    case = li.make_case(cfg, seed=2000 + d_k + m + T)
    cb = case["cb_init"]
    ref = oracle.build_lut(case["q"], cb)
    got = lk.lookat_build_lut(dev(case["q"]), dev(cb)).cpu().numpy()
    assert got.shape == ref.shape
    assert_lut_close(got, case["q"], cb, ref)


@pytest.mark.parametrize("d_k,m", [(128, 16), (64, 4), (64, 16), (128, 32), (64, 32)])
@pytest.mark.parametrize("q_dtype", ["float16", "float32"])
@pytest.mark.parametrize("B,T", [(1, 256), (3, 333), (2, 1031)])
def test_build_lut_batched_matrix_core_path(lk, d_k, m, q_dtype, B, T):
    """>= 256 queries per head: the MFMA kernel (d_sub in {2,4,8,16}); ragged 32-query tiles and
    tiles that straddle batch entries."""
    cfg = li.shrink(li.CONFIGS["C4"], B=B, H=2, L=4, T=T, d_k=d_k, m=m, n_calib=300, q_dtype=q_dtype)
    case = li.make_case(cfg, seed=2500 + d_k + m + T)
    cb = case["cb_init"]
    ref = oracle.build_lut(case["q"], cb)
    got = lk.lookat_build_lut(dev(case["q"]), dev(cb)).cpu().numpy()
    assert_lut_close(got, case["q"], cb, ref)


def test_build_lut_tables_beyond_the_cache(lk):
    """A table set over 256 MiB (here 262 MiB) takes the instance that writes with non-temporal stores;
    every entry is compared."""
    cfg = li.shrink(li.CONFIGS["C4"], B=2, H=3, L=4, T=2795, d_k=128, m=16, n_calib=300, q_dtype="float16")
    case = li.make_case(cfg, seed=2999)
    cb = case["cb_init"]
    assert 2 * 3 * 2795 * 16 * 256 * 4 > 256 << 20
    ref = oracle.build_lut(case["q"], cb)
    got = lk.lookat_build_lut(dev(case["q"]), dev(cb)).cpu().numpy()
    assert_lut_close(got, case["q"], cb, ref)


# ---------------------------------------------------------------- decode ---------------

def _decode_case(rng, B, H, L, d_k, m, lut_scale=2.0):
    lut = (rng.standard_normal((B, H, m, 256)) * lut_scale).astype(np.float32)
    codes = rng.integers(0, 256, size=(B, H, L, m), dtype=np.uint8)
    v = rng.standard_normal((B, H, L, d_k)).astype(np.float16)
    return lut, codes, v


@pytest.mark.parametrize("d_k,m", [(64, 4), (64, 2), (64, 8), (64, 16), (128, 8), (128, 16), (128, 2),
                                   (64, 1), (128, 32), (32, 4), (256, 8), (40, 5), (96, 4)])
@pytest.mark.parametrize("L", [1, 63, 64, 65, 257, 1000])
def test_decode_parity_shapes(lk, d_k, m, L):
    rng = np.random.default_rng(3000 + d_k * 7 + m * 3 + L)
    B, H = 2, 5   # B*H = 10: not a multiple of the 8 dies
    lut, codes, v = _decode_case(rng, B, H, L, d_k, m)
    scale = 1.0 / math.sqrt(d_k)
    ref, s_ref = oracle.attend_decode(lut, codes, v, scale, want_scores=True)
    for splits in (0, 1, 3):
        scores = torch.empty((B, H, L), dtype=torch.float32, device="cuda")
        out = lk.lookat_attend_decode(dev(lut), dev(codes), dev(v), scale, num_splits=splits, scores_out=scores)
        assert_out_close(out.cpu().numpy(), ref, "attend_decode, contexts up to 1000", s_ref, scale)
        assert_scores_close(scores.cpu().numpy(), lut, codes, s_ref)


# (d_k, m) -> does a 16-wavefront instance exist (it must fit 64 registers)
_LARGE_WG = {(64, 4): True, (128, 8): True, (64, 2): True, (128, 16): False}


@pytest.mark.parametrize("d_k,m", sorted(_LARGE_WG))
@pytest.mark.parametrize("L", [2048, 2049, 4133, 9000, 16421])
def test_decode_parity_long_ranges(lk, d_k, m, L):
    """Ranges of 2048 keys and more take the 16-wavefront instance of the kernel (the one that runs the
    32768-key workload): scores element by element and outputs at the arithmetic bar, on a peaked softmax
    (table entries of scale 8: a handful of keys carry percents of the weight), with the range count left to
    the library, one range, and two.  The test states which instance each case resolves to."""
    rng = np.random.default_rng(3500 + d_k * 7 + m * 3 + L)
    B, H = 2, 3
    lut, codes, v = _decode_case(rng, B, H, L, d_k, m, lut_scale=8.0)
    scale = 1.0 / math.sqrt(d_k)
    ref, s_ref = oracle.attend_decode(lut, codes, v, scale, want_scores=True)
    seen = set()
    for splits in (0, 1, 2):
        ranges, waves = lk.attend_decode_launch_shape(B, H, d_k, m, L, splits)
        per_range = -(-(-(-L // ranges)) // 64) * 64
        assert waves == (16 if _LARGE_WG[(d_k, m)] and per_range >= 2048 else 4)
        seen.add(waves)
        scores = torch.empty((B, H, L), dtype=torch.float32, device="cuda")
        out = lk.lookat_attend_decode(dev(lut), dev(codes), dev(v), scale, num_splits=splits, scores_out=scores)
        assert_out_close(out.cpu().numpy(), ref, f"attend_decode, long ranges, {waves}-wavefront instance", s_ref, scale)
        assert_scores_close(scores.cpu().numpy(), lut, codes, s_ref)
    if _LARGE_WG[(d_k, m)]:
        assert 16 in seen, "no case of this shape reached the 16-wavefront instance"


@pytest.mark.parametrize("splits", [1, 2, 3, 7, 16, 40])
def test_decode_split_count_invariance(lk, splits):
    """More ranges than 64-key tiles leaves some ranges empty: they must merge as zeros."""
    rng = np.random.default_rng(77)
    B, H, L, d_k, m = 1, 9, 777, 64, 4
    lut, codes, v = _decode_case(rng, B, H, L, d_k, m, lut_scale=6.0)
    ref, s_ref = oracle.attend_decode(lut, codes, v, 0.125, want_scores=True)
    out = lk.lookat_attend_decode(dev(lut), dev(codes), dev(v), 0.125, num_splits=splits).cpu().numpy()
    assert_out_close(out, ref, "attend_decode, range counts 1..40 on 777 keys", s_ref, 0.125)


def test_decode_peaked_and_flat_softmax(lk):
    rng = np.random.default_rng(78)
    B, H, L, d_k, m = 1, 2, 500, 64, 4
    lut, codes, v = _decode_case(rng, B, H, L, d_k, m)
    lut[0, 0] = 0.0
    lut[0, 0, 0, 7] = 4000.0          # one-hot: a single key owns code 7 in subspace 0
    codes[0, 0, :, 0] = 3
    codes[0, 0, 321, 0] = 7
    lut[0, 1] = -2.5                  # flat: output is the mean of the values
    for splits in (1, 4):
        out = lk.lookat_attend_decode(dev(lut), dev(codes), dev(v), 1.0, num_splits=splits).cpu().numpy()
        assert np.max(np.abs(out[0, 0] - v[0, 0, 321].astype(np.float32))) <= 1e-6
        assert np.max(np.abs(out[0, 1] - v[0, 1].astype(np.float64).mean(0))) <= OUT_ATOL
    ref = oracle.attend_decode(lut, codes, v, 1.0)
    assert np.max(np.abs(out - ref)) <= OUT_ATOL   # (exponents of magnitude 5770 in the one-hot head: contract bar only)
    assert_out_close(out[0, 1], ref[0, 1], "attend_decode, flat softmax")


def test_decode_on_cache_views(lk):
    """codes / values that are the first L rows of longer caches (strided (b,h) slabs)."""
    rng = np.random.default_rng(79)
    B, H, L, Lmax, d_k, m = 2, 3, 333, 512, 64, 4
    lut, codes, v = _decode_case(rng, B, H, Lmax, d_k, m)
    ref = oracle.attend_decode(lut, codes[:, :, :L], v[:, :, :L], 0.125)
    out = lk.lookat_attend_decode(dev(lut), dev(codes)[:, :, :L], dev(v)[:, :, :L], 0.125).cpu().numpy()
    assert_out_close(out, ref, "attend_decode on cache views")


# ---------------------------------------------------------------- whole path -----------

def _pipeline(lk, case, cb, scale, splits=0):
    """encode -> table -> decode on the GPU; returns numpy codes, lut, scores, out."""
    cfg = case["cfg"]
    codes = lk.lookat_encode_keys(dev(case["keys"]), dev(cb))
    lut = lk.lookat_build_lut(dev(case["q"]), dev(cb))
    scores = torch.empty((cfg.B, cfg.H, cfg.L), dtype=torch.float32, device="cuda")
    out = lk.lookat_attend_decode(lut.view(cfg.B, cfg.H, cfg.m, 256), codes, dev(case["values"]), scale,
                                  num_splits=splits, scores_out=scores)
    return codes.cpu().numpy(), lut.cpu().numpy(), scores.cpu().numpy(), out.cpu().numpy()


def _check_pipeline(lk, case, cb, splits=0):
    cfg = case["cfg"]
    scale = 1.0 / math.sqrt(cfg.d_k)
    codes_ref = oracle.encode_keys(case["keys"], cb)
    lut_ref = oracle.build_lut(case["q"], cb)
    codes, lut, scores, out = _pipeline(lk, case, cb, scale, splits)
    assert np.array_equal(codes, codes_ref)
    assert_lut_close(lut, case["q"], cb, lut_ref)
    # downstream of the table each side consumes its own table (the whole path is compared)
    out_ref, s_ref = oracle.attend_decode(lut_ref[:, :, 0], codes_ref, case["values"], scale, want_scores=True)
    assert_scores_close(scores, lut_ref[:, :, 0], codes_ref, s_ref)
    # (each side scores from its own table: the tables differ by fp32 rounding, which a peaked softmax
    # amplifies, so the whole path is held to the contract bar; the arithmetic bar is asserted where both
    # sides read the same table)
    err = np.max(np.abs(out - out_ref))
    record("whole path encode -> table -> attention", err)
    assert err <= OUT_ATOL
    return out, out_ref


def test_config_c0_whole_path(lk):
    """Single head, d_k=64, N=256, m=4: codebooks from 10 Lloyd iterations started at the keys."""
    case = li.make_case(li.CONFIGS["C0"], calib_is_cache=True)
    cb, _ = oracle.kmeans(case["calib"], case["cb_init"], 10)
    _check_pipeline(lk, case, cb)


def test_config_c1_one_layer_whole_path(lk):
    """GPT-2-small shape: 12 heads, d_k=64, context 1024, batch 1, m=2."""
    case = li.make_case(li.CONFIGS["C1"])
    cb, _ = oracle.kmeans(case["calib"], case["cb_init"], 3)
    _check_pipeline(lk, case, cb)


def test_config_c2_reduced_batch_whole_path(lk):
    """GPT-2-small shape, m=4, context 1024, batch 4 of 32 (the oracle's share that runs in seconds)."""
    case = li.make_case(li.shrink(li.CONFIGS["C2"], B=4, n_calib=1024))
    cb, _ = oracle.kmeans(case["calib"], case["cb_init"], 2)
    _check_pipeline(lk, case, cb, splits=4)


def test_config_c3_reduced_whole_path(lk):
    """Llama shape d_k=128, m=8 with a ragged long context and several ranges."""
    case = li.make_case(li.shrink(li.CONFIGS["C3"], B=2, H=3, L=5000 + 37, n_calib=512))
    cb, _ = oracle.kmeans(case["calib"], case["cb_init"], 1)
    _check_pipeline(lk, case, cb, splits=0)
    _check_pipeline(lk, case, cb, splits=5)


# ---------------------------------------------------------------- codebook learning ----

@pytest.mark.parametrize("d_k,m", [(64, 4), (64, 2), (128, 16), (24, 2)])
def test_kmeans_step_bit_exact(lk, d_k, m):
    """Assignment = the encoder (bit-exact); the update is an fp64 sum in key order, so the new
    codebooks must equal the oracle's exactly, iteration after iteration."""
    cfg = li.shrink(li.CONFIGS["C1"], H=3, L=8, d_k=d_k, m=m, n_calib=1500, rank=min(8, d_k))
    case = li.make_case(cfg, seed=4000 + d_k + m)
    calib, cb = case["calib"], case["cb_init"]
    cb_gpu = dev(cb)
    for it in range(3):
        ref, _ = oracle.kmeans_step(calib, cb)
        got, assign = lk.lookat_kmeans_step(dev(calib), cb_gpu)
        assert np.array_equal(assign.cpu().numpy(), oracle.encode_keys(calib[None], cb)[0])
        assert np.array_equal(got.cpu().numpy(), ref), f"iteration {it}"
        cb, cb_gpu = ref, got
    # the multi-iteration helper lands on the same codebooks
    again = lk.lookat_kmeans(dev(calib), dev(case["cb_init"]), 3).cpu().numpy()
    assert np.array_equal(again, cb)


@pytest.mark.parametrize("n_calib", [1, 17, 16384, 16385])
def test_kmeans_step_calibration_set_sizes(lk, n_calib):
    """One key, a ragged handful, and both sides of the size at which the update kernel changes from
    member lists in LDS to a scan of all keys: same bits as the oracle either way."""
    cfg = li.shrink(li.CONFIGS["C1"], H=2, L=8, d_k=16, m=2, n_calib=max(n_calib, 300), rank=8)
    case = li.make_case(cfg, seed=4200 + n_calib)
    calib = np.ascontiguousarray(case["calib"][:, :n_calib])   # (the initial codebooks are drawn from 300 keys)
    ref, _ = oracle.kmeans_step(calib, case["cb_init"])
    got, assign = lk.lookat_kmeans_step(dev(calib), dev(case["cb_init"]))
    assert np.array_equal(assign.cpu().numpy(), oracle.encode_keys(calib[None], case["cb_init"])[0])
    assert np.array_equal(got.cpu().numpy(), ref)


def test_kmeans_empty_cluster_keeps_centroid(lk):
    cfg = li.shrink(li.CONFIGS["C1"], H=1, L=8, n_calib=300, m=2)
    case = li.make_case(cfg, seed=4100)
    cb = case["cb_init"].copy()
    cb[0, 0, 17] = 1e6          # no calibration key is anywhere near: cluster 17 stays empty
    ref, _ = oracle.kmeans_step(case["calib"], cb)
    got, _ = lk.lookat_kmeans_step(dev(case["calib"]), dev(cb))
    got = got.cpu().numpy()
    assert np.array_equal(got, ref)
    assert np.array_equal(got[0, 0, 17], cb[0, 0, 17])


# ---------------------------------------------------------------- causal prefill scoring ----

def _prefill_bars(got, ref, q, cb, codes, lut_ref, label):
    """Causal scores against the oracle's.  The kernel never rounds a table entry to fp32 on its way to the
    score (the tables stay on chip), so a score's summands are the products q_j * c_j of every subspace and
    the bar is 1e-4 of sum_i sum_j |q_j| |C_i[c_i]_j|.  The narrower bar of the decode path, 1e-4 of
    sum_i |LUT_i[c_i]| (the magnitudes of the finished table entries), is counted alongside: entries that
    miss it are cases of cancellation INSIDE a table entry (|q . c| far below sum |q_j c_j|)."""
    vis = np.isfinite(ref)
    assert np.array_equal(np.isneginf(got), ~vis), "mask differs"
    B, H, T, m, K = lut_ref.shape
    d_sub = cb.shape[3]
    qa = np.abs(q.astype(np.float64)).reshape(B, H, T, m, d_sub)
    hidx = np.arange(H)[None, :, None]
    picked = np.stack([np.abs(cb.astype(np.float64))[hidx, i, codes[:, :, :, i].astype(np.int64)]
                       for i in range(m)], axis=3)                                   # [B,H,L,m,d_sub]
    mag = np.einsum("bhtid,bhlid->bhtl", qa, picked)
    err = np.abs(np.where(vis, got, 0.0).astype(np.float64) - np.where(vis, ref, 0.0).astype(np.float64))
    assert np.all(err[vis] <= REL * np.maximum(mag[vis], 1e-6)), f"max err {err[vis].max()}"
    narrow = np.zeros_like(mag)
    bidx = np.arange(B)[:, None, None]
    for i in range(m):
        ent = np.abs(lut_ref[:, :, :, i, :].astype(np.float64))                      # [B,H,T,K]
        narrow += ent[bidx, hidx, :, codes[:, :, :, i].astype(np.int64)].transpose(0, 1, 3, 2)   # [B,H,T,L]
    miss = int(np.count_nonzero(err[vis] > REL * np.maximum(narrow[vis], 1e-6)))
    tally = _PREFILL_NARROW.setdefault(label, {"entries": 0, "missed": 0})
    tally["entries"] += int(vis.sum())
    tally["missed"] += miss
    record(label + ": worst |err| / (1e-4 * sum_i |LUT_i[c_i]|)",
           float(np.max(err[vis] / (REL * np.maximum(narrow[vis], 1e-6)))))
    record(label + ": entries checked", tally["entries"])
    record(label + ": entries outside the table-entry bar", tally["missed"])
    # the wider form may be needed only by a vanishing share of the entries
    assert miss <= 1e-5 * vis.sum() + 2, f"{miss} of {vis.sum()} entries miss the table-entry bar"


_PREFILL_NARROW = {}   # label -> entries checked / entries outside the table-entry bar

# lookat_score_prefill has two kernels: blocks of 24 or more queries are scored as a dense product against
# the keys' centroids on the matrix cores, shorter blocks by lookup-and-sum in LDS.  "library"
# takes the library's choice, "lookup" forces the lookup-and-sum kernel through its measurement-aid entry
# point, so that it stays covered on the shapes the library no longer routes to it.
_PREFILL_ENTRIES = {"library": ("lookat_score_prefill", "score_prefill"),
                    "lookup": ("lookat_probe_score_prefill_lookup", "score_prefill, lookup-and-sum kernel forced")}


def _prefill_check(lk, case, cb, codes, path="library"):
    q = case["q"]
    entry, label = _PREFILL_ENTRIES[path]
    lut_ref = oracle.build_lut(q, cb)
    ref = oracle.score_prefill(lut_ref, codes)
    got = getattr(lk, entry)(dev(q), dev(cb), dev(codes)).cpu().numpy()
    assert got.shape == ref.shape
    _prefill_bars(got, ref, q, cb, codes, lut_ref, label)


@pytest.mark.parametrize("d_k,m", [(128, 16), (128, 8), (64, 4), (64, 2), (64, 16)])
@pytest.mark.parametrize("q_dtype,path", [("float16", "library"), ("float16", "lookup"), ("float32", "library"),
                                          ("float32", "lookup")])
@pytest.mark.parametrize("T,extra", [(70, 0), (333, 0), (45, 50), (1, 0), (530, 135), (64, 0), (40, 24), (300, 1300),
                                     (40, 2101), (100, 4200), (32, 0), (31, 97), (129, 3), (96, 160), (23, 41), (24, 0)])
def test_score_prefill_parity(lk, d_k, m, q_dtype, path, T, extra):
    """Ragged query tiles (T not a multiple of 4 or of 32), one workgroup per (b,h) and several, queries that
    are the tail of a longer cache (extra > 0), a single query, contexts beyond the 2048 keys whose codes
    the lookup kernel's scoring threads keep in registers (one and two further rounds of keys), L odd (scalar
    stores), key panels that end inside a 128-key panel or exactly on one, T on either side of the 24 queries
    from which blocks go to the matrix cores."""
    L = T + extra
    cfg = li.shrink(li.CONFIGS["C4"], B=2, H=3, L=L, T=T, d_k=d_k, m=m, n_calib=400, q_dtype=q_dtype)
    case = li.make_case(cfg, seed=5000 + d_k + m + T)
    cb = case["cb_init"]
    codes = oracle.encode_keys(case["keys"], cb)
    _prefill_check(lk, case, cb, codes, path)


def test_score_prefill_matrix_core_kernel_wide_range_codebook(lk):
    """The matrix-core kernel scales each wavefront's centroids by a power of two and splits them into two
    fp16 terms, which keeps 22 bits of every entry down to 2^-27 of the wavefront's largest: a codebook whose
    subspaces sit at scales from 1e-3 to 1e3 (every wavefront meets all of them), with queries that weight the
    small subspaces up so that all of them matter in the sum, must still meet the bar relative to the summed
    products."""
    rng = np.random.default_rng(5200)
    B, H, T, L, d_k, m = 1, 2, 160, 300, 128, 16
    d_sub = d_k // m
    sub_scale = 10.0 ** rng.uniform(-3, 3, size=(H, m, 1, 1))
    cb = (rng.standard_normal((H, m, 256, d_sub)) * sub_scale).astype(np.float32)
    q = (rng.standard_normal((B, H, T, m, d_sub)) / sub_scale[None, :, :, 0, :].reshape(1, H, 1, m, 1)).reshape(B, H, T, d_k)
    q = q.astype(np.float16)
    codes = rng.integers(0, 256, size=(B, H, L, m), dtype=np.uint8)
    lut_ref = oracle.build_lut(q, cb)
    ref = oracle.score_prefill(lut_ref, codes)
    got = lk.lookat_score_prefill(dev(q), dev(cb), dev(codes)).cpu().numpy()
    vis = np.isfinite(ref)
    assert np.array_equal(np.isneginf(got), ~vis)
    qa = np.abs(q.astype(np.float64)).reshape(B, H, T, m, d_sub)
    hidx = np.arange(H)[None, :, None]
    picked = np.stack([np.abs(cb.astype(np.float64))[hidx, i, codes[:, :, :, i].astype(np.int64)] for i in range(m)], axis=3)
    mag = np.einsum("bhtid,bhlid->bhtl", qa, picked)
    err = np.abs(np.where(vis, got, 0.0).astype(np.float64) - np.where(vis, ref, 0.0).astype(np.float64))
    record("score_prefill, wide-range codebook: worst |err| / sum_j |q_j c_j|", float(np.max(err[vis] / np.maximum(mag[vis], 1e-30))))
    assert np.all(err[vis] <= REL * np.maximum(mag[vis], 1e-6)), f"max err {err[vis].max()}"


def test_score_prefill_single_head_and_padded_cache(lk):
    """One (b,h) with many tiles (its tiles are dealt to many workgroups) and codes that are the front
    part of a longer cache (slab stride larger than L*m)."""
    T, L, Lmax = 600, 700, 1000
    cfg = li.shrink(li.CONFIGS["C4"], B=1, H=1, L=Lmax, T=T, d_k=128, m=16, n_calib=400)
    case = li.make_case(cfg, seed=5077)
    cb = case["cb_init"]
    codes_all = oracle.encode_keys(case["keys"], cb)                 # [1,1,Lmax,m]
    codes = codes_all[:, :, :L]
    q = case["q"]
    ref = oracle.score_prefill(oracle.build_lut(q, cb), np.ascontiguousarray(codes))
    cache = dev(codes_all)
    got = lk.lookat_score_prefill(dev(q), dev(cb), cache[:, :, :L]).cpu().numpy()
    _prefill_bars(got, ref, q, cb, np.ascontiguousarray(codes), oracle.build_lut(q, cb), "score_prefill")


def test_score_prefill_matches_decode_rows(lk):
    """Row t of the causal block equals the decode scores of query t over the first t+1 keys."""
    cfg = li.shrink(li.CONFIGS["C4"], B=1, H=2, L=200, T=200, n_calib=400)
    case = li.make_case(cfg, seed=5100)
    cb = case["cb_init"]
    codes = lk.lookat_encode_keys(dev(case["keys"]), dev(cb))
    block = lk.lookat_score_prefill(dev(case["q"]), dev(cb), codes).cpu().numpy()
    lut = lk.lookat_build_lut(dev(case["q"]), dev(cb))
    for t in (0, 7, 8, 131, 199):
        s = torch.empty((1, 2, t + 1), dtype=torch.float32, device="cuda")
        lk.lookat_attend_decode(lut[:, :, t].contiguous(), codes[:, :, :t + 1], dev(case["values"])[:, :, :t + 1],
                                0.1, scores_out=s)
        d = np.abs(block[:, :, t, :t + 1] - s.cpu().numpy())
        assert d.max() <= 1e-5


# ---------------------------------------------------------------- fused decode step ----
#
# Three kinds of input per shape and length:
#   "recipe":  queries N(0,1)/8 (the workload recipe): a nearly flat softmax;
#   "peaked":  the same queries times 8: a few keys carry most of the weight;
#   "aligned": the appended key is planted on a centroid far from the data and the query points at it,
#              scaled so that the appended key takes about 3/4 of the softmax weight.  A step that scored
#              row L-1 from the stale cache row, or dropped it, would move the output by O(1).

@functools.lru_cache(maxsize=64)
def _step_inputs(base, B, H, Lmax, d_k, m, qk_dtype, seed):
    cfg = li.shrink(li.CONFIGS[base], B=B, H=H, L=Lmax, d_k=d_k, m=m, n_calib=400, key_dtype=qk_dtype,
                    q_dtype=qk_dtype, rank=8 if d_k == 64 else 16)
    return li.make_case(cfg, seed=seed)


def _step_case(base, B, H, Lmax, L, d_k, m, qk_dtype, seed, kind, g=1):
    """keys [B,H,L,d_k], k_new [B,H,d_k], q [B,H*g,d_k], values [B,H,L,d_k], codebooks; and the oracle's
    three steps on them: codes [B,H,L,m], out [B,H*g,d_k], scores [B,H*g,L], weight of row L-1 [B,H*g]."""
    case = _step_inputs(base, B, H, Lmax, d_k, m, qk_dtype, seed)
    rng = np.random.default_rng(seed * 31 + L * 7 + g)
    cb = case["cb_init"].copy()
    keys = case["keys"][:, :, :L].copy()
    v = case["values"][:, :, :L]
    scale = 1.0 / math.sqrt(d_k)
    if g == 1:
        q = case["q"][:, :, 0].copy()
    else:
        q = (rng.standard_normal((B, H * g, d_k)) / 8).astype(qk_dtype)
    if kind == "peaked":
        q = (q.astype(np.float32) * 8).astype(qk_dtype)
    elif kind == "aligned":
        u = rng.choice(np.array([-8.0, 8.0], dtype=np.float32), size=(H, d_k))      # exact in fp16
        cb[:, :, 255] = u.reshape(H, m, d_k // m)
        keys[:, :, L - 1] = u[None].astype(qk_dtype)
        codes1 = oracle.encode_keys(keys, cb)
        # scores are linear in q: with q = u they are s1; beta*u gives beta*s1.  Pick beta per (b,h) by
        # bisection so that row L-1 gets about 3/4 of the weight.
        lut1 = oracle.build_lut(np.broadcast_to(u[None, :, None], (B, H, 1, d_k)).astype(np.float32), cb)[:, :, 0]
        s1 = oracle.adc_scores(lut1, codes1).astype(np.float64)                      # [B,H,L]
        gap = s1[:, :, L - 1:L] - s1                                                 # >= 0 where row L-1 leads
        assert (gap >= 0).all(), "the planted key does not lead the scores"
        lo, hi = np.zeros((B, H)), np.full((B, H), 4.0)
        for _ in range(60):
            mid = 0.5 * (lo + hi)
            w = 1.0 / np.exp(-scale * mid[..., None] * gap).sum(-1)                  # weight of row L-1
            lo, hi = np.where(w < 0.75, mid, lo), np.where(w < 0.75, hi, mid)
        beta = np.repeat(np.maximum(hi, 1e-4), g, axis=1)                            # [B,H*g] (L = 1: any beta)
        if g > 1:   # every query head of the group at its own sharpness
            beta = beta * rng.uniform(1.0, 1.5, size=beta.shape)
        q = (beta[..., None] * np.repeat(u, g, axis=0)[None]).astype(qk_dtype)
    codes = oracle.encode_keys(keys, cb)
    lut = oracle.build_lut(q[:, :, None], np.repeat(cb, g, axis=0))[:, :, 0]          # [B,H*g,m,256]
    if g == 1:
        out, s, alpha = oracle.attend_decode(lut, codes, v, scale, want_scores=True, want_alpha=True)
        w_new = alpha[:, :, L - 1]
    else:
        out, s = oracle.attend_decode_gqa(lut, codes, v, scale, want_scores=True)
        w_new = None
    if kind == "aligned":
        assert (codes[:, :, L - 1] == 255).all()
        if w_new is not None:
            assert (w_new > 0.5).all() and (L == 1 or (w_new < 0.95).all()), \
                f"weight of the appended key {w_new.min()}..{w_new.max()}"
    return {"cb": cb, "keys": keys, "k_new": np.ascontiguousarray(keys[:, :, L - 1]), "q": q, "values": case["values"],
            "scale": scale, "codes": codes, "out": out, "scores": s}


def _run_step(lk, c, L, Lmax, stale, call):
    """Cache as a serving loop holds it: rows 0..L-2 coded, row L-1 stale, capacity Lmax.  Returns out."""
    B, H, _, m = c["codes"].shape
    cache = torch.full((B, H, Lmax, m), stale, dtype=torch.uint8, device="cuda")
    cache[:, :, :L - 1] = dev(c["codes"][:, :, :L - 1])
    values = dev(c["values"])
    out = call(dev(c["q"]), dev(c["k_new"]), dev(c["cb"]), cache[:, :, :L], values[:, :, :L], c["scale"])
    got = cache.cpu().numpy()
    assert np.array_equal(got[:, :, :L], c["codes"]), "code cache after the step"
    assert (got[:, :, L:] == stale).all(), "rows past L were touched"
    return out, cache


_STEP_SHAPES = [(64, 4), (64, 2), (64, 8), (64, 16), (128, 8), (128, 16), (128, 2), (128, 4)]


@pytest.mark.parametrize("d_k,m", _STEP_SHAPES)
@pytest.mark.parametrize("qk_dtype", ["float16", "float32"])
@pytest.mark.parametrize("L", [1, 64, 65, 300, 1024, 1537, 4133])
def test_decode_step_matches_oracle(lk, d_k, m, qk_dtype, L):
    """Contexts from one key to several rounds of the workgroup's 512-key step (the last two lengths run
    the streaming loop behind the tiles requested up front, with a ragged tail)."""
    B, H, Lmax = 2, 5, max(1100, L + 67)
    c = _step_case("C2", B, H, Lmax, L, d_k, m, qk_dtype, 6000 + d_k + m, "recipe")
    out, _ = _run_step(lk, c, L, Lmax, 0xAB, lk.lookat_decode_step)
    assert_out_close(out.cpu().numpy(), c["out"], "decode_step, recipe queries", c["scores"], c["scale"])


@pytest.mark.parametrize("d_k,m", [(64, 4), (64, 16), (128, 8), (128, 2)])
@pytest.mark.parametrize("qk_dtype", ["float16", "float32"])
@pytest.mark.parametrize("kind", ["peaked", "aligned"])
@pytest.mark.parametrize("L", [1, 2, 64, 65, 512, 513, 1024, 1537, 4133, 9000])
def test_decode_step_peaked_and_aligned(lk, d_k, m, qk_dtype, kind, L):
    """The appended key must be scored from the codes the step computes, not from the stale cache row: inputs
    on which one key's error shows (see the head of this section).  Row L-1 is the last lane of a tile
    (64, 512, 1024), the first lane of a fresh tile (65, 513, 1537) and mid-tile in the streaming loop."""
    B, H, Lmax = 2, 3, L + 67
    c = _step_case("C2", B, H, Lmax, L, d_k, m, qk_dtype, 6700 + d_k + m, kind)
    out, _ = _run_step(lk, c, L, Lmax, 0xAB, lk.lookat_decode_step)
    assert_out_close(out.cpu().numpy(), c["out"], f"decode_step, {kind} queries", c["scores"], c["scale"])


@pytest.mark.parametrize("d_k,m", [(64, 2), (64, 4), (64, 8), (64, 16), (128, 4), (128, 8), (128, 16)])
@pytest.mark.parametrize("qk_dtype", ["float16", "float32"])
@pytest.mark.parametrize("kind", ["recipe", "peaked", "aligned"])
@pytest.mark.parametrize("B,L", [(2, 1), (2, 65), (4, 512), (6, 1024), (4, 1537), (2, 4133)])
def test_decode_step_paired_entries_match_oracle_and_fused_step(lk, d_k, m, qk_dtype, kind, B, L):
    """The instance that serves two batch entries of a head per workgroup (each half's table builders fetch
    half the subspaces' codebook rows and compute both entries' tables and distances): codes and outputs
    against the oracle on the three kinds of input, and bit-identical to lookat_decode_step.  H = 3 and
    B in {2, 4, 6}: 3, 6 and 9 pairs, so the last round of workgroups is ragged."""
    if kind != "recipe" and qk_dtype == "float32":
        pytest.skip("peaked and aligned inputs run in fp16 (the dtype only changes how q and k_new are read)")
    H, Lmax = 3, L + 67
    c = _step_case("C2" if d_k == 64 else "C3", B, H, Lmax, L, d_k, m, qk_dtype, 6900 + d_k + m + B, kind)
    out, cache = _run_step(lk, c, L, Lmax, 0xAB, functools.partial(lk.lookat_probe_decode_step_entries, 2))
    assert_out_close(out.cpu().numpy(), c["out"], f"decode_step, paired entries, {kind} queries", c["scores"], c["scale"])
    assert lk.decode_step_entries_per_workgroup(B, H, d_k, m, L) == 1
    for single in (lk.lookat_decode_step, functools.partial(lk.lookat_probe_decode_step_entries, 1)):
        out1, cache1 = _run_step(lk, c, L, Lmax, 0xAB, single)
        assert torch.equal(cache, cache1)
        assert torch.equal(out, out1), "the paired instance must repeat the one-entry instance's arithmetic"


def test_decode_step_paired_entries_rejects_odd_batch_and_wide_heads(lk):
    c = _step_case("C2", 3, 2, 100, 70, 64, 4, "float16", 6990, "recipe")
    with pytest.raises(lk.LookatError):
        _run_step(lk, c, 70, 100, 0xAB, functools.partial(lk.lookat_probe_decode_step_entries, 2))
    with pytest.raises(lk.LookatError):
        _run_step(lk, c, 70, 100, 0xAB, functools.partial(lk.lookat_probe_decode_step_entries, 3))
    c = _step_case("C3", 2, 2, 100, 70, 128, 2, "float16", 6991, "recipe")   # one codebook row = 64 registers
    with pytest.raises(lk.LookatError):
        _run_step(lk, c, 70, 100, 0xAB, functools.partial(lk.lookat_probe_decode_step_entries, 2))


# (L, ranges): (700, 2) two ranges; (4133, 3) and (9000, 7) ragged last range; (1, 4) more ranges than keys;
# (4133, 0) the library's choice; (129, 2) and (385, 3): row L-1 alone in the last range; (128, 2) and (384, 3):
# row L-1 the last key of a full last range; (193, 3): the ranges are [0,128), [128,193), [192.. empty)
_SPLIT_CASES = [(700, 2), (4133, 3), (4133, 0), (9000, 7), (1, 4), (129, 2), (385, 3), (128, 2), (384, 3), (193, 3)]


@pytest.mark.parametrize("d_k,m", [(128, 8), (64, 4), (64, 16), (128, 2)])
@pytest.mark.parametrize("kind", ["recipe", "peaked", "aligned"])
@pytest.mark.parametrize("L,splits", _SPLIT_CASES)
def test_decode_step_split_matches_oracle(lk, d_k, m, kind, L, splits):
    """The fused step cut into ranges (few (b,h) pairs, long context): codes and outputs against the oracle,
    and the same codes as the one-range call."""
    B, H, Lmax = 1, 3, L + 40
    c = _step_case("C3", B, H, Lmax, L, d_k, m, "float32", 6300 + d_k + m + L, kind)
    call = lambda q, k, cb, codes, values, scale: lk.lookat_decode_step_split(q, k, cb, codes, values, scale,
                                                                             num_splits=splits)
    out, cache = _run_step(lk, c, L, Lmax, 0xCD, call)
    assert_out_close(out.cpu().numpy(), c["out"], f"decode_step_split, {kind} queries", c["scores"], c["scale"])
    cache2 = cache.clone()
    cache2[:, :, L - 1] = 0
    out1 = lk.lookat_decode_step(dev(c["q"]), dev(c["k_new"]), dev(c["cb"]), cache2[:, :, :L], dev(c["values"])[:, :, :L],
                                 c["scale"])
    assert torch.equal(cache2, cache)
    assert float((out1 - out).abs().max()) <= 1e-5


def test_decode_step_equals_three_calls(lk):
    """Same shape as one layer of the GPT-2-small batch-32 workload, reduced batch."""
    cfg = li.shrink(li.CONFIGS["C2"], B=4, n_calib=1024)
    case = li.make_case(cfg, seed=6100)
    cb = lk.lookat_kmeans(dev(case["calib"]), dev(case["cb_init"]), 2)
    scale = 0.125
    keys, values, q = dev(case["keys"]), dev(case["values"]), dev(case["q"]).float()   # one dtype for q and keys
    codes3 = lk.lookat_encode_keys(keys, cb)
    lut = lk.lookat_build_lut(q, cb)
    out3 = lk.lookat_attend_decode(lut.view(cfg.B, cfg.H, cfg.m, 256), codes3, values, scale)
    cache = codes3.clone()
    cache[:, :, -1] = 0
    out1 = lk.lookat_decode_step(q[:, :, 0], keys[:, :, -1], cb, cache, values, scale)
    assert torch.equal(cache, codes3)
    assert float((out1 - out3).abs().max()) <= 1e-5


# ---------------------------------------------------------------- grouped queries ----

# fp16 queries and keys over the whole grid; fp32 at the smaller groups and contexts
_STEP_GQA_CASES = [(dt, g, L, splits)
                   for dt in ("float16", "float32") for g in (2, 4, 8)
                   for (L, splits) in ((1, 0), (65, 0), (1024, 1), (3000, 3), (5000, 0))
                   if dt == "float16" or (g < 8 and L <= 1024)]


@pytest.mark.parametrize("d_k,m", [(128, 8), (64, 4), (64, 16), (128, 2)])
@pytest.mark.parametrize("kind", ["recipe", "peaked", "aligned"])
@pytest.mark.parametrize("qk_dtype,g,L,splits", _STEP_GQA_CASES)
def test_decode_step_gqa_matches_oracle(lk, d_k, m, g, L, splits, qk_dtype, kind):
    """Fused step with g query heads per key/value head: code cache and every query head's output against
    the oracle's three steps (encode per key/value head, tables per query head, grouped attention), on the
    three kinds of input of this section."""
    if kind != "recipe" and qk_dtype == "float32":
        pytest.skip("peaked and aligned inputs run in fp16 (the dtype only changes how q and k_new are read)")
    B, H, Lmax = 2, 2, L + 29
    c = _step_case("C3", B, H, Lmax, L, d_k, m, qk_dtype, 6500 + d_k + m + g + L, kind, g=g)
    call = lambda q, k, cb, codes, values, scale: lk.lookat_decode_step_gqa(q, k, cb, codes, values, scale,
                                                                           num_splits=splits)
    out, _ = _run_step(lk, c, L, Lmax, 0x5A, call)
    assert_out_close(out.cpu().numpy(), c["out"], f"decode_step_gqa, {kind} queries", c["scores"], c["scale"])



@pytest.mark.parametrize("d_k,m", [(128, 8), (64, 4), (128, 16), (64, 2), (64, 16)])
@pytest.mark.parametrize("g", [2, 4, 8])
@pytest.mark.parametrize("L,splits", [(1, 0), (65, 0), (300, 1), (1000, 3), (2500, 0)])
def test_attend_decode_gqa_parity(lk, d_k, m, g, L, splits):
    """g query heads per key/value head: scores and outputs of every query head against the oracle."""
    B, H = 2, 3
    rng = np.random.default_rng(9000 + d_k + m + g + L)
    d_sub = d_k // m
    cb = (rng.standard_normal((H, m, 256, d_sub)) * 0.7).astype(np.float32)
    codes = rng.integers(0, 256, size=(B, H, L, m), dtype=np.uint8)
    v = rng.standard_normal((B, H, L, d_k)).astype(np.float16)
    q = (rng.standard_normal((B, H * g, 1, d_k)) / 8).astype(np.float16)
    lut = oracle.build_lut(q, np.repeat(cb, g, axis=0))[:, :, 0]            # [B, H*g, m, 256]
    scale = 1.0 / math.sqrt(d_k)
    out_ref, s_ref = oracle.attend_decode_gqa(lut, codes, v, scale, want_scores=True)
    s_gpu = torch.empty((B, H * g, L), dtype=torch.float32, device="cuda")
    out = lk.lookat_attend_decode_gqa(dev(lut), dev(codes), dev(v), scale, num_splits=splits, scores_out=s_gpu)
    assert out.shape == (B, H * g, d_k)
    codes_q = np.repeat(codes, g, axis=1)                                   # codes as each query head sees them
    assert_scores_close(s_gpu.cpu().numpy(), lut, codes_q, s_ref)
    assert_out_close(out.cpu().numpy(), out_ref, "attend_decode_gqa", s_ref, scale)


@pytest.mark.parametrize("g", [4, 8])
@pytest.mark.parametrize("L,splits,lut_scale", [(8229, 0, 0.05), (16421, 1, 0.05), (16421, 0, 3.0), (9000, 2, 40.0)])
def test_attend_decode_gqa_matrix_core_sum_long_context(lk, g, L, splits, lut_scale):
    """d_k = 128 with 4 or 8 query heads per key/value head takes the weighted value sum on the matrix cores,
    the weights split into two fp16 halves.  Long contexts with a near-flat softmax (every weight about 1/L:
    the split's error would add up over 16 K keys), a peaked one, and one so peaked that most weights are
    below fp16's range: outputs to the arithmetic bar of tests/bars.py, scores to theirs."""
    B, H, d_k, m = 1, 2, 128, 8
    rng = np.random.default_rng(9200 + g + L + int(lut_scale * 10))
    lut = (rng.standard_normal((B, H * g, m, 256)) * lut_scale).astype(np.float32)
    codes = rng.integers(0, 256, size=(B, H, L, m), dtype=np.uint8)
    v = rng.standard_normal((B, H, L, d_k)).astype(np.float16)
    scale = 1.0 / math.sqrt(d_k)
    out_ref, s_ref = oracle.attend_decode_gqa(lut, codes, v, scale, want_scores=True)
    s_gpu = torch.empty((B, H * g, L), dtype=torch.float32, device="cuda")
    out = lk.lookat_attend_decode_gqa(dev(lut), dev(codes), dev(v), scale, num_splits=splits, scores_out=s_gpu)
    assert_scores_close(s_gpu.cpu().numpy(), lut, np.repeat(codes, g, axis=1), s_ref)
    assert_out_close(out.cpu().numpy(), out_ref, "attend_decode_gqa, matrix-core value sum, long context", s_ref, scale)


def test_attend_decode_gqa_equals_per_head_calls(lk):
    """The grouped kernel against lookat_attend_decode on caches repeated per query head, and
    on views of a longer cache."""
    B, H, g, L, Lmax, d_k, m = 2, 2, 4, 777, 1024, 128, 8
    rng = np.random.default_rng(9100)
    lut = dev((rng.standard_normal((B, H * g, m, 256)) * 2).astype(np.float32))
    cache_c = torch.randint(0, 256, (B, H, Lmax, m), dtype=torch.uint8, device="cuda")
    cache_v = torch.randn((B, H, Lmax, d_k), device="cuda").half()
    codes, values = cache_c[:, :, :L], cache_v[:, :, :L]
    out = lk.lookat_attend_decode_gqa(lut, codes, values, 0.09)
    ref = lk.lookat_attend_decode(lut, codes.repeat_interleave(g, dim=1).contiguous(),
                                  values.repeat_interleave(g, dim=1).contiguous(), 0.09)
    assert float((out - ref).abs().max()) <= 1e-5


@pytest.mark.parametrize("d_k,m", [(64, 4), (128, 8), (64, 16), (32, 2), (256, 8)])
@pytest.mark.parametrize("B,H,L,splits", [(2, 5, 1, 0), (2, 5, 65, 3), (3, 5, 777, 40), (1, 3, 4133, 0), (2, 3, 2049, 0),
                                          (48, 8, 200, 0), (25, 16, 130, 0), (1, 2, 9000, 5)])
def test_ticket_merge_probe_matches_oracle(lk, d_k, m, B, H, L, splits):
    """The measurement-aid kernel (flat geometry, pieces of a (b,h) merged in-kernel by ticket): scores and
    outputs against the oracle on shapes that give one piece per (b,h), ranges of a (b,h), shares of one and a
    half (b,h) (384 and 400 pairs on 256 compute units: tail + whole + head) and more ranges than tiles; two
    calls in a row on one workspace (the counters must come back to zero)."""
    rng = np.random.default_rng(9500 + d_k + m + B * H + L)
    lut, codes, v = _decode_case(rng, B, H, L, d_k, m, lut_scale=6.0)
    scale = 1.0 / math.sqrt(d_k)
    ref, s_ref = oracle.attend_decode(lut, codes, v, scale, want_scores=True)
    need = lk.probe_attend_decode_ticket_workspace_bytes(B, H, d_k, m, L, splits)
    ws = torch.zeros(max(need, 16), dtype=torch.uint8, device="cuda")
    lut_d, codes_d, v_d = dev(lut), dev(codes), dev(v)
    for call in range(2):
        scores = torch.empty((B, H, L), dtype=torch.float32, device="cuda")
        out, pieces = lk.lookat_probe_attend_decode_ticket(lut_d, codes_d, v_d, scale, num_splits=splits, workspace=ws,
                                                           scores_out=scores)
        assert (pieces > 1) == (need > 0)
        assert_out_close(out.cpu().numpy(), ref, "ticket-merge probe", s_ref, scale)
        assert_scores_close(scores.cpu().numpy(), lut, codes, s_ref)
    if need:
        tickets = ws[: B * H * 4].view(torch.int32)
        assert int(tickets.abs().max()) == 0, "ticket counters not back at zero"


# ---------------------------------------------------------------- seeded random shapes ----------

def _random_shape_cases(n, seed):
    """n seeded draws of (B, H, L, cache padding, (d_k, m), query heads per key/value head, ranges, dtype):
    combinations the hand-picked grids above do not enumerate (odd batch and head counts against every
    kernel instance, short and ragged contexts in padded caches, every group size with every split count)."""
    rng = np.random.default_rng(seed)
    shapes = [(64, 4), (64, 2), (64, 8), (64, 16), (128, 8), (128, 16), (128, 2), (128, 4)]
    cases = []
    for _ in range(n):
        d_k, m = shapes[int(rng.integers(len(shapes)))]
        B, H = int(rng.integers(1, 7)), int(rng.integers(1, 6))
        L = int([rng.integers(1, 130), rng.integers(130, 1200), rng.integers(1200, 4200)][int(rng.integers(3))])
        pad = int(rng.integers(0, 3)) * int(rng.integers(1, 90))
        g = int(rng.choice([1, 1, 2, 4, 8]))
        if g == 8 and m == 16:      # eight 16 KB tables and the reduction buffer exceed the 160 KB of LDS
            g = 4
        splits = int(rng.choice([0, 0, 1, 2, 3, 5]))
        dtype = ["float16", "float32"][int(rng.integers(2))]
        cases.append((B, H, L, pad, d_k, m, g, splits, dtype))
    return cases


@pytest.mark.parametrize("B,H,L,pad,d_k,m,g,splits,qk_dtype", _random_shape_cases(48, 20260110))
def test_random_shapes_three_calls_and_fused_step(lk, B, H, L, pad, d_k, m, g, splits, qk_dtype):
    """On each drawn shape: the three library calls (encode into a padded cache, tables, attention with
    scores, grouped or not, on views of the padded caches) and the fused step on a cache whose last row is
    stale, all against the oracle's three steps."""
    Lmax = L + pad
    c = _step_case("C3" if d_k == 128 else "C2", B, H, Lmax, L, d_k, m, qk_dtype, 9500 + B * 7 + H * 5 + L + m + g, "recipe", g=g)
    scale = c["scale"]
    # three calls, on views of caches with Lmax rows per (b,h)
    cache = torch.full((B, H, Lmax, m), 0x3C, dtype=torch.uint8, device="cuda")
    lk.lookat_encode_keys(dev(c["keys"]), dev(c["cb"]), cache=cache, position=0)
    got = cache.cpu().numpy()
    assert np.array_equal(got[:, :, :L], c["codes"]) and (got[:, :, L:] == 0x3C).all()
    values = dev(c["values"])                                   # [B,H,Lmax,d_k]
    cb_q = np.repeat(c["cb"], g, axis=0)
    lut_ref = oracle.build_lut(c["q"][:, :, None], cb_q)[:, :, 0]
    lut = lk.lookat_build_lut(dev(c["q"][:, :, None]), dev(cb_q)).view(B, H * g, m, 256)
    assert_lut_close(lut.cpu().numpy()[:, :, None], c["q"][:, :, None], cb_q, lut_ref[:, :, None])
    scores = torch.empty((B, H * g, L), dtype=torch.float32, device="cuda")
    lut_d = dev(lut_ref)                                        # attention from the oracle's table: one table, two readers
    if g == 1:
        out = lk.lookat_attend_decode(lut_d, cache[:, :, :L], values[:, :, :L], scale, num_splits=splits, scores_out=scores)
    else:
        out = lk.lookat_attend_decode_gqa(lut_d, cache[:, :, :L], values[:, :, :L], scale, num_splits=splits,
                                          scores_out=scores)
    assert_scores_close(scores.cpu().numpy(), lut_ref, np.repeat(c["codes"], g, axis=1), c["scores"])
    assert_out_close(out.cpu().numpy(), c["out"], "random shapes, attention", c["scores"], scale)
    # fused step
    if g == 1 and splits == 0:
        call = lk.lookat_decode_step
    elif g == 1:
        call = lambda q, k, cb, codes, vals, sc: lk.lookat_decode_step_split(q, k, cb, codes, vals, sc, num_splits=splits)
    else:
        call = lambda q, k, cb, codes, vals, sc: lk.lookat_decode_step_gqa(q, k, cb, codes, vals, sc, num_splits=splits)
    out2, _ = _run_step(lk, c, L, Lmax, 0x77, call)
    assert_out_close(out2.cpu().numpy(), c["out"], "random shapes, fused step", c["scores"], scale)


# ---------------------------------------------------------------- HIP graphs ----------


def _capture(fn):
    """fn recorded into a graph on torch's capture stream, after one warm-up call on a side stream."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        fn()
    torch.cuda.synchronize()
    return graph


@pytest.mark.parametrize("g,d_k,m,L,splits,B,H", [(4, 128, 8, 3000, 3, 2, 2), (1, 64, 4, 1024, 0, 2, 2), (2, 64, 16, 1537, 2, 2, 2),
                                                  (1, 64, 4, 800, 0, 22, 12)])
def test_decode_step_graph_replays_equal_eager(lk, g, d_k, m, L, splits, B, H):
    """The fused step (ranges plus merge kernel where it splits; in the last case the instance that serves two
    batch entries per workgroup, which the library takes at 264 (b,h)) recorded into a graph: every one of three
    replays, with eager launches of the same entry point on another context length and synchronisations in
    between, leaves the code cache and the outputs bit-identical to the eager call, which meets the oracle."""
    Lmax = L + 29
    if B * H > 256:
        assert g == 1 and lk.decode_step_entries_per_workgroup(B, H, d_k, m, L) == 2
    c = _step_case("C3", B, H, Lmax, L, d_k, m, "float16", 9100 + d_k + m + g + L, "recipe", g=g)
    q, k_new, cb, values = dev(c["q"]), dev(c["k_new"]), dev(c["cb"]), dev(c["values"])
    cache = torch.full((B, H, Lmax, m), 0x5A, dtype=torch.uint8, device="cuda")
    cache[:, :, :L - 1] = dev(c["codes"][:, :, :L - 1])
    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")
    out = torch.zeros((B, H * g, d_k), dtype=torch.float32, device="cuda")
    other = torch.zeros_like(out)

    def step():
        lk.lookat_decode_step_gqa(q, k_new, cb, cache[:, :, :L], values[:, :, :L], c["scale"], num_splits=splits,
                                  workspace=ws, out=out)

    step()
    torch.cuda.synchronize()
    eager_out, eager_cache = out.clone(), cache.clone()
    assert np.array_equal(eager_cache.cpu().numpy()[:, :, :L], c["codes"])
    assert_out_close(eager_out.cpu().numpy(), c["out"], "decode_step_gqa before capture", c["scores"], c["scale"])
    graph = _capture(step)
    for replay in range(3):
        cache[:, :, L - 1] = 0x5A
        out.fill_(float("nan"))
        ws.fill_(0xFF)
        # eager work of the program's own between the replays: the same entry point on a shorter context
        lk.lookat_decode_step_gqa(q, k_new, cb, cache[:, :, :L - 7], values[:, :, :L - 7], c["scale"],
                                  num_splits=splits, out=other)
        torch.cuda.synchronize()
        cache[:, :, L - 8] = eager_cache[:, :, L - 8]
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(cache, eager_cache), f"code cache after replay {replay}"
        assert torch.equal(out, eager_out), f"outputs after replay {replay}"


@pytest.mark.parametrize("q_dtype,T,L", [("float16", 96, 256), ("float32", 130, 333), ("float16", 8, 200)])
def test_score_prefill_graph_replays_equal_eager(lk, q_dtype, T, L):
    """Block scoring recorded into a graph (the matrix-core kernel for T >= 24, fp16 and split-fp32 queries;
    the lookup kernel below): three replays into a poisoned output, eager calls on another block in between."""
    cfg = li.shrink(li.CONFIGS["C4"], B=2, H=3, L=L, T=T, d_k=128, m=16, n_calib=400, q_dtype=q_dtype)
    case = li.make_case(cfg, seed=9200 + T)
    cb = case["cb_init"]
    codes = dev(oracle.encode_keys(case["keys"], cb))
    q, cbd = dev(case["q"]), dev(cb)
    scores = torch.zeros((2, 3, T, L), dtype=torch.float32, device="cuda")
    lk.lookat_score_prefill(q, cbd, codes, scores_out=scores)
    torch.cuda.synchronize()
    eager = scores.clone()
    lut_ref = oracle.build_lut(case["q"], cb)
    _prefill_bars(eager.cpu().numpy(), oracle.score_prefill(lut_ref, codes.cpu().numpy()), case["q"], cb,
                  codes.cpu().numpy(), lut_ref, "score_prefill, before capture")
    graph = _capture(lambda: lk.lookat_score_prefill(q, cbd, codes, scores_out=scores))
    for replay in range(3):
        scores.fill_(float("nan"))
        lk.lookat_score_prefill(q[:, :, :T - 3].contiguous(), cbd, codes[:, :, :L - 5])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(scores, eager), f"scores after replay {replay}"


def test_probe_stream_read_shapes_run(lk):
    """Every launch shape of the read probe streams the buffer without writing anything."""
    buf = torch.arange(1 << 18, dtype=torch.int32, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    for threads in (64, 256, 1024):
        for loads in (1, 8, 16):
            for wgs, contig in ((0, False), (7, False), (7, True)):
                lk.lookat_probe_stream_read_shaped(buf, sink, threads, loads, wgs, contig, True)
    lk.lookat_probe_empty_launch(384, 256)
    torch.cuda.synchronize()
    assert int(sink.abs().max()) == 0


def test_probe_stream_write_fills_exactly_the_buffer(lk):
    buf = torch.zeros(4096 + 8, dtype=torch.int32, device="cuda")
    lk.lookat_probe_stream_write(buf[4:4 + 4096], 0x5A5A1234)
    torch.cuda.synchronize()
    host = buf.cpu().numpy()
    assert (host[4:4 + 4096] == 0x5A5A1234).all() and (host[:4] == 0).all() and (host[-4:] == 0).all()
