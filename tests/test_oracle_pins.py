"""Pins for the CPU oracle: what the paper and the mathematics fix, checked without any GPU code.

Every check compares the oracle with something other than itself: brute force written here in pure Python/numpy,
numpy's own matmul / float16 conversion, closed forms printed in the paper (tests/golden/), or invariants.
"""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
from paper_2305_10727_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split()
            try:
                k = float(k)
            except ValueError:
                pass
            out[k] = float(v)
    return out


# ------------------------------------------------------------------ brute force helpers (independent of the oracle)
PAIRS = list(itertools.combinations(range(4), 2))  # lexicographic order


def brute_top2(mags):
    """max sum of magnitudes over the 6 index pairs; lexicographically smallest pair among the maxima"""
    best, best_pair = None, None
    for pr in PAIRS:
        s = mags[pr[0]] + mags[pr[1]]
        if best is None or s > best:
            best, best_pair = s, pr
    return best_pair


def brute_prune(W):
    W = np.asarray(W)
    out = np.zeros_like(W)
    mask = np.zeros((W.shape[0], W.shape[1] // 4), np.uint8)
    for n in range(W.shape[0]):
        for g in range(W.shape[1] // 4):
            grp = W[n, 4 * g:4 * g + 4]
            mags = [abs(float(v)) for v in grp]
            p0, p1 = brute_top2(mags)
            out[n, 4 * g + p0] = grp[p0]
            out[n, 4 * g + p1] = grp[p1]
            mask[n, g] = (1 << p0) | (1 << p1)
    return out, mask


def adversarial_groups(dtype):
    tiny = np.finfo(dtype).tiny
    sub = np.finfo(dtype).smallest_subnormal
    rows = [
        [0, 0, 0, 0], [-0.0, 0.0, -0.0, 0.0], [1, 1, 1, 1], [-1, 1, -1, 1], [1, 2, 2, 1], [2, 1, 1, 2], [3, 3, 1, 3],
        [1, 3, 3, 3], [0, 0, 0, 5], [0, 0, 5, 0], [5, 0, 0, 0], [sub, 0, 0, sub], [sub, 2 * sub, tiny, -tiny],
        [-tiny, tiny, sub, -sub], [1, -1, 0.5, -0.5], [0.5, -1, 1, 0.5], [6e4, 1, -6e4, 2], [4, 3, 2, 1],
        [1, 2, 3, 4], [2, 2, 3, 3], [-0.0, 0, 1, 0],
    ]
    return np.array(rows, dtype=dtype).reshape(1, -1)


# ------------------------------------------------------------------ a1 prune
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_prune_matches_brute_force(dtype):
    rng = np.random.default_rng(1)
    cases = [
        rng.standard_normal((7, 64)).astype(dtype),
        rng.integers(-2, 3, size=(16, 128)).astype(dtype),  # many ties
        adversarial_groups(dtype),
    ]
    grid = np.array(list(itertools.product(range(-2, 3), repeat=4)), dtype=dtype).reshape(5, -1)  # exhaustive {-2..2}^4
    cases.append(grid)
    for W in cases:
        got, mask = oracle.prune_2to4(W)
        exp, emask = brute_prune(W)
        assert np.array_equal(mask, emask)
        assert np.array_equal(got.view(np.uint32 if dtype == np.float32 else np.uint16),
                              exp.view(np.uint32 if dtype == np.float32 else np.uint16)) or \
            np.array_equal(np.where(got == 0, 0, got), np.where(exp == 0, 0, exp))
        # dropped entries are written as +0.0
        dropped = np.repeat(np.unpackbits(mask[..., None], axis=-1, bitorder="little")[..., :4].reshape(W.shape) == 0, 1, axis=1)
        bits = got.view(np.uint32 if dtype == np.float32 else np.uint16)
        assert (bits[dropped] == 0).all()


def test_prune_invariants():
    W = synth.weights(96, 192, seed=3)
    P, mask = oracle.prune_2to4(W)
    # exactly two kept positions per group, at most two non-zeros, kept entries unchanged
    assert (np.unpackbits(mask[..., None], axis=-1).sum(-1) == 2).all()
    assert ((P.reshape(96, -1, 4) != 0).sum(-1) <= 2).all()
    assert ((P == W) | (P == 0)).all()
    # optimal: kept magnitude sum >= that of any other pair
    a = np.abs(W).reshape(96, -1, 4)
    kept = np.abs(P).reshape(96, -1, 4).sum(-1)
    for p0, p1 in PAIRS:
        assert (kept >= a[..., p0] + a[..., p1]).all()
    # idempotent
    P2, mask2 = oracle.prune_2to4(P)
    assert np.array_equal(P2, P) and np.array_equal(mask2, mask)
    # half of the entries survive
    assert (P != 0).sum() == W.size // 2
    with pytest.raises(ValueError):
        oracle.prune_2to4(np.zeros((2, 6), np.float32))
    # infinities are simply the largest magnitudes
    Pinf, minf = oracle.prune_2to4(np.array([[np.inf, 1, -np.inf, 2]], np.float32))
    assert minf[0, 0] == 0b0101 and np.isinf(Pinf[0, [0, 2]]).all()


# ------------------------------------------------------------------ a3 compress / decompress
def brute_compress(W):
    N, K = W.shape
    vals = np.zeros((N, K // 2), W.dtype)
    meta = np.zeros((N, (K // 4 + 1) // 2), np.uint8)
    viol = 0
    for n in range(N):
        for g in range(K // 4):
            grp = W[n, 4 * g:4 * g + 4]
            mags = [abs(float(v)) for v in grp]
            p0, p1 = brute_top2(mags)
            vals[n, 2 * g], vals[n, 2 * g + 1] = grp[p0], grp[p1]
            meta[n, g // 2] |= (p0 | (p1 << 2)) << (4 * (g & 1))
            viol += any(mags[i] != 0 for i in range(4) if i not in (p0, p1))
    return vals, meta, viol


@pytest.mark.parametrize("dtype", [np.float16, np.int8])
def test_compress_matches_brute_force_and_round_trips(dtype):
    rng = np.random.default_rng(2)
    if dtype == np.int8:
        dense = rng.integers(-127, 128, size=(9, 72)).astype(np.int8)
        ties = rng.integers(-1, 2, size=(9, 72)).astype(np.int8)
    else:
        dense = rng.standard_normal((9, 72)).astype(np.float16)
        ties = rng.integers(-1, 2, size=(9, 72)).astype(np.float16)
    for W in (dense, ties):
        v, m, viol = oracle.compress(W)
        ev, em, eviol = brute_compress(W)
        assert np.array_equal(v, ev) and np.array_equal(m, em) and viol == eviol
        # every nibble: first position < second position
        nib = np.stack([m & 0xF, m >> 4], -1).reshape(m.shape[0], -1)[:, :W.shape[1] // 4]
        assert ((nib & 3) < (nib >> 2)).all()
    # round trip on a tensor that already is 2:4: identity, no violations
    W32 = rng.standard_normal((9, 72)).astype(np.float32)
    P, _ = oracle.prune_2to4(W32)
    Wp = (np.clip(np.rint(P * 50), -127, 127).astype(np.int8)) if dtype == np.int8 else P.astype(np.float16)
    v, m, viol = oracle.compress(Wp)
    assert viol == 0
    back = oracle.decompress(v, m, Wp.shape[1])
    assert np.array_equal(back, Wp)
    # compress o decompress is the identity on the values
    v2, m2, _ = oracle.compress(back)
    assert np.array_equal(v2, v)
    # a dense tensor is reported as violating
    assert oracle.compress(dense)[2] > 0


def test_storage_closed_forms_from_paper():
    g = read_golden("storage_savings.txt")
    N, K = 64, 256
    for dtype, key in ((np.float16, "fp16_saving_percent"), (np.int8, "int8_saving_percent")):
        W = np.zeros((N, K), dtype)
        v, m, _ = oracle.compress(W)
        dense_bytes = W.nbytes
        comp_bytes = v.nbytes + m.nbytes
        assert v.shape == (N, int(K * g["kept_fraction_of_K"]))
        assert m.nbytes * 8 == v.size * g["metadata_bits_per_kept_value"]
        assert 100.0 * (1.0 - comp_bytes / dense_bytes) == pytest.approx(g[key], abs=1e-12)
    # fp32 dense model vs int8 2:4 model
    v, m, _ = oracle.compress(np.zeros((N, K), np.int8))
    assert (N * K * 4) / (v.nbytes + m.nbytes) == pytest.approx(g["fp32_dense_over_int8_2to4_size_ratio"], abs=1e-12)


# ------------------------------------------------------------------ fp16 conversion
def test_f16_conversions_against_numpy():
    allbits = np.arange(65536, dtype=np.uint16)
    as32 = allbits.view(np.float16).astype(np.float32)
    for h in list(range(0, 65536, 97)) + [0, 1, 0x3FF, 0x400, 0x7BFF, 0x7C00, 0x8000, 0x8001, 0xFBFF, 0xFC00]:
        f = oracle.f16_to_f32(h)
        assert f == as32[h] or (math.isnan(f) and math.isnan(as32[h]))
        if not math.isnan(f):
            assert oracle.f32_to_f16(f) == h
    rng = np.random.default_rng(5)
    xs = np.concatenate([
        rng.standard_normal(4000).astype(np.float32) * np.float32(10.0) ** rng.integers(-9, 6, 4000).astype(np.float32),
        np.array([65504, 65519.99, 65520, 1e9, 6.1e-5, 6.103515625e-05, 5.96e-8, 2.98e-8, 2.9802322e-8, 2.99e-8, 8.94e-8,
                  1.0009765625, 1.00048828125, 1.00146484375, 2049, 2051, -0.0, 0.0], np.float32)])
    with np.errstate(over="ignore"):
        exp = xs.astype(np.float16).view(np.uint16)
    for x, e in zip(xs, exp):
        assert oracle.f32_to_f16(x) == e, (x, e)
    # from a double: ties decided once, in fp64 (1 + 2^-11 + 2^-30 must round up although its fp32 image is a tie)
    assert oracle.f64_to_f16(1.0 + 2.0 ** -11) == 0x3C00
    assert oracle.f64_to_f16(1.0 + 2.0 ** -11 + 2.0 ** -30) == 0x3C01
    assert oracle.f64_to_f16(1.0 + 3 * 2.0 ** -11) == 0x3C02


# ------------------------------------------------------------------ a2 / a4 quantise
def test_quantize_properties():
    W = synth.weights(64, 128, seed=7)
    P, _ = oracle.prune_2to4(W)
    q, s = oracle.quantize_rows_int8(P)
    q_dense, s_dense = oracle.quantize_rows_int8(W)
    # the row maximum always survives pruning, so the per-channel scale does not change
    assert np.array_equal(s, s_dense)
    assert np.array_equal(s, (np.abs(W).max(1) / np.float32(127.0)).astype(np.float32))
    assert np.abs(q.astype(np.int32)).max() == 127 and q.min() >= -127
    # the row maximum maps to +-127 exactly; error bound s/2 (plus fp32 rounding of the division)
    assert (np.abs(q).max(1) == 127).all()
    err = np.abs(P.astype(np.float64) - s[:, None].astype(np.float64) * q)
    assert (err <= 0.5 * s[:, None] * (1 + 1e-6)).all()
    # zeros stay zero: the quantised tensor is still 2:4
    assert ((q.reshape(64, -1, 4) != 0).sum(-1) <= 2).all()
    # integers with amax 127 are reproduced exactly (scale 1)
    Z = np.random.default_rng(0).integers(-127, 128, size=(5, 32)).astype(np.float32)
    Z[:, 0] = 127
    qz, sz = oracle.quantize_rows_int8(Z)
    assert (sz == 1).all() and np.array_equal(qz, Z.astype(np.int8))
    # all-zero row: scale 1, codes 0
    qz, sz = oracle.quantize_rows_int8(np.zeros((2, 8), np.float32))
    assert (sz == 1).all() and (qz == 0).all()
    # round-half-even: x/s exactly k + 0.5
    X = np.array([[127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5]], np.float32)
    qh, sh = oracle.quantize_rows_int8(X)
    assert sh[0] == 1 and list(qh[0]) == [127, 0, 2, 2, 0, -2, -2, 126]
    # static scale: clamps at +-127
    qs, _ = oracle.quantize_rows_int8(np.array([[1000.0, -1000.0, 3.0, -3.49]], np.float32), scale=np.array([1.0], np.float32))
    assert list(qs[0]) == [127, -127, 3, -3]


def test_quantize_tensor_matches_numpy_float64_rounding():
    X = synth.activations(197, 192, "normal_clip4", seed=0)
    q, s = oracle.quantize_tensor_int8(X)
    assert np.float32(s) == np.float32(np.abs(X).max()) / np.float32(127.0)
    # fp32 division then rint; compare with numpy's own fp32 division and rint (both IEEE)
    exp = np.clip(np.rint(X / np.float32(s)), -127, 127).astype(np.int8)
    assert np.array_equal(q, exp)
    assert np.abs(q.astype(int)).max() == 127
    assert (np.abs(X - np.float64(s) * q) <= 0.5 * s * (1 + 1e-6)).all()
    q2, s2 = oracle.quantize_tensor_int8(X, scale=0.05)
    assert s2 == np.float32(0.05) and np.array_equal(q2, np.clip(np.rint(X / np.float32(0.05)), -127, 127).astype(np.int8))


# ------------------------------------------------------------------ a5 GEMM
def _int8_problem(M, K, N, seed):
    X = synth.activations(M, K, "normal_clip4", seed=seed, ids=(1,))
    W = synth.weights(N, K, seed=seed, ids=(1,))
    P, _ = oracle.prune_2to4(W)
    Wq, s_w = oracle.quantize_rows_int8(P)
    Xq, s_a = oracle.quantize_tensor_int8(X)
    vals, meta, viol = oracle.compress(Wq)
    assert viol == 0
    return Xq, s_a, Wq, s_w, vals, meta


def test_int8_sparse_gemm_equals_dense_on_masked_weights_and_numpy():
    Xq, s_a, Wq, s_w, vals, meta = _int8_problem(37, 192, 48, seed=11)
    dense = oracle.gemm_int8_dense(Xq, Wq)
    sparse = oracle.spgemm_int8(Xq, vals, meta)
    ref = Xq.astype(np.int64) @ Wq.astype(np.int64).T
    assert np.array_equal(dense, ref)  # numpy's matmul: catches a transposed operand or a wrong stride
    assert np.array_equal(sparse, dense)  # the sparse form computes the same C
    # extreme values: no saturation, plain int32 wrap-free accumulation
    Xe = np.full((3, 64), -127, np.int8); We = np.zeros((5, 64), np.int8); We[:, 0::4] = 127; We[:, 3::4] = -127
    v, m, _ = oracle.compress(We)
    assert np.array_equal(oracle.spgemm_int8(Xe, v, m), Xe.astype(np.int64) @ We.astype(np.int64).T)


def test_sparse_gemm_special_cases_pin_the_metadata():
    rng = np.random.default_rng(4)
    K, N = 64, 24
    W = rng.integers(-9, 10, size=(N, K)).astype(np.float32)
    P, mask = oracle.prune_2to4(W)
    Wq = P.astype(np.int8)
    vals, meta, _ = oracle.compress(Wq)
    # X = identity: the product returns the decompressed weight matrix, transposed
    I = np.eye(K, dtype=np.int8)
    assert np.array_equal(oracle.spgemm_int8(I, vals, meta), Wq.T.astype(np.int32))
    # all kept values = 1: each output is the sum of the X entries at the kept positions
    ones = np.ones_like(vals)
    X = rng.integers(-5, 6, size=(7, K)).astype(np.int8)
    keep = np.unpackbits(mask[..., None], axis=-1, bitorder="little")[..., :4].reshape(N, K)
    # positions recorded by compress (zeros filled lowest-index-first) may differ from the prune mask only where the
    # kept value is zero; recompute the positions from the metadata itself, by hand
    pos = np.zeros((N, K), np.int64)
    for n in range(N):
        for g in range(K // 4):
            nib = (meta[n, g // 2] >> (4 * (g & 1))) & 0xF
            pos[n, 4 * g + (nib & 3)] += 1
            pos[n, 4 * g + (nib >> 2)] += 1
    assert np.array_equal(oracle.spgemm_int8(X, ones, meta), X.astype(np.int64) @ pos.T)
    assert ((pos == 1) >= (Wq != 0)).all() and ((keep == 1) >= (Wq != 0)).all()


def test_fp16_gemm_exact_on_small_integers_and_close_on_gaussians():
    K, N, M = 256, 40, 23
    X = synth.small_integers((M, K), -4, 4, seed=1).astype(np.float16)
    W = synth.small_integers((N, K), -4, 4, seed=2).astype(np.float32)
    P, _ = oracle.prune_2to4(W)
    Wh = P.astype(np.float16)
    vals, meta, viol = oracle.compress(Wh)
    assert viol == 0
    ref = X.astype(np.float64) @ Wh.astype(np.float64).T  # exact: all partial sums are small integers
    d32, d64 = oracle.gemm_fp16_dense(X, Wh)
    s32, s64 = oracle.spgemm_fp16(X, vals, meta)
    for a in (d32, d64, s32, s64):
        assert np.array_equal(a.astype(np.float64), ref)
    # Gaussian data: fp64 accumulation agrees with numpy's float64 matmul; fp32 sequential sum within K*eps*sum|terms|
    Xg = synth.activations(M, K, seed=3).astype(np.float16)
    Wg, _ = oracle.prune_2to4(synth.weights(N, K, seed=3))
    Wg = Wg.astype(np.float16)
    vals, meta, _ = oracle.compress(Wg)
    ref = Xg.astype(np.float64) @ Wg.astype(np.float64).T
    bound = np.abs(Xg.astype(np.float64)) @ np.abs(Wg.astype(np.float64)).T
    d32, d64 = oracle.gemm_fp16_dense(Xg, Wg)
    s32, s64 = oracle.spgemm_fp16(Xg, vals, meta)
    assert np.abs(d64 - ref).max() <= 1e-13 * bound.max() * K
    assert np.abs(s64 - ref).max() <= 1e-13 * bound.max() * K
    assert (np.abs(d32 - ref) <= K * 2.0 ** -24 * bound + 1e-30).all()
    assert (np.abs(s32 - ref) <= K * 2.0 ** -24 * bound + 1e-30).all()


# ------------------------------------------------------------------ a6 epilogue
def test_epilogue_special_cases_and_gelu_table():
    cdf = read_golden("normal_cdf.txt")
    xs = sorted(float(k) for k in cdf)
    # acc = x * 1024, s_a * s_w = 2^-10 (exact): v = x; GELU(x) = x * Phi(x)
    acc = np.array([[int(x * 1024) for x in xs]], np.int32)
    s_w = np.full(len(xs), np.float32(1.0), np.float32)
    out = oracle.epilogue_int8_f64(acc, 2.0 ** -10, s_w, None, gelu=True)
    for j, x in enumerate(xs):
        assert out["ref"][0, j] == pytest.approx(x * cdf[x], rel=2e-9, abs=1e-12)
    out32 = oracle.epilogue_int8_f32(acc, 2.0 ** -10, s_w, None, gelu=True)
    for j, x in enumerate(xs):
        assert out32["v32"][0, j] == pytest.approx(x * cdf[x], rel=1e-7, abs=1e-12)
    # identity epilogue on exactly representable numbers
    acc = np.arange(-2048, 2049, dtype=np.int32).reshape(1, -1)
    one = np.ones(acc.shape[1], np.float32)
    o = oracle.epilogue_int8_f64(acc, 1.0, one, None, gelu=False)
    assert np.array_equal(o["y16"].astype(np.int32), acc) and np.array_equal(o["ref"], acc.astype(np.float64))
    # bias and per-channel scale are applied along n, not m (asymmetric shapes catch a transposed index)
    acc = np.array([[1, 2, 3], [4, 5, 6]], np.int32)
    s_w = np.array([1.0, 0.5, 0.25], np.float32); b = np.array([10.0, 20.0, 30.0], np.float32)
    o = oracle.epilogue_int8_f64(acc, 2.0, s_w, b, gelu=False, out_scale=0.5)
    assert np.array_equal(o["ref"], np.array([[12.0, 22.0, 31.5], [18.0, 25.0, 33.0]]))
    assert np.array_equal(o["q8"], np.array([[24, 44, 63], [36, 50, 66]], np.int8))
    o32 = oracle.epilogue_int8_f32(acc, 2.0, s_w, b, gelu=False, out_scale=0.5)
    assert np.array_equal(o32["v32"].astype(np.float64), o["ref"]) and np.array_equal(o32["q8"], o["q8"])
    # GELU limits: GELU(0) = 0, identity for large x, vanishing for very negative x
    acc = np.array([[0, 8000, -8000]], np.int32)
    o = oracle.epilogue_int8_f64(acc, 0.001, np.ones(3, np.float32), None, gelu=True)
    assert o["ref"][0, 0] == 0 and o["ref"][0, 1] == pytest.approx(8.0, rel=1e-6) and abs(o["ref"][0, 2]) < 1e-12
    # fp16 path: bias added along n
    o = oracle.epilogue_fp16_f64(np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]]), b, gelu=False)
    assert np.array_equal(o["ref"], np.array([[11.0, 22.0, 33.0], [14.0, 25.0, 36.0]]))
    assert np.array_equal(o["y16"].astype(np.float64), o["ref"])


def test_fp16_epilogue_gelu_follows_the_bias_and_matches_the_table():
    """FP16 path with GELU: the bias is added first, then the activation [Sec. 2.2: GELU is the feed-forward activation,
    applied to the layer's output].  acc[m][n] = x_n - b_n with a different non-zero exactly representable b_n per
    channel, so acc + bias = x_n exactly and the result must be x_n * Phi(x_n) from the table; activation-then-bias,
    a dropped bias, a bias indexed along m, or a tanh-form GELU all miss the table by far more than the tolerance."""
    cdf = read_golden("normal_cdf.txt")
    xs = sorted(float(k) for k in cdf)
    b = np.array([0.25 * (j + 1) * (-1) ** j for j in range(len(xs))], np.float32)  # 0.25, -0.5, 0.75, ...
    acc = np.stack([np.array(xs) - b.astype(np.float64), np.array(xs[::-1]) - b.astype(np.float64)])
    o = oracle.epilogue_fp16_f64(acc, b, gelu=True)
    for j, x in enumerate(xs):
        assert o["ref"][0, j] == pytest.approx(x * cdf[x], rel=2e-9, abs=1e-12)
        xr = xs[len(xs) - 1 - j]
        assert o["ref"][1, j] == pytest.approx(xr * cdf[xr], rel=2e-9, abs=1e-12)
    # the fp16 result is the fp64 value rounded once (numpy's conversion as the independent rounding)
    assert np.array_equal(o["y16"].view(np.uint16), o["ref"].astype(np.float16).view(np.uint16))
    # the wrong orders really are distinguishable on this input
    wrong = np.array([(x - float(bj)) * cdf.get(x, 0.5) + float(bj) for x, bj in zip(xs, b)])
    assert np.abs(wrong - o["ref"][0]).max() > 1e-2
    # without GELU the same call returns acc + bias
    o = oracle.epilogue_fp16_f64(acc, b, gelu=False)
    assert np.array_equal(o["ref"][0], np.array(xs)) and np.array_equal(o["ref"][1], np.array(xs[::-1]))
    # limits: GELU(0) = 0, identity for large x, vanishing for very negative x
    o = oracle.epilogue_fp16_f64(np.array([[-1.0, 7.0, -9.0]]), np.array([1.0, 1.0, 1.0], np.float32), gelu=True)
    assert o["ref"][0, 0] == 0 and o["ref"][0, 1] == pytest.approx(8.0, rel=1e-12) and abs(o["ref"][0, 2]) < 1e-12


def test_epilogue_fp32_sequence_within_one_fp16_ulp_of_fp64():
    Xq, s_a, Wq, s_w, vals, meta = _int8_problem(29, 128, 64, seed=21)
    acc = oracle.spgemm_int8(Xq, vals, meta)
    b = synth.bias(64, seed=21)
    for gelu in (False, True):
        o64 = oracle.epilogue_int8_f64(acc, s_a, s_w, b, gelu=gelu)
        o32 = oracle.epilogue_int8_f32(acc, s_a, s_w, b, gelu=gelu)
        assert np.abs(o32["v32"] - o64["ref"]).max() <= 4e-7 * np.abs(o64["ref"]).max()
        d = np.abs(o32["y16"].view(np.int16).astype(np.int32) - o64["y16"].view(np.int16).astype(np.int32))
        assert d.max() <= 1
    # whole-layer helper used for timing = spgemm + fp64 epilogue
    y = oracle.linear_int8_sparse(Xq, vals, meta, s_a, s_w, b, gelu=True)
    assert np.array_equal(y.view(np.uint16), oracle.epilogue_int8_f64(acc, s_a, s_w, b, gelu=True)["y16"].view(np.uint16))


def test_end_to_end_dequantised_layer_approximates_the_float_layer():
    """prune -> quantise -> compress -> sparse GEMM -> dequant reproduces X @ prune(W)^T to quantisation accuracy"""
    M, K, N = 64, 192, 96
    X = synth.activations(M, K, "normal_clip4", seed=5)
    W = synth.weights(N, K, seed=5)
    P, _ = oracle.prune_2to4(W)
    Wq, s_w = oracle.quantize_rows_int8(P)
    Xq, s_a = oracle.quantize_tensor_int8(X)
    vals, meta, _ = oracle.compress(Wq)
    acc = oracle.spgemm_int8(Xq, vals, meta)
    y = oracle.epilogue_int8_f64(acc, s_a, s_w, None)["ref"]
    ref = X.astype(np.float64) @ P.astype(np.float64).T
    assert np.abs(y - ref).max() / np.abs(ref).max() < 0.03
    assert np.corrcoef(y.ravel(), ref.ravel())[0, 1] > 0.999


# ---------------------------------------------------------------- patch embedding (strided convolution, Sec. 3.3)
def _patches(img, P):
    """reshape-and-transpose form of cutting [B,C,H,W] into flattened P x P patches: rows (b, py, px), columns (c, i, j)"""
    B, C, H, W = img.shape
    return img.reshape(B, C, H // P, P, W // P, P).transpose(0, 2, 4, 1, 3, 5).reshape(B * (H // P) * (W // P), C * P * P)


def test_patch_convolution_equals_matmul_on_flattened_patches_and_counts_the_papers_flops():
    golden = dict(l.split() for l in open(os.path.join(GOLDEN, "patch_embedding_flops.txt")) if l.strip() and not l.startswith("#"))
    per_mac = int(golden["flops_per_multiply_accumulate"])
    rng = np.random.default_rng(7)
    for B, C, H, W, P, D in [(2, 3, 8, 12, 4, 5), (1, 3, 14, 28, 14, 6), (3, 1, 6, 6, 1, 4), (2, 2, 16, 16, 16, 3)]:
        img = rng.integers(-127, 128, (B, C, H, W), dtype=np.int8)
        Wc = rng.integers(-127, 128, (D, C, P, P), dtype=np.int8)
        acc, macs = oracle.patch_conv_int8(img, Wc)
        assert per_mac * macs == 2 * B * C * H * W * D            # the count printed in Sec. 3.3
        ref = _patches(img, P).astype(np.int64) @ Wc.reshape(D, -1).astype(np.int64).T
        assert np.array_equal(acc, ref)
        img16 = rng.standard_normal((B, C, H, W)).astype(np.float16)
        W16 = (rng.standard_normal((D, C, P, P)) * 0.1).astype(np.float16)
        a64, macs16 = oracle.patch_conv_f16(img16, W16)
        assert macs16 == macs
        ref64 = _patches(img16, P).astype(np.float64) @ W16.reshape(D, -1).astype(np.float64).T
        assert np.allclose(a64, ref64, rtol=1e-12, atol=1e-12)


def test_patch_convolution_special_cases():
    rng = np.random.default_rng(8)
    # one patch covering the whole image: a plain dot product per output channel
    img = rng.integers(-127, 128, (1, 3, 4, 4), dtype=np.int8)
    Wc = rng.integers(-127, 128, (2, 3, 4, 4), dtype=np.int8)
    acc, _ = oracle.patch_conv_int8(img, Wc)
    assert acc.shape == (1, 2)
    assert acc[0, 1] == int((img[0].astype(np.int64) * Wc[1].astype(np.int64)).sum())
    # locality: one pixel only influences the token of its own patch
    img = rng.integers(-100, 100, (2, 3, 8, 8), dtype=np.int8)
    Wc = rng.integers(1, 100, (4, 3, 4, 4), dtype=np.int8)
    a0, _ = oracle.patch_conv_int8(img, Wc)
    img2 = img.copy()
    img2[1, 2, 5, 2] += 1                                         # image 1, patch row 1, patch column 0
    a1, _ = oracle.patch_conv_int8(img2, Wc)
    changed = np.nonzero((a0 != a1).any(axis=1))[0]
    assert changed.tolist() == [1 * 4 + 1 * 2 + 0]
    assert np.array_equal(a1[6] - a0[6], Wc[:, 2, 1, 2].astype(np.int32))   # by exactly the weight at (c=2, i=1, j=2)
    # shape errors
    assert oracle.lib().oracle_patch_conv_int8(None, None, None, 1, 1, 5, 4, 2, 1) == -1


# ------------------------------------------------------------------ INT4 pair-wise 4:8 [Sec. 3.1]
def test_int4_pairwise_prune_matches_brute_force_and_keeps_whole_sub_chunks():
    rng = np.random.default_rng(41)
    N, K = 24, 64
    cases = [rng.standard_normal((N, K)).astype(np.float32),
             rng.integers(-3, 4, (N, K)).astype(np.float32)]  # a small grid: many tied scores
    for W in cases:
        P, mask = oracle.prune_4to8_pairs(W)
        for n in range(N):
            for c in range(K // 8):
                w = W[n, 8 * c:8 * c + 8]
                score = [float(np.float32(abs(w[2 * p])) + np.float32(abs(w[2 * p + 1]))) for p in range(4)]
                best = max(score[i] + score[j] for i, j in PAIRS)
                i, j = min(pr for pr in PAIRS if score[pr[0]] + score[pr[1]] == best)
                assert mask[n, c] == (1 << i) | (1 << j)
                exp = np.zeros(8, np.float32)
                exp[2 * i:2 * i + 2] = w[2 * i:2 * i + 2]
                exp[2 * j:2 * j + 2] = w[2 * j:2 * j + 2]
                assert np.array_equal(P[n, 8 * c:8 * c + 8], exp)
        # pattern invariants: exactly two sub-chunks kept, the kept ones never score below a dropped one
        assert all(bin(int(b)).count("1") == 2 for b in mask.ravel())
        nz = (P.reshape(N, K // 2, 2) != 0).any(axis=2).reshape(N, K // 8, 4).sum(axis=2)
        assert (nz <= 2).all()


def test_int4_pairwise_worked_example_and_storage_saving():
    """w, x, y, z = the non-zeros of a chunk, clustered in two sub-chunks (Sec. 3.1): the compressed row holds w x y z and
    the two sub-chunk positions.  Bytes written out by hand from the format's definition."""
    row = np.array([[0, 0, 3, -2, 0, 0, 7, 1, 5, -6, 0, 0, -1, 4, 0, 0]], np.int8)
    values, meta, viol = oracle.compress_int4_pairs(row)
    assert viol == 0
    assert values.tolist() == [[0xE3, 0x17, 0xA5, 0x4F]]   # (3,-2) (7,1) | (5,-6) (-1,4): low nibble first, two's complement
    assert meta.tolist() == [[0x0D | (0x08 << 4)]]          # sub-chunks (1,3) -> 1 | 3<<2 ; (0,2) -> 0 | 2<<2, second chunk high
    assert np.array_equal(oracle.decompress_int4_pairs(values, meta, 16), row)
    # a non-zero outside the two kept sub-chunks, and a code outside the 4-bit range, are violations
    bad = row.copy()
    bad[0, 0] = 1
    assert oracle.compress_int4_pairs(bad)[2] == 1
    bad = row.copy()
    bad[0, 9] = -9
    assert oracle.compress_int4_pairs(bad)[2] == 1
    g = read_golden("storage_savings.txt")
    N, K = 64, 256
    v, m, _ = oracle.compress_int4_pairs(np.zeros((N, K), np.int8))
    dense_int4_bytes = N * K // 2
    assert m.nbytes * 8 == (N * K // 8) * g["int4_index_bits_per_chunk_of_8"]
    assert 100.0 * (1.0 - (v.nbytes + m.nbytes) / dense_int4_bytes) == pytest.approx(g["int4_saving_percent"], abs=1e-12)
    # whole models also hold uncompressed parts, so the printed ratio lies a little below the format's own 12.8
    assert (N * K * 4) / (v.nbytes + m.nbytes) == pytest.approx(g["fp32_dense_over_int4_size_ratio_printed"], abs=0.15)


def test_int4_quantiser_and_round_trip_and_product():
    rng = np.random.default_rng(42)
    N, K, M = 48, 96, 20
    W = rng.standard_normal((N, K)).astype(np.float32) * np.float32(0.02)
    W[5] = 0.0
    P, _ = oracle.prune_4to8_pairs(W)
    Q, s = oracle.quantize_rows_int4(P)
    amax = np.abs(P).max(axis=1)
    s_np = np.where(amax == 0, np.float32(1), amax / np.float32(7)).astype(np.float32)
    assert np.array_equal(s, s_np)
    q_np = np.clip(np.rint(P / s_np[:, None]), -7, 7).astype(np.int8)  # numpy's float32 division and half-even rint
    assert np.array_equal(Q, q_np)
    assert (np.abs(Q).max(axis=1)[amax > 0] == 7).all() and (Q[5] == 0).all()
    assert np.abs(Q.astype(np.float64) * s[:, None] - P).max() <= s.max() / 2 * (1 + 1e-6)
    # the quantised tensor keeps the pattern, so it compresses without violations and decodes to itself
    v, m, viol = oracle.compress_int4_pairs(Q)
    assert viol == 0 and v.shape == (N, K // 4) and m.shape == (N, K // 16)
    D = oracle.decompress_int4_pairs(v, m, K)
    assert np.array_equal(D, Q)
    # the product on the decoded operand is the plain integer matrix product
    X = rng.integers(-127, 128, (M, K)).astype(np.int8)
    assert np.array_equal(oracle.gemm_int8_dense(X, D), X.astype(np.int64) @ Q.astype(np.int64).T)
    # K that is a multiple of 8 but not of 16: the last index byte holds one chunk
    Q2 = Q[:, :88]
    v2, m2, viol2 = oracle.compress_int4_pairs(Q2)
    assert viol2 == 0 and m2.shape == (N, 6) and (m2[:, 5] >> 4 == 0).all()
    assert np.array_equal(oracle.decompress_int4_pairs(v2, m2, 88), Q2)


def test_int4_one_sub_chunk_per_group_is_both_patterns_and_decodes_to_the_2to4_form():
    """The constrained choice (one kept sub-chunk in each group of 4): brute force over its 4 allowed combinations, the
    result obeys the pair-wise 4:8 pattern and the 2:4 pattern, and its INT8 2:4 compressed form derived from the INT4
    storage decompresses (with the 2:4 decompressor) to the same matrix as the INT4 decoder gives."""
    rng = np.random.default_rng(43)
    N, K = 32, 96
    for W in (rng.standard_normal((N, K)).astype(np.float32), rng.integers(-3, 4, (N, K)).astype(np.float32)):
        P, mask = oracle.prune_4to8_pairs(W, one_per_group=True)
        for n in range(N):
            for c in range(K // 8):
                w = W[n, 8 * c:8 * c + 8]
                score = [float(np.float32(abs(w[2 * p])) + np.float32(abs(w[2 * p + 1]))) for p in range(4)]
                allowed = [(i, j) for i in (0, 1) for j in (2, 3)]
                best = max(score[i] + score[j] for i, j in allowed)
                i, j = min(pr for pr in allowed if score[pr[0]] + score[pr[1]] == best)
                assert mask[n, c] == (1 << i) | (1 << j)
        assert ((P.reshape(N, K // 4, 4) != 0).sum(axis=2) <= 2).all()             # 2:4
        nzp = (P.reshape(N, K // 2, 2) != 0).any(axis=2).reshape(N, K // 8, 4)
        assert (nzp.sum(axis=2) <= 2).all()                                         # pair-wise 4:8
        # never better than the free choice, which keeps the two best of all four sub-chunks
        F, _ = oracle.prune_4to8_pairs(W)
        assert np.abs(P).sum() <= np.abs(F).sum() + 1e-3
        Q, s = oracle.quantize_rows_int4(P)
        v4, m4, viol = oracle.compress_int4_pairs(Q)
        assert viol == 0 and oracle.compress(Q)[2] == 0
        v8, m8, bad = oracle.int4_pairs_to_sparse_int8(v4, m4, K)
        # (a chunk with codes that quantised to zero may carry other positions than the pruning chose: the matrix is the
        # same, and the matrix is what both decoders must agree on)
        D4 = oracle.decompress_int4_pairs(v4, m4, K)
        assert bad == 0 and np.array_equal(oracle.decompress(v8, m8, K), D4) and np.array_equal(D4, Q)
    # with codes that are all non-zero the positions are forced, so the shape test must pass everywhere
    W = (rng.integers(1, 4, (N, K)) * rng.choice([-1, 1], (N, K))).astype(np.float32)
    P, _ = oracle.prune_4to8_pairs(W, one_per_group=True)
    Q = P.astype(np.int8)
    v4, m4, viol = oracle.compress_int4_pairs(Q)
    v8, m8, bad = oracle.int4_pairs_to_sparse_int8(v4, m4, K)
    assert viol == 0 and bad == 0
    assert np.array_equal(oracle.decompress(v8, m8, K), Q)
    X = rng.integers(-127, 128, (9, K)).astype(np.int8)
    assert np.array_equal(oracle.spgemm_int8(X, v8, m8), X.astype(np.int64) @ Q.astype(np.int64).T)
    # a free-choice row with both kept sub-chunks in one group of 4 is reported; zeros inside a kept sub-chunk are fine
    row = np.array([[1, 2, 3, 4, 0, 0, 0, 0, 0, 5, 0, 0, 0, 0, 0, 0]], np.int8)
    v4, m4, _ = oracle.compress_int4_pairs(row)
    v8, m8, bad = oracle.int4_pairs_to_sparse_int8(v4, m4, 16)
    assert bad == 1 and np.array_equal(oracle.decompress(v8, m8, 16)[0, 8:], row[0, 8:])


def test_n_of_m_pruning_against_sorting_and_the_2to4_rule():
    """n:m patterns of the limitation paragraph (1:4, 2:16) and a few more: a stable argsort written here picks the same
    elements; 2:4 is the original rule; 1:4 and 2:16 tensors obey 2:4 (the compressor reports no violation)."""
    rng = np.random.default_rng(44)
    N, K = 16, 64
    for W in (rng.standard_normal((N, K)).astype(np.float32), rng.integers(-2, 3, (N, K)).astype(np.float32)):
        for n, m in ((1, 4), (2, 16), (2, 4), (4, 8), (1, 2), (3, 16)):
            P = oracle.prune_n_of_m(W, n, m)
            G = W.reshape(N, K // m, m)
            order = np.argsort(-np.abs(G), axis=2, kind="stable")   # descending magnitude, lower index first among equals
            keep = np.zeros(G.shape, bool)
            np.put_along_axis(keep, order[:, :, :n], True, axis=2)
            assert np.array_equal(P, np.where(keep, G, np.float32(0)).reshape(N, K))
            assert ((P.reshape(N, K // m, m) != 0).sum(axis=2) <= n).all()
        assert np.array_equal(oracle.prune_n_of_m(W, 2, 4), oracle.prune_2to4(W)[0])
        for n, m in ((1, 4), (2, 16)):
            P = oracle.prune_n_of_m(W, n, m)
            assert oracle.compress(P.astype(np.float16))[2] == 0
            assert np.array_equal(oracle.prune_2to4(P)[0], P)      # already 2:4: pruning again changes nothing
