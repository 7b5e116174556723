"""Pins for the CPU oracle: everything here checks oracle/ against something
that is not the oracle — hand-worked vectors, closed forms, brute force written
from the definitions in pure Python / float64, library routines, invariants.
No GPU needed."""
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
from scipy.stats import norm

from oracle import bitnet_a48 as O

HERE = os.path.dirname(os.path.abspath(__file__))
GOLD = json.load(open(os.path.join(HERE, "golden", "worked_vectors.json")))
EPS = 1e-5
F32 = np.float32


def f32(x):
    return np.float32(x)


# ------------------------------------------------------------------ eq. 4
def test_round_clip_half_even_and_clip():
    x = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 7.5, 8.4, -8.5, -9.0, 6.5], dtype=F32)
    got = O.round_clip(x, -8, 7)
    assert got.tolist() == [0, 2, 2, -0.0, -2, -2, 7, 7, -8, -8, 6]


# ------------------------------------------------------------------ eq. 7
@pytest.mark.parametrize("case", GOLD["int4"])
def test_int4_worked_vectors(case):
    x = np.array([case["x"]], dtype=F32)
    q, d = O.quant_int4(x, EPS)
    assert q[0].tolist() == case["q"]
    assert d[0] == f32(case["d"])


def test_int4_range_and_gaussian_closed_form():
    # Closed form for a Gaussian token: beta = sigma*sqrt(2/pi); code c covers
    # |x| in [(c-.5), (c+.5)) * beta/sqrt7.  Table 2 of the paper prints
    # 12.0-12.1 % zeros for the QKV / gate inputs.
    rng = np.random.default_rng(7)
    X = rng.standard_normal((256, 8192)).astype(F32) * f32(3.0)
    q, d = O.quant_int4(X, EPS)
    assert q.min() == -8 and q.max() == 7
    unit = math.sqrt(2 / math.pi) / math.sqrt(7)
    p0 = 2 * norm.cdf(0.5 * unit) - 1
    p7 = 1 - norm.cdf(6.5 * unit)
    pm8 = norm.cdf(-7.5 * unit)
    n = q.size
    for val, p in ((0, p0), (7, p7), (-8, pm8)):
        frac = np.mean(q == val)
        assert abs(frac - p) < 5 * math.sqrt(p * (1 - p) / n) + 2e-4, (val, frac, p)
    lo, hi = GOLD["table2"]["int4_zero_fraction_percent"]
    assert lo - 0.1 <= 100 * np.mean(q == 0) <= hi + 0.1
    # asymmetric clip: +7.6 units -> 7, -7.6 units -> -8
    assert abs(np.mean(q == -7) - (norm.cdf(-6.5 * unit) - norm.cdf(-7.5 * unit))) < 1e-3


def _int4_bruteforce(row):
    """eq. 7 in exact rationals except for the float32 roundings the reading fixes."""
    K = len(row)
    S = sum(abs(Fraction(float(v))) for v in row)
    beta = f32(float(S / K))
    s = f32(O.SQRT7 / f32(beta + f32(EPS)))
    out = []
    for v in row:
        p = f32(f32(v) * s)
        r = round(Fraction(float(p)))          # Python round(): half to even on exact rationals
        out.append(int(min(max(r, -8), 7)))
    return out, f32(beta / O.SQRT7)


def test_int4_bruteforce_rows():
    rng = np.random.default_rng(11)
    X = rng.standard_normal((12, 37)).astype(F32)
    X[3] *= 50
    X[5] = 0
    X[6, :] = 0.25
    q, d = O.quant_int4(X, EPS)
    for m in range(X.shape[0]):
        qb, db = _int4_bruteforce(X[m])
        assert q[m].tolist() == qb
        assert d[m] == db


# ------------------------------------------------------------------ Section 4.3: the other INT4 quantizers
def _int4_variant_bruteforce(row, kind):
    """The variant in exact rationals except for the float32 roundings the reading fixes."""
    K = len(row)
    if kind == "absmean2":
        S = sum(abs(Fraction(float(v))) for v in row)
        stat = f32(f32(2) * f32(float(S / K)))
        num, den = O.SQRT7, O.SQRT7
    else:
        stat = f32(max(abs(float(v)) for v in row))
        num, den = f32(7), f32(7)
    s = f32(num / f32(stat + f32(EPS)))
    out = []
    for v in row:
        p = f32(f32(v) * s)
        out.append(int(min(max(round(Fraction(float(p))), -8), 7)))
    return out, f32(stat / den)


@pytest.mark.parametrize("kind", ["absmean2", "absmax"])
def test_int4_variants(kind):
    # hand-worked: |x| = 1, 1, 2, 2, 4, 4, 8, 8 -> mean 3.75, max 8
    x = np.array([[1, -1, 2, -2, 4, -4, 8, -8]], dtype=F32)
    q, d = O.quant_int4_variant(x, EPS, kind)
    if kind == "absmean2":      # beta = 7.5, x * sqrt7 / 7.5 = .353, .706, 1.411, 2.822
        assert q[0].tolist() == [0, 0, 1, -1, 1, -1, 3, -3]
        assert d[0] == f32(f32(7.5) / O.SQRT7)
    else:                       # x * 7 / 8.00001 = .875, 1.75, 3.4999956, 6.999991
        assert q[0].tolist() == [1, -1, 2, -2, 3, -3, 7, -7]
        assert d[0] == f32(f32(8) / f32(7))
    rng = np.random.default_rng(21)
    X = rng.standard_normal((10, 41)).astype(F32)
    X[2] *= 30
    X[4] = 0
    X[5, :] = -0.5
    q, d = O.quant_int4_variant(X, EPS, kind)
    for m in range(X.shape[0]):
        qb, db = _int4_variant_bruteforce(X[m], kind)
        assert q[m].tolist() == qb and d[m] == db
    assert q.min() >= -8 and q.max() <= 7
    # power-of-two rescaling of a token changes nothing but the scale (eps = 0)
    q1, d1 = O.quant_int4_variant(X[:4], 0.0, kind)
    q2, d2 = O.quant_int4_variant(X[:4] * f32(8), 0.0, kind)
    assert np.array_equal(q1, q2) and np.array_equal(d2, d1 * f32(8))
    if kind == "absmax":        # the largest magnitude of a token gets code +-7, nothing clips
        big = np.abs(X).argmax(axis=1)
        rows = [m for m in range(X.shape[0]) if m != 4]
        assert all(abs(int(q[m, big[m]])) == 7 for m in rows)
        assert np.abs(q).max() == 7
    else:                       # twice the beta of eq. 7: exactly twice its step
        qa, da = O.quant_int4(X, EPS)
        assert np.array_equal(d, da * f32(2))
    # textbook uniform quantizer with step d: unclipped values land within half a step
    deq = q.astype(np.float64) * d[:, None].astype(np.float64)
    unclipped = (q > -8) & (q < 7)
    half = 0.5 * np.repeat(d[:, None].astype(np.float64), X.shape[1], 1) * (1 + 1e-4) + 1e-5
    assert np.all(np.abs(deq - X)[unclipped] <= half[unclipped])


def test_int4_is_per_token_and_uniform_step():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((6, 64)).astype(F32)
    q, d = O.quant_int4(X, EPS)
    X2 = X.copy()
    X2[0] *= 100                      # changing one token must not change the others
    q2, d2 = O.quant_int4(X2, EPS)
    assert np.array_equal(q[1:], q2[1:]) and np.array_equal(d[1:], d2[1:])
    # textbook uniform quantizer with step d: unclipped values land within half a step
    deq = q.astype(np.float64) * d[:, None].astype(np.float64)
    unclipped = (q > -8) & (q < 7)
    assert np.all(np.abs(deq - X)[unclipped] <= 0.5 * d[:, None].repeat(64, 1)[unclipped] * (1 + 1e-4))
    # all-zero token: beta = 0 -> codes 0, scale 0
    qz, dz = O.quant_int4(np.zeros((1, 16), F32), EPS)
    assert not qz.any() and dz[0] == 0


# ------------------------------------------------------------------ eq. 2
@pytest.mark.parametrize("case", GOLD["ternary"])
def test_ternary_worked_vector(case):
    T, alpha = O.ternarize(np.array(case["W"], dtype=F32), EPS)
    assert T.tolist() == case["T"]
    assert alpha == f32(case["alpha"])


def test_ternary_closed_form_and_bruteforce():
    rng = np.random.default_rng(3)
    W = (0.02 * rng.standard_normal((512, 1024))).astype(F32)
    T, alpha = O.ternarize(W, EPS)
    assert set(np.unique(T).tolist()) == {-1, 0, 1}
    assert abs(float(alpha) - 0.02 * math.sqrt(2 / math.pi)) < 2e-5
    # zero iff |w| < (alpha+eps)/2 ; Gaussian: P = 2*Phi(0.5*sqrt(2/pi)) - 1 = 31.0 %
    p0 = 2 * norm.cdf(0.5 * math.sqrt(2 / math.pi)) - 1
    assert abs(np.mean(T == 0) - p0) < 3e-3
    assert abs(np.mean(T == 1) - np.mean(T == -1)) < 5e-3
    # brute force on a small block, exact rationals + the fixed float32 roundings
    Ws = W[:5, :9]
    Ts, a = O.ternarize(Ws, EPS)
    S = sum(abs(Fraction(float(v))) for v in Ws.ravel())
    a_ref = f32(float(S / Ws.size))
    assert a == a_ref                                  # the scale is alpha, not alpha + eps
    t = f32(a_ref + f32(EPS))
    for i in range(5):
        for j in range(9):
            r = round(Fraction(float(f32(Ws[i, j] / t))))
            assert Ts[i, j] == min(max(r, -1), 1)
    # sign symmetry
    Tn, an = O.ternarize(-W, EPS)
    assert an == alpha and np.array_equal(Tn, -T)


# ------------------------------------------------------------------ eq. 1 (Top_k)
def _topk_bruteforce(row, k):
    """Rank definition: element i is kept iff fewer than k elements beat it, where j
    beats i if |x_j| > |x_i|, or |x_j| == |x_i| and j < i."""
    a = [abs(float(v)) for v in row]
    keep = []
    for i in range(len(a)):
        rank = sum(1 for j in range(len(a)) if a[j] > a[i] or (a[j] == a[i] and j < i))
        keep.append(rank < k)
    return keep


def test_topk_bruteforce_ties_zeros():
    rng = np.random.default_rng(9)
    X = np.round(rng.standard_normal((10, 48)) * 2).astype(F32) / 2      # many ties
    X[2, ::3] = -0.0
    X[4] = 1.0                                                            # all equal
    X[5] = 0.0
    X[6] = np.eye(1, 48, 17, dtype=F32)[0] * -3                           # one-hot
    for k in (1, 7, 24, 47, 48):
        m = O.topk_mask(X, k)
        assert np.all(m.sum(1) == k)
        for r in range(X.shape[0]):
            assert m[r].tolist() == _topk_bruteforce(X[r], k), (r, k)
    # all-equal row keeps the first k channels; k = K keeps everything
    assert O.topk_mask(X, 5)[4].tolist() == [True] * 5 + [False] * 43
    assert O.topk_mask(X, 48).all()


def test_topk_half_matches_table2_out_sparsity():
    X = np.random.default_rng(1).standard_normal((32, 512)).astype(F32)
    m = O.topk_mask(X, 256)
    assert 100.0 * (1 - m.mean()) == GOLD["table2"]["out_sparsity_percent"]
    kept_min = np.where(m, np.abs(X), np.inf).min(1)
    drop_max = np.where(~m, np.abs(X), -np.inf).max(1)
    assert np.all(kept_min >= drop_max)


# ------------------------------------------------------------------ eq. 3
@pytest.mark.parametrize("case", GOLD["topk_int8"])
def test_topk_int8_worked_vectors(case):
    x = np.array([case["x"]], dtype=F32)
    q, d, m = O.quant_topk_int8(x, case["k"], EPS)
    assert m[0].astype(int).tolist() == case["mask"]
    assert q[0].tolist() == case["q"]
    assert d[0] == f32(case["d"])


def test_int8_properties():
    rng = np.random.default_rng(2)
    X = (rng.standard_normal((40, 96)) * rng.uniform(0.01, 30, (40, 1))).astype(F32)
    q, d = O.quant_int8(X, EPS)
    assert q.min() >= -127 and q.max() <= 127              # symmetric scale never reaches -128
    am = np.abs(X).argmax(1)
    assert np.all(np.abs(q[np.arange(40), am]) == 127)
    qn, dn = O.quant_int8(-X, EPS)
    assert np.array_equal(qn, -q) and np.array_equal(dn, d)
    # textbook per-token absmax INT8 (float64): codes agree except at half-way cases
    s64 = 127.0 / (np.abs(X).max(1, keepdims=True).astype(np.float64) + EPS)
    p64 = X.astype(np.float64) * s64
    far = np.abs(p64 - np.floor(p64) - 0.5) > 1e-3
    assert np.array_equal(np.rint(p64)[far], q.astype(np.float64)[far])
    # top-k with k = K is the plain dense INT8 quantizer
    qk, dk, mk = O.quant_topk_int8(X, 96, EPS)
    assert mk.all() and np.array_equal(qk, q) and np.array_equal(dk, d)
    # masked codes are zero, kept codes are unchanged
    qs, ds, ms = O.quant_topk_int8(X, 48, EPS)
    assert np.array_equal(qs[ms], q[ms]) and not qs[~ms].any() and np.array_equal(ds, d)
    assert np.all(ms.sum(1) == 48)


# ------------------------------------------------------------------ matmul + rescale
def test_matmul_int_bruteforce_and_special_cases():
    rng = np.random.default_rng(4)
    q = rng.integers(-8, 8, (5, 13)).astype(np.int8)
    T = rng.integers(-1, 2, (7, 13)).astype(np.int8)
    acc = O.matmul_int(q, T)
    assert acc.shape == (5, 7) and acc.dtype == np.int32
    for m in range(5):
        for n in range(7):
            assert acc[m, n] == sum(int(q[m, k]) * int(T[n, k]) for k in range(13))
    # W == +1 everywhere: every output is the token's code sum
    ones = np.ones((3, 13), np.int8)
    assert np.array_equal(O.matmul_int(q, ones), np.repeat(q.sum(1, dtype=np.int32)[:, None], 3, 1))
    # one-hot token picks a column of T
    oh = np.zeros((1, 13), np.int8)
    oh[0, 4] = -5
    assert np.array_equal(O.matmul_int(oh, T)[0], -5 * T[:, 4].astype(np.int32))
    # worst-case magnitudes at the largest K stay exact
    qq = np.full((2, 11008), -128, np.int8)
    TT = np.full((3, 11008), -1, np.int8)
    assert np.all(O.matmul_int(qq, TT) == 128 * 11008)


def test_bf16_round_matches_torch():
    rng = np.random.default_rng(6)
    x = np.concatenate([
        rng.standard_normal(5000).astype(F32) * 100,
        np.array([1 + 2 ** -8, 1 + 3 * 2 ** -8, -(1 + 2 ** -8), 0.0, 3.0e38, 1e-40], dtype=F32),
    ])
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(O.bf16_round(x), ref)


def _dense_f64(X_deq, W_deq):
    return X_deq.astype(np.float64) @ W_deq.astype(np.float64).T


def test_bitlinear_a4_against_dense_f64_of_dequantized_operands():
    rng = np.random.default_rng(8)
    X = rng.standard_normal((9, 40)).astype(F32)
    W = (0.02 * rng.standard_normal((11, 40))).astype(F32)
    r = O.bitlinear_a4(X, W, EPS)
    assert r["y"].shape == (9, 11)
    Xd = r["q"].astype(np.float64) * r["d"].astype(np.float64)[:, None]
    Wd = r["T"].astype(np.float64) * np.float64(r["alpha"])
    ref = _dense_f64(Xd, Wd)
    assert np.allclose(r["y"], ref, rtol=1e-6, atol=1e-9)
    # and it approximates the product of the raw activations with the ternary weights
    full = _dense_f64(X, Wd)
    cos = (ref * full).sum() / np.linalg.norm(ref) / np.linalg.norm(full)
    assert cos > 0.97
    yb = O.bitlinear_a4(X, W, EPS, "bf16")["y"]
    assert np.array_equal(yb, torch.from_numpy(r["y"]).to(torch.bfloat16).float().numpy())


def test_bitlinear_a8_sparse_against_dense_f64():
    rng = np.random.default_rng(10)
    X = rng.standard_normal((6, 64)).astype(F32)
    W = (0.02 * rng.standard_normal((10, 64))).astype(F32)
    r = O.bitlinear_a8_sparse(X, W, 32, EPS)
    Xd = np.where(r["mask"], X, 0)                    # sparsify-then-quantize view of eq. 1
    q_dense, d = O.quant_int8(X, EPS)
    assert np.array_equal(r["q"], np.where(r["mask"], q_dense, 0))
    ref = _dense_f64(r["q"].astype(np.float64) * r["d"].astype(np.float64)[:, None],
                     r["T"].astype(np.float64) * np.float64(r["alpha"]))
    assert np.allclose(r["y"], ref, rtol=1e-6, atol=1e-9)
    # INT8 is fine grained: close to the float product of the sparsified input with ternary weights
    ref2 = _dense_f64(Xd, r["T"].astype(np.float64) * np.float64(r["alpha"]))
    assert np.abs(ref - ref2).max() < 0.02 * np.abs(ref2).max() + 1e-3


def test_relu2_glu():
    rng = np.random.default_rng(12)
    g = rng.standard_normal((5, 33)).astype(F32) * 3
    u = rng.standard_normal((5, 33)).astype(F32) * 3
    h = O.relu2_glu(g, u)
    ref = u.astype(np.float64) * np.maximum(g.astype(np.float64), 0) ** 2
    assert np.all(np.abs(h - ref) <= np.abs(ref) * 2.0 ** -8 + 1e-30)       # one bf16 ulp
    assert np.all(h[g <= 0] == 0)
    assert np.all((h >= 0) == ((u >= 0) | (g <= 0)) | (h == 0))
    assert np.array_equal(h, O.bf16_round(h))


def test_ffn_block_shapes_and_chain():
    rng = np.random.default_rng(13)
    X = rng.standard_normal((4, 32)).astype(F32)
    Wg = (0.02 * rng.standard_normal((48, 32))).astype(F32)
    Wu = (0.02 * rng.standard_normal((48, 32))).astype(F32)
    Wd = (0.02 * rng.standard_normal((32, 48))).astype(F32)
    r = O.ffn_block(X, Wg, Wu, Wd, 24, EPS)
    assert r["h"].shape == (4, 48) and r["down"]["y"].shape == (4, 32)
    assert np.array_equal(r["h"], O.relu2_glu(r["gate"]["y"], r["up"]["y"]))
    assert np.all(r["down"]["mask"].sum(1) == 24)


# ------------------------------------------------------------------ eq. 8-9 (FP4)
GRID15 = sorted(set([s * v for s in (-1, 1) for v in (0, .5, 1, 1.5, 2, 3, 4, 6)]))


def _nearest_e2m1(v):
    """Nearest E2M1 magnitude, ties to the even code, by distance to all 8 grid points."""
    grid = [0, .5, 1, 1.5, 2, 3, 4, 6]
    a = abs(v)
    best = min(range(8), key=lambda c: (abs(Fraction(a) - Fraction(grid[c])), c % 2))
    return best


def test_fp4_exhaustive_binades_against_nearest_grid_point():
    # every bf16 magnitude in [2^-4, 8): put 6.0 in the block so the scale is 2^0
    mags = []
    for e in range(-4, 3):
        for m in range(128):
            mags.append((1 + m / 128.0) * 2.0 ** e)
    mags = [v for v in mags if v <= 6.0]
    vals = np.array(mags + [-v for v in mags], dtype=F32)
    pad = (-len(vals)) % 31
    vals = np.concatenate([vals, np.zeros(pad, F32)])
    blocks = vals.reshape(-1, 31)
    X = np.concatenate([np.full((blocks.shape[0], 1), 6.0, F32), blocks], axis=1)  # [B, 32]
    codes, e = O.quant_fp4(X)
    assert np.all(e == 0)
    for b in range(X.shape[0]):
        for j in range(32):
            c = int(codes[b, j])
            want = _nearest_e2m1(float(X[b, j]))
            assert (c & 7) == want, (X[b, j], c, want)
            assert bool(c & 8) == (X[b, j] < 0 and want != 0)


def test_fp4_scale_choice_and_invariants():
    rng = np.random.default_rng(14)
    X = (rng.standard_normal((16, 128)) * np.exp(rng.uniform(-12, 12, (16, 1)))).astype(F32)
    X[3, 32:64] = 0
    codes, e = O.quant_fp4(X)
    assert codes.max() <= 15
    deq = O.fp4_dequant(codes, e)
    a = np.abs(X.astype(np.float64)).reshape(16, 4, 32).max(2)
    scaled = a / np.exp2(e.astype(np.float64))
    nz = a > 0
    assert np.all((scaled[nz] > 3.0) & (scaled[nz] <= 6.0))       # never clips, never wastes a binade
    assert np.all(e[~nz] == 0) and not codes[3, 32:64].any()
    # half-a-step accuracy (step = 2 * 2^e at most) and idempotence
    err = np.abs(deq - X).reshape(16, 4, 32)
    assert np.all(err <= np.exp2(e.astype(np.float64))[:, :, None] * 1.0 + 1e-300)
    c2, e2 = O.quant_fp4(deq.astype(F32))                # values already on the grid are kept
    assert np.array_equal(O.fp4_dequant(c2, e2), deq)
    # the paper's formula with an integer bias b = floor(log2(12 / max)), E = 2, M = 1
    Mb = 1
    for (r, blk) in ((0, 0), (5, 2), (9, 3)):
        x = X[r, blk * 32:(blk + 1) * 32].astype(np.float64)
        b = math.floor(math.log2((2 - 2.0 ** -Mb) / np.abs(x).max()) + 2 ** 2 - 1)
        assert e[r, blk] == 1 - b
        with np.errstate(divide="ignore"):
            p = np.maximum(np.floor(np.log2(np.abs(x))) + b, 1)
        step = np.exp2(p - Mb - b)
        ref = step * np.rint(x / step)
        assert np.array_equal(ref, deq[r, blk * 32:(blk + 1) * 32])


def test_fp4_e1m2_format():
    """Section 4.3's other 4-bit float format (E = 1, M = 2) through the same eq. 8-9."""
    # hand-worked block, maximum 1.75 -> scale 2^0, step 1/4: ties go to the even code
    x = np.zeros((1, 32), F32)
    x[0, :8] = [1.75, -0.3, 0.12, 0.13, 0.125, 0.375, -0.875, 1.7]
    codes, e = O.quant_fp4(x, "e1m2")
    assert e[0, 0] == 0
    assert list(codes[0, :8]) == [7, 8 | 1, 0, 1, 0, 2, 8 | 4, 7]     # -0.875 * 4 = -3.5 -> 4 (even)
    assert not codes[0, 8:].any()
    # every bf16 magnitude in [2^-6, 1.75] with 1.75 in the block: nearest grid point by exact fractions
    mags = [(1 + m / 128.0) * 2.0 ** ex for ex in range(-6, 1) for m in range(128)]
    mags = [v for v in mags if v <= 1.75]
    vals = np.array(mags + [-v for v in mags], dtype=F32)
    vals = np.concatenate([vals, np.zeros((-len(vals)) % 31, F32)]).reshape(-1, 31)
    X = np.concatenate([np.full((vals.shape[0], 1), 1.75, F32), vals], axis=1)
    codes, e = O.quant_fp4(X, "e1m2")
    assert np.all(e == 0)
    for b in range(X.shape[0]):
        for j in range(32):
            a = Fraction(abs(float(X[b, j])))
            want = min(range(8), key=lambda c: (abs(a - Fraction(c, 4)), c % 2))
            assert (int(codes[b, j]) & 7) == want, (X[b, j], codes[b, j], want)
            assert bool(codes[b, j] & 8) == (X[b, j] < 0 and want != 0)
    # scale choice, accuracy, idempotence, and the printed formula with an integer bias (E = 1, M = 2)
    rng = np.random.default_rng(21)
    X = (rng.standard_normal((16, 128)) * np.exp(rng.uniform(-12, 12, (16, 1)))).astype(F32)
    X[2, 64:96] = 0
    codes, e = O.quant_fp4(X, "e1m2")
    deq = O.fp4_dequant(codes, e, "e1m2")
    a = np.abs(X.astype(np.float64)).reshape(16, 4, 32).max(2)
    scaled = a / np.exp2(e.astype(np.float64))
    nz = a > 0
    assert np.all((scaled[nz] > 0.875) & (scaled[nz] <= 1.75))      # never clips, never wastes a binade
    assert np.all(e[~nz] == 0) and not codes[2, 64:96].any()
    err = np.abs(deq - X).reshape(16, 4, 32)
    assert np.all(err <= np.exp2(e.astype(np.float64))[:, :, None] * 0.125)   # half a step of 1/4
    c2, e2 = O.quant_fp4(deq.astype(F32), "e1m2")
    assert np.array_equal(O.fp4_dequant(c2, e2, "e1m2"), deq)
    Eb, Mb = 1, 2
    for (r, blk) in ((0, 0), (5, 2), (9, 3)):
        x = X[r, blk * 32:(blk + 1) * 32].astype(np.float64)
        b = math.floor(math.log2((2 - 2.0 ** -Mb) / np.abs(x).max()) + 2 ** Eb - 1)
        assert e[r, blk] == 1 - b
        with np.errstate(divide="ignore"):
            p = np.maximum(np.floor(np.log2(np.abs(x))) + b, 1)
        step = np.exp2(p - Mb - b)
        assert np.array_equal(step * np.rint(x / step), deq[r, blk * 32:(blk + 1) * 32])
    # the two formats differ where they should: E2M1 reaches 6 with coarse steps, E1M2 is uniform
    d21 = O.fp4_dequant(*O.quant_fp4(X), "e2m1")
    assert not np.array_equal(d21, deq)


def test_swish_glu():
    """h = u g sigmoid(g): closed forms and identities of the textbook function."""
    g = np.array([0.0, 1.0, -1.0, 30.0, -30.0, 200.0, -200.0], F32)
    h = O.swish_glu(g, np.ones_like(g)).astype(np.float64)
    want = [0.0, 1 / (1 + math.exp(-1.0)), -1 / (1 + math.exp(1.0)), 30.0, -30.0 * math.exp(-30.0), 200.0, 0.0]
    for got, w in zip(h, want):
        assert abs(got - w) <= 2.0 ** -8 * abs(w)                  # one bf16 rounding
    assert h[6] == 0.0 and not np.isnan(h).any()                   # exp overflow handled
    # swish(x) - swish(-x) = x, checked before the final rounding by taking u as a power of two
    rng = np.random.default_rng(22)
    x = rng.uniform(-8, 8, 4096).astype(F32)
    hp = O.swish_glu(x, np.ones_like(x)).astype(np.float64)
    hm = O.swish_glu(-x, np.ones_like(x)).astype(np.float64)
    assert np.all(np.abs((hp - hm) - x) <= 2.0 ** -7 * np.maximum(np.abs(hp), np.abs(hm)) + 1e-30)
    # minimum of the function: -0.27846 at x = -1.27846 (root of 1 + e^-x (1 + ... ) = 0)
    xs = np.linspace(-3, 0, 30001).astype(F32)
    hs = O.swish_glu(xs, np.ones_like(xs))
    # (bfloat16 resolution flattens the bottom: the location is only good to a few hundredths)
    assert abs(float(xs[hs.argmin()]) + 1.27846) < 0.1 and abs(float(hs.min()) + 0.27846) < 2e-3
    # linear in u, results are bfloat16 values, ties to even from float64
    u = rng.standard_normal(4096).astype(F32)
    h2 = O.swish_glu(x, u)
    assert np.array_equal(O.bf16_round(h2), h2)
    ref = u.astype(np.float64) * (x.astype(np.float64) / (1 + np.exp(-x.astype(np.float64))))
    assert np.all(np.abs(h2 - ref) <= 2.0 ** -8 * np.abs(ref) * (1 + 1e-9) + 1e-40)
    # a value exactly between two bfloat16 neighbours goes to the even one: 1 + 2^-8 with sigmoid = 1
    big = np.array([64.0], F32)                                    # sigmoid(64) == 1.0 in float64
    hb = O.swish_glu(big, np.array([(1 + 2.0 ** -8) / 64.0], F32))
    assert hb[0] == 1.0


def test_bitlinear_fp4_against_dense():
    rng = np.random.default_rng(15)
    X = rng.standard_normal((5, 64)).astype(F32)
    W = (0.02 * rng.standard_normal((7, 64))).astype(F32)
    r = O.bitlinear_fp4(X, W, EPS)
    # brute-force triple loop in Python floats
    deq = O.fp4_dequant(r["codes"], r["e"])
    for m in range(5):
        for n in range(7):
            s = math.fsum(float(deq[m, k]) * int(r["T"][n, k]) for k in range(64))
            assert abs(r["y"][m, n] - float(r["alpha"]) * s) <= 1e-12 * (1 + abs(s))
    for v in np.unique(deq / np.exp2(r["e"].astype(np.float64)).repeat(32, 1)):
        assert v in GRID15


# ------------------------------------------------------------------ Section 4.2: low-bit attention states
@pytest.mark.parametrize("bits", [4, 3])
def test_quant_heads(bits):
    Qb = 2 ** (bits - 1) - 1
    off = 2 ** (bits - 1)
    # hand-worked head, gamma = 7 (eps = 0): 4 bits -> q = x exactly; 3 bits -> q = rint(3 x / 7)
    x = np.array([[[7.0, -7.0, 3.5, -3.5, 1.0, 0.0, -0.4, 5.9]]], F32)
    codes, d = O.quant_heads(x, bits, 0.0)
    if bits == 4:
        assert codes[0, 0].tolist() == [15, 1, 12, 4, 9, 8, 8, 14]      # 3.5 -> 4 (even), -3.5 -> -4, 5.9 -> 6
        assert d[0, 0] == f32(1.0)
    else:
        assert codes[0, 0].tolist() == [7, 1, 6, 2, 4, 4, 4, 7]         # 1.5 -> 2 (even), 3/7 -> 0, 2.53 -> 3
        assert d[0, 0] == f32(f32(7) / f32(3))
    # brute force in exact rationals except for the float32 roundings the reading fixes
    rng = np.random.default_rng(41)
    X = rng.standard_normal((5, 3, 24)).astype(F32)
    X[1, 0] *= 40
    X[2, 1] = 0
    X[3, 2, :] = -0.75
    codes, d = O.quant_heads(X, bits, EPS)
    for t in range(5):
        for h in range(3):
            row = X[t, h]
            gamma = f32(max(abs(float(v)) for v in row))
            s = f32(f32(Qb) / f32(gamma + f32(EPS)))
            want = [int(min(max(round(Fraction(float(f32(f32(v) * s)))), -Qb), Qb)) + off for v in row]
            assert codes[t, h].tolist() == want and d[t, h] == f32(gamma / f32(Qb))
    # unsigned codes in [1, 2^bits - 1]; the largest magnitude of a head sits at an end of the range;
    # an all-zero head is all `off` with scale 0; heads do not influence one another
    assert codes.min() >= 1 and codes.max() <= 2 * off - 1
    big = np.abs(X).reshape(15, 24).argmax(1)
    cc = codes.reshape(15, 24)
    for i in range(15):
        if i != 2 * 3 + 1:
            assert cc[i, big[i]] in (1, 2 * off - 1)
    assert np.all(codes[2, 1] == off) and d[2, 1] == 0
    X2 = X.copy()
    X2[0, 0] *= 9
    c2, d2 = O.quant_heads(X2, bits, EPS)
    keep = np.ones((5, 3), bool)
    keep[0, 0] = False
    assert np.array_equal(c2[keep], codes[keep]) and np.array_equal(d2[keep], d[keep])
    # uniform quantizer with step d: within half a step; x -> -x mirrors the codes; 2^k gains pass (eps = 0)
    deq = (codes.astype(np.float64) - off) * d[:, :, None].astype(np.float64)
    assert np.all(np.abs(deq - X) <= 0.5 * d[:, :, None] * (1 + 1e-4) + 1e-5)
    cn, dn = O.quant_heads(-X, bits, EPS)
    assert np.array_equal(cn.astype(int), 2 * off - codes.astype(int)) and np.array_equal(dn, d)
    Xnz = X[[0, 1, 3, 4]]                                  # (eps = 0 needs gamma > 0)
    c0, d0 = O.quant_heads(Xnz, bits, 0.0)
    c8, d8 = O.quant_heads(Xnz * f32(8), bits, 0.0)
    assert np.array_equal(c0, c8) and np.array_equal(d8, d0 * f32(8))
    # 4 bits: the same integers as the INT4 absmax quantizer of the ablations (7 levels) on the same row
    if bits == 4:
        q7, d7 = O.quant_int4_variant(X.reshape(15, 24), EPS, "absmax")
        assert np.array_equal(codes.reshape(15, 24).astype(int) - 8, q7.astype(int))
        assert np.array_equal(d.reshape(15), d7)


def test_kv_cache_mixed_width():
    """Table 3's 3-bit key / value cache with the first token's heads at 4 bits: the hand-worked
    two-token example (literal bytes), a bit-by-bit decode of the layout in plain Python, exact-rational
    dequantization, and the properties of a uniform quantizer."""
    g = GOLD["kv_cache"]
    x = np.array(g["x"], F32)
    raw, d = O.kv_cache_pack(x, 0.0)
    assert raw.tolist() == g["bytes"] and d.reshape(-1).tolist() == g["scales"]
    assert O.quant_heads(x[:1], 4, 0.0)[0][0, 0].tolist() == g["codes_token0"]
    assert O.quant_heads(x[1:], 3, 0.0)[0][0, 0].tolist() == g["codes_token1"]
    assert np.array_equal(O.kv_cache_unpack(raw, d, 2, 1, 8), np.array(g["values"], F32))
    # seeded tokens: sizes, every code recovered bit by bit from the documented layout, values as
    # exact rationals (code - offset) * d rounded once to float32
    rng = np.random.default_rng(61)
    T, H, D = 5, 3, 24
    X = rng.standard_normal((T, H, D)).astype(F32)
    X[2, 1] *= 30
    X[3, 0] = 0
    raw, d = O.kv_cache_pack(X, EPS)
    assert raw.size == H * D // 2 + (T - 1) * H * 3 * D // 8 and d.shape == (T, H)
    bits_all = "".join(format(int(b), "08b")[::-1] for b in raw)          # bit i of the stream at index i
    pos = 0
    vals = O.kv_cache_unpack(raw, d, T, H, D)
    for t in range(T):
        bits = 4 if t == 0 else 3
        codes, dt = O.quant_heads(X[t:t + 1], bits, EPS)
        assert np.array_equal(dt[0], d[t])
        for h in range(H):
            for j in range(D):
                code = int(bits_all[pos:pos + bits][::-1], 2)
                pos += bits
                assert code == int(codes[0, h, j])
                want = f32(float(Fraction(code - 2 ** (bits - 1)) * Fraction(float(d[t, h]))))
                assert vals[t, h, j] == want
    assert pos == 8 * raw.size
    # within half a step of the input (plus the eps shrink), zero head -> zeros, sign symmetry
    assert np.all(np.abs(vals - X) <= 0.5 * d[:, :, None] * (1 + 1e-4) + 1e-5)
    assert not vals[3, 0].any()
    rawn, dn = O.kv_cache_pack(-X, EPS)
    assert np.array_equal(O.kv_cache_unpack(rawn, dn, T, H, D), -vals)
    # dequant_heads alone: the uniform-width form
    for bits in (4, 3):
        c, dd = O.quant_heads(X, bits, EPS)
        v = O.dequant_heads(c, dd, bits)
        off = 2 ** (bits - 1)
        assert np.array_equal(v, ((c.astype(np.float64) - off) * dd[:, :, None].astype(np.float64)).astype(F32))


def test_up_projection_sparsity_composition():
    """The gate-first up projection needs a multiply only where the input code and the gate are both
    non-zero; the paper's 7B figures (12.0 % zero codes, 67.5 % closed gates) compose to its 71.4 %.
    Here on the oracle's own codes and gates: Gaussian tokens (11.99 % zero codes in closed form) and
    gates closed with probability 0.675, independent of the input."""
    c = GOLD["table2"]["up_composition"]
    assert abs(100 * (1 - (1 - c["gate_input_zero_percent"] / 100) * (1 - c["gate_output_zero_percent"] / 100))
               - c["up_percent"]) < 0.05
    rng = np.random.default_rng(51)
    X = rng.standard_normal((64, 2048)).astype(F32)
    q, _ = O.quant_int4(X, EPS)
    g = rng.standard_normal((64, 512)).astype(F32) - f32(norm.ppf(0.675))      # P(g <= 0) = 0.675
    u = rng.standard_normal((64, 512)).astype(F32)
    h = O.relu2_glu(g, u)
    open_gate = g > 0
    assert abs(np.mean(~open_gate) - 0.675) < 0.01
    assert not h[~open_gate].any()                         # a closed gate needs no up projection at all
    needed = (q != 0)[:, :, None] & open_gate[:, None, :]  # [token, input channel, output channel]
    assert abs(100 * (1 - needed.mean()) - c["up_percent"]) < 0.8


# ------------------------------------------------------------------ symmetries of the whole layers
def test_layer_symmetries():
    """What the equations imply whatever the arithmetic details: tokens are independent, sign flips and
    power-of-two gains pass through exactly (with eps = 0), output channels permute with the rows of W."""
    rng = np.random.default_rng(31)
    X = O.bf16_round(rng.standard_normal((6, 96)).astype(F32))
    X[:, 5] *= 17.0
    W = (0.02 * rng.standard_normal((10, 96))).astype(F32)
    base4 = O.bitlinear_a4(X, W, 0.0)
    base8 = O.bitlinear_a8_sparse(X, W, 48, 0.0)
    # tokens are independent: any permutation or subset of rows gives the same rows
    perm = rng.permutation(6)
    assert np.array_equal(O.bitlinear_a4(X[perm], W, 0.0)["y"], base4["y"][perm])
    assert np.array_equal(O.bitlinear_a8_sparse(X[perm[:3]], W, 48, 0.0)["y"], base8["y"][perm[:3]])
    # x -> -x: codes and outputs change sign, scales and the Top_k mask stay (|x| decides both)
    n4 = O.bitlinear_a4(-X, W, 0.0)
    n8 = O.bitlinear_a8_sparse(-X, W, 48, 0.0)
    assert np.array_equal(n4["d"], base4["d"]) and np.array_equal(n8["mask"], base8["mask"])
    # (the INT4 grid -8..7 is not symmetric: where a value clips, one side reads -8 and the other +7;
    # nothing else differs)
    diff = n4["q"] != -base4["q"]
    assert np.all(np.minimum(base4["q"], n4["q"])[diff] == -8) and np.all(np.maximum(base4["q"], n4["q"])[diff] == 7)
    assert diff.sum() > 0                                  # the outlier channel does clip
    assert np.array_equal(n8["q"], -base8["q"]) and np.array_equal(n8["y"], -base8["y"])
    # x -> 2^k x with eps = 0: same codes, scale and output times 2^k exactly
    for k in (-3, 5):
        g = np.ldexp(X, k).astype(F32)
        s4 = O.bitlinear_a4(g, W, 0.0)
        s8 = O.bitlinear_a8_sparse(g, W, 48, 0.0)
        assert np.array_equal(s4["q"], base4["q"]) and np.array_equal(s8["q"], base8["q"])
        assert np.array_equal(s4["d"], np.ldexp(base4["d"], k))
        assert np.array_equal(s4["y"], np.ldexp(base4["y"], k)) and np.array_equal(s8["y"], np.ldexp(base8["y"], k))
    # W -> -W: ternary codes and outputs change sign, alpha stays; rows of W permute the output channels
    m4 = O.bitlinear_a4(X, -W, 0.0)
    assert np.array_equal(m4["T"], -base4["T"]) and m4["alpha"] == base4["alpha"]
    assert np.array_equal(m4["y"], -base4["y"])
    pn = rng.permutation(10)
    assert np.array_equal(O.bitlinear_a4(X, W[pn], 0.0)["y"], base4["y"][:, pn])
    # channels permute together in X and W: the integer sums do not change, and alpha, d neither
    pk = rng.permutation(96)
    p4 = O.bitlinear_a4(X[:, pk], W[:, pk], 0.0)
    assert np.array_equal(p4["acc"], base4["acc"]) and np.array_equal(p4["y"], base4["y"])


def test_ste_backward():
    """Section 2.2's straight-through backward of a quantized linear: the hand-worked example, central
    differences of the forward pass in its dequantized operands (the forward is linear in each, so the
    differences are exact up to rounding), torch's autograd of the same dense product, and what the
    estimator means: dX does not depend on the activations or on the Top_k mask, dW is zero in the
    columns of channels no token kept."""
    g = GOLD["ste_backward"]
    dX, dW = O.ste_backward(np.array(g["dY"]), np.array(g["q"]), np.array(g["d"]), np.array(g["T"]), g["alpha"])
    assert dX.tolist() == g["dX"] and dW.tolist() == g["dW"]

    rng = np.random.default_rng(77)
    M, K, N = 5, 12, 7
    X = (rng.standard_normal((M, K)) * 3).astype(F32)
    W = (rng.standard_normal((N, K)) * 0.02).astype(F32)
    lay = O.bitlinear_a8_sparse(X, W, K // 2, EPS)
    q, d, T, alpha = lay["q"], lay["d"], lay["T"], lay["alpha"]
    R = rng.standard_normal((M, N))                                     # dL/dY of the loss L = sum(Y * R)
    dX, dW = O.ste_backward(R, q, d, T, alpha)
    Xq = d.astype(np.float64)[:, None] * q.astype(np.float64)
    Wq = np.float64(alpha) * T.astype(np.float64)

    def loss(xq, wq):                                                   # the forward pass, element by element
        tot = 0.0
        for m in range(M):
            for n in range(N):
                tot += R[m, n] * sum(xq[m, k] * wq[n, k] for k in range(K))
        return tot

    h = 0.5
    for (m, k) in ((0, 0), (2, 5), (4, 11)):
        e = np.zeros_like(Xq)
        e[m, k] = h
        assert abs((loss(Xq + e, Wq) - loss(Xq - e, Wq)) / (2 * h) - dX[m, k]) < 1e-9
    for (n, k) in ((0, 3), (3, 0), (6, 11)):
        e = np.zeros_like(Wq)
        e[n, k] = h
        assert abs((loss(Xq, Wq + e) - loss(Xq, Wq - e)) / (2 * h) - dW[n, k]) < 1e-9

    xt = torch.tensor(Xq, requires_grad=True)
    wt = torch.tensor(Wq, requires_grad=True)
    (xt @ wt.T * torch.tensor(R)).sum().backward()
    assert np.allclose(xt.grad.numpy(), dX, rtol=1e-12, atol=1e-12)
    assert np.allclose(wt.grad.numpy(), dW, rtol=1e-12, atol=1e-12)

    # the estimator passes over Top_k and the quantizer: another token matrix changes dW only
    lay2 = O.bitlinear_a8_sparse(X[::-1].copy() * F32(1.7), W, 2, EPS)
    dX2, dW2 = O.ste_backward(R, lay2["q"], lay2["d"], T, alpha)
    assert np.array_equal(dX2, dX) and not np.array_equal(dW2, dW)
    dead = ~lay2["mask"].any(axis=0)                                    # channels no token kept
    assert dead.any() and not dW2[:, dead].any()
    assert dX[:, ~lay["mask"].all(axis=0)].any()                        # masked entries still get a gradient
    # shapes, and linearity in dY
    assert dX.shape == (M, K) and dW.shape == (N, K)
    a, b = O.ste_backward(2.0 * R, q, d, T, alpha)
    assert np.array_equal(a, 2.0 * dX) and np.array_equal(b, 2.0 * dW)
