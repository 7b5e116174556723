"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Integer codes, masks, index lists and int32 accumulators must be bit-exact;
rescaled outputs within 1e-3 relative (they are in fact bit-exact too, which is also checked
where the rounding order is fixed)."""
import numpy as np
import pytest
import torch

from oracle import bitnet_a48 as O
from paper_2411_04965_amd import binding as B
from paper_2411_04965_amd import synth as S
from tests.gpu_util import (EPS, assert_close_rel, decode_fp4, decode_heads, decode_fp4_mx, decode_int4, decode_int4_mx6,
                            decode_int8, decode_w_gemm, decode_w_kmajor, decode_w_mx2, decode_w_mx4, decode_w_rows, dev, host,
                            pack)

pytestmark = pytest.mark.gpu
BF16 = torch.bfloat16
F32 = torch.float32


def say(msg):
    print("[case] " + msg, flush=True)


# ------------------------------------------------------------------ pack_ternary (eq. 2)
@pytest.mark.parametrize("N,K,dtype", [(512, 256, F32), (256, 512, F32), (37, 100, F32),
                                       (1030, 5460, BF16), (2048, 5460, F32)])
@pytest.mark.parametrize("layout", [B.BL_W_GEMM, B.BL_W_KMAJOR, B.BL_W_MX4, B.BL_W_ROWS, B.BL_W_MX2])
def test_pack_ternary(N, K, dtype, layout):
    say("pack_ternary N=%d K=%d %s layout=%d" % (N, K, dtype, layout))
    W = S.latent_weights(N, K, seed=S.seed_for(0, N + K))
    if dtype == BF16:
        W = S.snap_bf16(W)
    T_ref, alpha_ref = O.ternarize(W, EPS)
    packed, alpha = pack(W, layout, dtype)
    assert host(alpha)[0] == alpha_ref
    T_lib = host(B.unpack_ternary(packed, N, K, layout))
    assert np.array_equal(T_lib, T_ref)
    dec = {B.BL_W_GEMM: decode_w_gemm, B.BL_W_KMAJOR: decode_w_kmajor, B.BL_W_MX4: decode_w_mx4,
           B.BL_W_ROWS: decode_w_rows, B.BL_W_MX2: decode_w_mx2}[layout]
    assert np.array_equal(dec(host(packed), N, K), T_ref)


# ------------------------------------------------------------------ quantize_act
def _x(kind, M, K, seed, dtype):
    if kind == "gauss":
        x = S.gauss_outlier(M, K, max(1, K // 64), 20.0, seed)
    elif kind == "heavy":
        x = S.heavy(M, K, seed)
    elif kind == "glu":
        x = S.glu_like(M, K, seed)
    elif kind == "ties":
        rng = np.random.default_rng(seed)
        x = (np.round(rng.standard_normal((M, K)) * 2) / 2).astype(np.float32)
        x[0] = 0
        x[1 % M] = 1.0
        x[2 % M, ::3] = -0.0
    if dtype == BF16:
        x = S.snap_bf16(x)
    return x


@pytest.mark.parametrize("kind,M,K,dtype", [("gauss", 16, 256, F32), ("heavy", 33, 4096, BF16),
                                            ("gauss", 7, 5460, BF16), ("ties", 9, 1000, F32),
                                            ("gauss", 5, 301, BF16), ("heavy", 3, 11008, BF16)])
def test_quantize_int4(kind, M, K, dtype):
    say("quantize_act INT4 %s M=%d K=%d %s" % (kind, M, K, dtype))
    x = _x(kind, M, K, S.seed_for(0, 7 * M + K), dtype)
    q_ref, d_ref = O.quant_int4(x, EPS)
    r = B.quantize_act(dev(x, dtype), B.BL_ACT_INT4_ABSMEAN, 0, EPS, want_rowsum=True)
    assert np.array_equal(host(r["scale"]), d_ref)
    assert np.array_equal(host(B.unpack_act(r["q"], B.BL_ACT_INT4_ABSMEAN, M, K)), q_ref)
    assert np.array_equal(decode_int4(host(r["q"]), M, K), q_ref)
    assert np.array_equal(host(r["rowsum"]), q_ref.sum(1, dtype=np.int32))
    # the same levels in the form the block-float GEMM reads (E3M2 codes, 32-token blocks)
    r = B.quantize_act(dev(x, dtype), B.BL_ACT_INT4_ABSMEAN_MX6, 0, EPS, want_rowsum=True)
    assert np.array_equal(host(r["scale"]), d_ref)
    assert np.array_equal(host(B.unpack_act(r["q"], B.BL_ACT_INT4_ABSMEAN_MX6, M, K)), q_ref)
    assert np.array_equal(decode_int4_mx6(host(r["q"]), M, K), q_ref)
    assert np.array_equal(host(r["rowsum"]), q_ref.sum(1, dtype=np.int32))


@pytest.mark.parametrize("mode,kind", [(B.BL_ACT_INT4_ABSMEAN2, "absmean2"), (B.BL_ACT_INT4_ABSMAX, "absmax")])
@pytest.mark.parametrize("xkind,M,K,dtype", [("gauss", 16, 256, F32), ("glu", 33, 11008, BF16),
                                             ("ties", 9, 1000, F32), ("heavy", 5, 301, BF16)])
def test_quantize_int4_variants(mode, kind, xkind, M, K, dtype):
    """The two other INT4 quantizers of the ablations (beta = 2 mean|x|; absmax with 7 levels)."""
    say("quantize_act INT4 variant %s %s M=%d K=%d %s" % (kind, xkind, M, K, dtype))
    x = _x(xkind, M, K, S.seed_for(0, 17 * M + K), dtype)
    q_ref, d_ref = O.quant_int4_variant(x, EPS, kind)
    r = B.quantize_act(dev(x, dtype), mode, 0, EPS, want_rowsum=True)
    assert np.array_equal(host(r["scale"]), d_ref)
    assert np.array_equal(decode_int4(host(r["q"]), M, K), q_ref)
    assert np.array_equal(host(B.unpack_act(r["q"], mode, M, K)), q_ref)
    assert np.array_equal(host(r["rowsum"]), q_ref.sum(1, dtype=np.int32))
    # the linear layers take these codes as INT4 codes
    N = 64
    W = S.latent_weights(N, K, S.seed_for(0, 18))
    T, alpha = O.ternarize(W, EPS)
    p, a = pack(W)
    Y, acc = B.bitlinear_gemm(r["q"], r["scale"], mode, M, K, p, a, N, y_dtype=F32, want_acc=True)
    acc_ref = O.matmul_int(q_ref, T)
    assert np.array_equal(host(acc), acc_ref)
    assert np.array_equal(host(Y), O.rescale(acc_ref, d_ref, alpha, "f32"))


@pytest.mark.parametrize("kind,M,K,topk,dtype", [
    ("gauss", 16, 512, 256, F32), ("heavy", 33, 4096, 2048, BF16), ("glu", 9, 5460, 2730, BF16),
    ("ties", 9, 1000, 500, F32), ("ties", 9, 1000, 1, BF16), ("ties", 9, 1000, 1000, BF16),
    ("gauss", 5, 301, 77, BF16), ("glu", 4, 11008, 5504, BF16), ("heavy", 2, 8640, 4320, BF16)])
def test_quantize_topk_int8(kind, M, K, topk, dtype):
    say("quantize_act TOPK %s M=%d K=%d topk=%d %s" % (kind, M, K, topk, dtype))
    x = _x(kind, M, K, S.seed_for(0, 11 * M + K + topk), dtype)
    q_ref, d_ref, mask_ref = O.quant_topk_int8(x, topk, EPS)
    r = B.quantize_act(dev(x, dtype), B.BL_ACT_TOPK_INT8_ABSMAX, topk, EPS, want_rowsum=True,
                       want_sel=True)
    assert np.array_equal(host(r["scale"]), d_ref)
    q_gpu = decode_int8(host(r["q"]), M, K)
    assert np.array_equal(q_gpu, q_ref)
    assert np.array_equal(host(B.unpack_act(r["q"], B.BL_ACT_TOPK_INT8_ABSMAX, M, K)), q_ref)
    sel = host(r["sel"])
    assert sel.shape == (M, topk)
    for m in range(M):                                   # exactly topk channels, ascending
        assert np.array_equal(sel[m], np.flatnonzero(mask_ref[m]))
    assert np.array_equal(host(r["rowsum"]), q_ref.sum(1, dtype=np.int32))


@pytest.mark.parametrize("kind,M,K,topk", [
    ("ties", 2051, 1000, 500), ("heavy", 2051, 4096, 2048), ("glu", 2050, 5460, 2730), ("ties", 2049, 5460, 1),
    ("heavy", 2051, 8640, 4320), ("glu", 2051, 11008, 5504), ("ties", 2048, 12288, 12288), ("ties", 2051, 11008, 5504),
    ("heavy", 2049, 8000, 4000)])
def test_quantize_topk_int8_many_tokens(kind, M, K, topk):
    """From 2048 tokens on the selection runs with one or two waves per token (no index lists asked for):
    every register-block count, a last workgroup that is not full, heavy ties, topk = 1 and = K."""
    say("quantize_act TOPK many tokens %s M=%d K=%d topk=%d" % (kind, M, K, topk))
    x = _x(kind, M, K, S.seed_for(0, 13 * M + K + topk), BF16)
    rows = np.unique(np.concatenate([np.arange(0, M, 9), [1, 2, M - 3, M - 2, M - 1]]))
    q_ref, d_ref, _ = O.quant_topk_int8(x[rows], topk, EPS)
    r = B.quantize_act(dev(x, BF16), B.BL_ACT_TOPK_INT8_ABSMAX, topk, EPS, want_rowsum=True)
    assert np.array_equal(host(r["scale"])[rows], d_ref)
    assert np.array_equal(decode_int8(host(r["q"]), M, K)[rows], q_ref)
    assert np.array_equal(host(r["rowsum"])[rows], q_ref.sum(1, dtype=np.int32))


def test_quantize_topk_int8_seeded_sweep():
    """40 seeded draws of (tokens, width, topk, input kind) over the register kernels' range: widths
    that are multiples of 4 up to 12288, few and many tokens, topk from 1 to K, inputs with many
    equal magnitudes (coarse grids, zeros) so that the threshold falls inside a run of ties."""
    rng = np.random.default_rng(S.seed_for(0, 4242))
    for it in range(40):
        many = it % 4 == 3
        M = int(rng.integers(2048, 2080)) if many else int(rng.integers(1, 70))
        K = 4 * int(rng.integers(1, 1537 if many else 3073))
        topk = int(rng.choice([1, K, max(1, K // 2), int(rng.integers(1, K + 1))]))
        kind = ["ties", "glu", "heavy", "grid"][it % 4 if not many else int(rng.integers(0, 4))]
        say("sweep %d: M=%d K=%d topk=%d %s" % (it, M, K, topk, kind))
        if kind == "grid":          # a handful of distinct magnitudes: long runs of equal keys
            x = (rng.integers(-3, 4, (M, K)) * 0.5).astype(np.float32)
        else:
            x = _x(kind, M, K, S.seed_for(0, 5000 + it), BF16)
        rows = np.arange(M) if M < 70 else np.unique(rng.integers(0, M, 48))
        q_ref, d_ref, _ = O.quant_topk_int8(x[rows], topk, EPS)
        r = B.quantize_act(dev(x, BF16), B.BL_ACT_TOPK_INT8_ABSMAX, topk, EPS, want_rowsum=True)
        assert np.array_equal(host(r["scale"])[rows], d_ref)
        assert np.array_equal(decode_int8(host(r["q"]), M, K)[rows], q_ref)
        assert np.array_equal(host(r["rowsum"])[rows], q_ref.sum(1, dtype=np.int32))


def _rows_around_the_shortcut(M, K, n_big, seed):
    """Rows with exactly n_big values within 8 binades of the row maximum; the rest are zeros or values
    below gamma / 256 (their codes are 0 whether Top_k keeps them or not), some of them equal to each other."""
    rng = np.random.default_rng(seed)
    x = np.zeros((M, K), np.float32)
    for m in range(M):
        big = rng.choice(K, n_big, replace=False)
        x[m, big] = (rng.standard_normal(n_big) * 3 + np.sign(rng.standard_normal(n_big)) * 0.5).astype(np.float32)
        x[m, big[0]] = 40.0                                                    # the row maximum: gamma / 256 = 0.156
        x[m, big] = np.where(np.abs(x[m, big]) < 0.2, 0.25, x[m, big])
        small = np.setdiff1d(np.arange(K), big)
        tiny = rng.choice(small, len(small) // 3, replace=False)
        x[m, tiny] = (rng.integers(1, 5, len(tiny)) * 0.03125 * np.sign(rng.standard_normal(len(tiny)))).astype(np.float32)
    return S.snap_bf16(x)


@pytest.mark.parametrize("M,K", [(3, 11008), (2050, 5460), (2, 4096), (40, 9000)])
def test_quantize_topk_shortcut_boundary(M, K):
    """The Top-K kernels skip the threshold search when no more than topk keys lie within 8 binades of the
    row maximum: topk one below, at and one above that count, and far above it, on rows whose remaining
    values are zeros and tied small values; codes, scales and code sums bit for bit the oracle's.  Covers
    the four-wave, the one-wave and (through the decode linear, one token) the eight-wave body."""
    n_big = K // 5
    x = _rows_around_the_shortcut(M, K, n_big, S.seed_for(0, 77 + K))
    rows = np.arange(M) if M < 64 else np.array([0, 1, 7, M // 2, M - 1])
    for topk in (n_big - 1, n_big, n_big + 1, K // 2, K):
        say("shortcut boundary M=%d K=%d n_big=%d topk=%d" % (M, K, n_big, topk))
        q_ref, d_ref, _ = O.quant_topk_int8(x[rows], topk, EPS)
        r = B.quantize_act(dev(x, BF16), B.BL_ACT_TOPK_INT8_ABSMAX, topk, EPS, want_rowsum=True)
        assert np.array_equal(host(r["scale"])[rows], d_ref)
        assert np.array_equal(decode_int8(host(r["q"]), M, K)[rows], q_ref)
        assert np.array_equal(host(r["rowsum"])[rows], q_ref.sum(1, dtype=np.int32))
    # one token through the decode linear (the selection runs inside the GEMV launch)
    N = 2064
    W = S.latent_weights(N, K, S.seed_for(0, 78 + K))
    p, a = pack(W)
    for topk in (n_big - 1, n_big, n_big + 1, K // 2):
        ref = O.bitlinear_a8_sparse(x[:1], W, topk, EPS, "f32")
        _check_linear(B.bitlinear_a8_sparse(dev(x[:1], BF16), topk, p, a, N, EPS, B.BL_W_GEMM, F32, True), ref, F32)


@pytest.mark.parametrize("M,K,topk,dtype", [(9, 5460, 2730, F32), (2051, 5460, 2730, F32), (33, 11008, 5504, BF16),
                                            (2050, 4096, 2048, BF16), (5, 1000, 1, BF16), (7, 12288, 12288, F32)])
def test_quantize_glu_topk_int8(M, K, topk, dtype):
    """eq. 5 folded into the top-K quantizer's load: codes, scales and code sums equal those of the
    oracle's ReLU^2 GLU followed by its top-K + INT8 quantizer, and of the two separate kernels."""
    say("quantize_act_glu M=%d K=%d topk=%d %s" % (M, K, topk, dtype))
    g = S.heavy(M, K, S.seed_for(1, 70 + M))
    u = S.heavy(M, K, S.seed_for(1, 71 + K))
    g[0] = -np.abs(g[0])                                   # a token whose gate is closed everywhere
    if dtype == BF16:
        g, u = S.snap_bf16(g), S.snap_bf16(u)
    rows = np.unique(np.concatenate([np.arange(0, M, 11), [0, M - 1]]))
    h_ref = O.relu2_glu(g[rows], u[rows])
    q_ref, d_ref, _ = O.quant_topk_int8(h_ref, topk, EPS)
    r = B.quantize_act_glu(dev(g, dtype), dev(u, dtype), topk, EPS, want_rowsum=True)
    assert np.array_equal(host(r["scale"])[rows], d_ref)
    assert np.array_equal(decode_int8(host(r["q"]), M, K)[rows], q_ref)
    assert np.array_equal(host(r["rowsum"])[rows], q_ref.sum(1, dtype=np.int32))
    r2 = B.quantize_act(B.relu2_glu(dev(g, dtype), dev(u, dtype)), B.BL_ACT_TOPK_INT8_ABSMAX, topk, EPS)
    assert torch.equal(r2["q"], r["q"]) and torch.equal(r2["scale"], r["scale"])


@pytest.mark.parametrize("kind,M,K,dtype", [("gauss", 16, 256, F32), ("heavy", 20, 3200, BF16),
                                            ("glu", 6, 8640, BF16), ("ties", 9, 992, F32)])
def test_quantize_fp4(kind, M, K, dtype):
    say("quantize_act FP4 %s M=%d K=%d %s" % (kind, M, K, dtype))
    x = _x(kind, M, K, S.seed_for(4, M + K), dtype)
    x[M - 1, :32] *= 1e-30                                # tiny block
    if dtype == BF16:
        x = S.snap_bf16(x)
    codes_ref, e_ref = O.quant_fp4(x)
    r = B.quantize_act(dev(x, dtype), B.BL_ACT_FP4_E2M1_B32)
    Kp = B.padded_k(K)
    sc = host(r["scale"]).reshape(M, Kp // 32)
    assert np.array_equal(sc[:, :K // 32].astype(np.int16) - 127, e_ref)
    assert np.all(sc[:, K // 32:] == 127)
    assert np.array_equal(decode_fp4(host(r["q"]), M, K), codes_ref)
    lib_codes = host(B.unpack_act(r["q"], B.BL_ACT_FP4_E2M1_B32, M, K)).view(np.uint8)
    assert np.array_equal(lib_codes, codes_ref)
    # the same codes and scales in the block order of the block-float GEMM
    r = B.quantize_act(dev(x, dtype), B.BL_ACT_FP4_E2M1_B32_MX)
    codes_mx, e_mx = decode_fp4_mx(host(r["q"]), host(r["scale"]), M, K)
    assert np.array_equal(codes_mx, codes_ref)
    assert np.array_equal(e_mx[:, :K // 32].astype(np.int16) - 127, e_ref)
    assert np.all(e_mx[:, K // 32:] == 127)
    lib_codes = host(B.unpack_act(r["q"], B.BL_ACT_FP4_E2M1_B32_MX, M, K)).view(np.uint8)
    assert np.array_equal(lib_codes, codes_ref)


@pytest.mark.parametrize("kind,M,K,dtype", [("gauss", 16, 256, F32), ("heavy", 20, 3200, BF16),
                                            ("glu", 6, 8640, BF16), ("ties", 9, 992, F32)])
def test_quantize_fp4_e1m2(kind, M, K, dtype):
    """Section 4.3's E1M2 arm of eq. 8-9: codes and block exponents bit for bit; the linear entry
    points refuse the format (no matrix instruction takes it)."""
    say("quantize_act FP4 E1M2 %s M=%d K=%d %s" % (kind, M, K, dtype))
    x = _x(kind, M, K, S.seed_for(4, 50 + M + K), dtype)
    x[M - 1, :32] *= 1e-30                                # tiny block
    x[0, 32:64] = 0                                       # empty block
    x[1, 64:96] = np.linspace(-1.75, 1.75, 32)            # the top value and ties at multiples of 1/8
    if dtype == BF16:
        x = S.snap_bf16(x)
    codes_ref, e_ref = O.quant_fp4(x, "e1m2")
    r = B.quantize_act(dev(x, dtype), B.BL_ACT_FP4_E1M2_B32)
    Kp = B.padded_k(K)
    sc = host(r["scale"]).reshape(M, Kp // 32)
    assert np.array_equal(sc[:, :K // 32].astype(np.int16) - 127, e_ref)
    assert np.all(sc[:, K // 32:] == 127)
    assert np.array_equal(decode_fp4(host(r["q"]), M, K), codes_ref)
    lib_codes = host(B.unpack_act(r["q"], B.BL_ACT_FP4_E1M2_B32, M, K)).view(np.uint8)
    assert np.array_equal(lib_codes, codes_ref)
    W = S.latent_weights(32, K, S.seed_for(4, 51))
    pw, aw = pack(W)
    Y = torch.empty((M, 32), dtype=torch.float32, device="cuda")
    rc = B.lib().bitlinear_gemm(r["q"].data_ptr(), r["scale"].data_ptr(), B.BL_ACT_FP4_E1M2_B32, M, K,
                                pw.data_ptr(), B.BL_W_GEMM, aw.data_ptr(), 32, Y.data_ptr(), B.BL_F32,
                                None, None, 0, None)
    assert rc == -6, rc                                   # BL_EUNSUPPORTED


@pytest.mark.parametrize("M,N,dtype", [(7, 300, F32), (33, 5460, BF16), (1, 1, F32), (64, 11008, BF16)])
def test_swish_glu(M, N, dtype):
    """Section 4.3's Swish GLU against the exactly evaluated function: at most one bfloat16 ulp off
    (2^-100 absolute for results smaller than that), and that only where the float32 chain's error
    straddles a rounding boundary (rare)."""
    say("swish_glu M=%d N=%d %s" % (M, N, dtype))
    g = S.heavy(M, N, S.seed_for(6, M + N))
    u = S.heavy(M, N, S.seed_for(6, M + N + 1))
    g.flat[:4] = [0.0, -200.0, 200.0, -1.27846][:g.size if g.size < 4 else 4]
    if dtype == BF16:
        g, u = S.snap_bf16(g), S.snap_bf16(u)
    else:
        g, u = g.astype(np.float32), u.astype(np.float32)
    h_ref = O.swish_glu(g, u)
    Hh = host(B.swish_glu(dev(g, dtype), dev(u, dtype))).astype(np.float32)
    assert not np.isnan(Hh).any()
    ulp = np.exp2(np.floor(np.log2(np.maximum(np.abs(h_ref), 2.0 ** -126))) - 7)
    diff = np.abs(Hh.astype(np.float64) - h_ref.astype(np.float64))
    # (below g = -88.7 float32 exp(-g) overflows and the result is 0 instead of about 1e-40)
    assert np.all(diff <= np.maximum(ulp, 2.0 ** -100)), float((diff / ulp).max())
    assert (diff > 0).mean() <= 0.002, float((diff > 0).mean())


@pytest.mark.parametrize("T,H,D,dtype", [(5, 3, 128, BF16), (33, 32, 128, BF16), (7, 4, 64, F32), (9, 2, 96, BF16),
                                         (6, 5, 80, BF16), (3, 2, 256, F32), (4, 1, 8, BF16), (2048, 32, 128, BF16)])
@pytest.mark.parametrize("bits", [4, 3])
def test_quantize_heads(T, H, D, dtype, bits):
    """Section 4.2's per-head absmax quantizer of the attention states (4 and 3 bits, unsigned codes):
    codes and scales bit for bit against the oracle, both kernels (a head per 16 lanes; a head per
    wave), head widths that fill and do not fill the 16 lanes, an all-zero head."""
    say("quantize_heads T=%d H=%d D=%d %s bits=%d" % (T, H, D, dtype, bits))
    x = S.heavy(T * H, D, S.seed_for(7, T + H + D)).reshape(T, H, D)
    x[0, 0] = 0
    x[T - 1, H - 1, :4] = [3.5, -3.5, 1.5, -0.5]          # ties after scaling when the maximum is 7 or 3
    x[T - 1, H - 1, 4] = 7.0 if bits == 4 else 3.0
    x[T - 1, H - 1, 5:] = 0
    x = S.snap_bf16(x) if dtype == BF16 else x.astype(np.float32)
    codes_ref, d_ref = O.quant_heads(x, bits, EPS)
    q, d = B.quantize_heads(dev(x, dtype), bits, EPS)
    assert q.numel() == T * H * D * bits // 8
    assert np.array_equal(host(d), d_ref)
    assert np.array_equal(decode_heads(host(q), T, H, D, bits), codes_ref)


# ------------------------------------------------------------------ whole linears
@pytest.mark.parametrize("T,H,D", [(5, 3, 128), (33, 32, 128), (9, 2, 96), (3, 2, 256)])
@pytest.mark.parametrize("bits", [4, 3])
def test_dequantize_heads(T, H, D, bits):
    """Codes of the per-head quantizer read back: (code - 2^(bits-1)) * scale, bit for bit the oracle's."""
    say("dequantize heads T=%d H=%d D=%d bits=%d" % (T, H, D, bits))
    X = S.heavy(T, H * D, S.seed_for(5, 40 + T)).reshape(T, H, D)
    codes, d = O.quant_heads(X, bits, EPS)
    want = O.dequant_heads(codes, d, bits)
    q, sc = B.quantize_heads(dev(X, BF16), bits, EPS)
    assert np.array_equal(host(B.dequantize_heads(q, sc, T, H, D, bits, F32)), want)
    assert np.array_equal(host(B.dequantize_heads(q, sc, T, H, D, bits, BF16)), O.bf16_round(want))


@pytest.mark.parametrize("T,H,D,dtype", [(7, 3, 128, BF16), (40, 32, 128, BF16), (5, 2, 64, F32), (1, 4, 96, BF16)])
def test_kv_cache_mixed_width(T, H, D, dtype):
    """Table 3's key / value cache (first token at 4 bits, later tokens at 3): a prefill append of the first
    tokens and one-token appends after it give the oracle's bytes and scales; whole and partial reads give
    its values."""
    say("kv cache T=%d H=%d D=%d" % (T, H, D))
    X = S.heavy(T, H * D, S.seed_for(5, 60 + T)).reshape(T, H, D) if dtype == BF16 else \
        S.gauss_outlier(T, H * D, 4, 20.0, S.seed_for(5, 61 + T)).reshape(T, H, D)
    raw, d = O.kv_cache_pack(X, EPS)
    vals = O.kv_cache_unpack(raw, d, T, H, D)
    assert B.lib().kv_cache_bytes(T, H, D) == raw.size
    cache, scales = B.kv_cache_new(T, H, D, "cuda")
    Xd = dev(X.reshape(T, H * D), dtype).reshape(T, H, D)
    t_pre = max(1, T // 2)
    B.kv_cache_append(Xd[:t_pre].contiguous(), 0, cache, scales, EPS)
    for t in range(t_pre, T):
        B.kv_cache_append(Xd[t:t + 1].contiguous(), t, cache, scales, EPS)
    assert np.array_equal(cache.cpu().numpy(), raw)
    assert np.array_equal(host(scales), d)
    assert np.array_equal(host(B.kv_cache_read(cache, scales, 0, T, H, D, F32)), vals)
    assert np.array_equal(host(B.kv_cache_read(cache, scales, 0, T, H, D, BF16)), O.bf16_round(vals))
    if T > 2:
        assert np.array_equal(host(B.kv_cache_read(cache, scales, 1, T - 2, H, D, F32)), vals[1:T - 1])
    L = B.lib()
    assert L.kv_cache_bytes(4, 2, 12) == 0
    assert L.kv_cache_append(Xd.data_ptr(), B.BL_BF16, 1, 2, 48, 0, EPS, cache.data_ptr(), scales.data_ptr(), None) == -2  # D % 32
    assert L.kv_cache_read(cache.data_ptr(), scales.data_ptr(), -1, 1, H, D, Xd.data_ptr(), B.BL_BF16, None) == -1


def _check_linear(res, ref, y_dtype):
    Y, acc = res
    assert np.array_equal(host(acc), ref["acc"]), "int32 accumulators differ"
    assert_close_rel(host(Y), ref["y"])
    assert np.array_equal(host(Y), ref["y"]), "rescaled output not bit-exact"


def test_config0_pair():
    """Single BitLinear pair: A4 256->512 on 16 tokens, then A8-sparse 512->256 (top-256)."""
    say("config 0 pair")
    X = S.gauss_outlier(16, 256, 4, 20.0, S.seed_for(0, 0))
    W1 = S.latent_weights(512, 256, S.seed_for(0, 1))
    W2 = S.latent_weights(256, 512, S.seed_for(0, 2))
    ref1 = O.bitlinear_a4(X, W1, EPS, "f32")
    p1, a1 = pack(W1)
    Y1, acc1 = B.bitlinear_a4(dev(X), p1, a1, 512, EPS, y_dtype=F32, want_acc=True)
    _check_linear((Y1, acc1), ref1, F32)
    # chained: the sparse linear consumes Y1
    ref2 = O.bitlinear_a8_sparse(ref1["y"], W2, 256, EPS, "f32")
    for layout in (B.BL_W_GEMM, B.BL_W_KMAJOR):
        p2, a2 = pack(W2, layout)
        if layout == B.BL_W_KMAJOR:
            res = B.bitlinear_a8_sparse(Y1[:8].contiguous(), 256, p2, a2, 256, EPS, layout, F32, True)
            sub = dict(acc=ref2["acc"][:8], y=ref2["y"][:8])
            _check_linear(res, sub, F32)
        else:
            res = B.bitlinear_a8_sparse(Y1, 256, p2, a2, 256, EPS, layout, F32, True)
            _check_linear(res, ref2, F32)
    # independent sparse input
    X2 = S.gauss_outlier(16, 512, 8, 20.0, S.seed_for(0, 3))
    ref3 = O.bitlinear_a8_sparse(X2, W2, 256, EPS, "bf16")
    p2, a2 = pack(W2)
    _check_linear(B.bitlinear_a8_sparse(dev(X2), 256, p2, a2, 256, EPS, B.BL_W_GEMM, BF16, True), ref3, BF16)
    assert np.all((ref3["q"] != 0).sum(1) <= 256) and np.all(ref3["mask"].sum(1) == 256)


@pytest.mark.parametrize("M,N,K", [(300, 520, 1000), (130, 2048, 5460), (257, 5460, 2048),
                                   (1100, 1100, 768)])
def test_prefill_gemm_shapes(M, N, K):
    """Several tiles, ragged M / N / K tails, both tile sizes, both activation formats."""
    say("prefill M=%d N=%d K=%d" % (M, N, K))
    X = S.heavy(M, K, S.seed_for(1, M + N))
    W = S.latent_weights(N, K, S.seed_for(1, K + N + 1))
    p, a = pack(W)
    ref = O.bitlinear_a4(X, W, EPS, "bf16")
    _check_linear(B.bitlinear_a4(dev(X, BF16), p, a, N, EPS, y_dtype=BF16, want_acc=True), ref, BF16)
    Xs = S.glu_like(M, K, S.seed_for(1, M + N + 7))
    ref = O.bitlinear_a8_sparse(Xs, W, K // 2, EPS, "bf16")
    _check_linear(B.bitlinear_a8_sparse(dev(Xs, BF16), K // 2, p, a, N, EPS, B.BL_W_GEMM, BF16, True), ref, BF16)


def test_config1_ffn_block():
    """One FFN block at 1.3B width: 2048 tokens, 2048 -> 5460 (gate, up), ReLU^2 GLU, top-2730 + INT8 -> 2048."""
    say("config 1 ffn block")
    M, H, Fd = 2048, 2048, 5460
    X = S.heavy(M, H, S.seed_for(1, 0))
    Wg = S.latent_weights(Fd, H, S.seed_for(1, 1))
    Wu = S.latent_weights(Fd, H, S.seed_for(1, 2))
    Wd = S.latent_weights(H, Fd, S.seed_for(1, 3))
    ref = O.ffn_block(X, Wg, Wu, Wd, Fd // 2, EPS)
    pg, ag = pack(Wg)
    pu, au = pack(Wu)
    pd, ad = pack(Wd)
    Xd = dev(X, BF16)
    G, accg = B.bitlinear_a4(Xd, pg, ag, Fd, EPS, y_dtype=F32, want_acc=True)
    U, accu = B.bitlinear_a4(Xd, pu, au, Fd, EPS, y_dtype=F32, want_acc=True)
    _check_linear((G, accg), ref["gate"], F32)
    _check_linear((U, accu), ref["up"], F32)
    Hh = B.relu2_glu(G, U)
    assert np.array_equal(host(Hh), ref["h"])
    Yd, accd = B.bitlinear_a8_sparse(Hh, Fd // 2, pd, ad, H, EPS, B.BL_W_GEMM, BF16, True)
    _check_linear((Yd, accd), ref["down"], BF16)


# ------------------------------------------------------------------ decode shapes (config 2)
DECODE = [("qkv", 12288, 4096, "a4"), ("o", 4096, 4096, "a8s"), ("gate", 11008, 4096, "a4"),
          ("down", 4096, 11008, "a8s")]
_wcache = {}


def _decode_weights(name, N, K):
    if name not in _wcache:
        W = S.latent_weights(N, K, S.seed_for(2, len(name) + N))
        T, alpha = O.ternarize(W, EPS)
        packs = {B.BL_W_GEMM: pack(W)}
        if name in ("o", "down"):
            packs[B.BL_W_KMAJOR] = pack(W, B.BL_W_KMAJOR)
        else:
            packs[B.BL_W_MX4] = pack(W, B.BL_W_MX4)
            packs[B.BL_W_MX2] = pack(W, B.BL_W_MX2)
        _wcache[name] = (T, alpha, packs)
    return _wcache[name]


@pytest.mark.parametrize("name,N,K,kind", DECODE)
@pytest.mark.parametrize("M", [1, 8, 32, 64])
def test_config2_decode(name, N, K, kind, M):
    say("config 2 decode %s M=%d" % (name, M))
    T, alpha, packs = _decode_weights(name, N, K)
    if kind == "a4":
        X = S.heavy(M, K, S.seed_for(2, 100 + M))
        q, d = O.quant_int4(X, EPS)
    else:
        X = S.glu_like(M, K, S.seed_for(2, 200 + M)) if name == "down" else S.heavy(M, K, S.seed_for(2, 300 + M))
        q, d, _ = O.quant_topk_int8(X, K // 2, EPS)
    acc = O.matmul_int(q, T)
    ref = dict(acc=acc, y=O.rescale(acc, d, alpha, "bf16"))
    Xd = dev(X, BF16)
    for layout, (p, a) in packs.items():
        if layout == B.BL_W_KMAJOR and M > 8:
            continue
        assert host(a)[0] == alpha
        if kind == "a4":
            res = B.bitlinear_a4(Xd, p, a, N, EPS, y_dtype=BF16, want_acc=True, layout=layout)
        else:
            res = B.bitlinear_a8_sparse(Xd, K // 2, p, a, N, EPS, layout, BF16, True)
        _check_linear(res, ref, BF16)


@pytest.mark.parametrize("M", [1, 8, 32])
def test_decode_graph_replays(M):
    """The decode linears inside a captured graph, as the benchmark times them: every replay gives
    the oracle's bits, with other work on the same buffers and synchronisations between replays
    (the kernels keep partial sums and counters in the workspace, so a replay must not depend on
    what the one before left there)."""
    say("decode graph replays M=%d" % M)
    cases = []
    for name, N, K, kind in (("gate", 1024, 2048, "a4"), ("down", 2048, 2816, "a8")):
        W = S.latent_weights(N, K, S.seed_for(2, 900 + N))
        T, alpha = O.ternarize(W, EPS)
        X = S.heavy(M, K, S.seed_for(2, 901 + M)) if kind == "a4" else S.glu_like(M, K, S.seed_for(2, 902 + M))
        if kind == "a4":
            q, d = O.quant_int4(X, EPS)
            mode = B.BL_ACT_INT4_ABSMEAN
        else:
            q, d, _ = O.quant_topk_int8(X, K // 2, EPS)
            mode = B.BL_ACT_TOPK_INT8_ABSMAX
        y_ref = O.rescale(O.matmul_int(q, T), d, alpha, "bf16")
        p, a = pack(W)
        Xd = dev(X, BF16)
        ws = B.workspace(mode, M, N, K, "cuda")
        Y = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        cases.append((kind, N, K, p, a, Xd, ws, Y, y_ref))

    def run():
        for kind, N, K, p, a, Xd, ws, Y, _ in cases:
            if kind == "a4":
                B.bitlinear_a4(Xd, p, a, N, EPS, ws=ws, out=Y)
            else:
                B.bitlinear_a8_sparse(Xd, K // 2, p, a, N, EPS, ws=ws, out=Y)

    run()
    torch.cuda.synchronize()
    for c in cases:
        assert np.array_equal(host(c[7]), c[8])
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            run()
    for rep in range(4):
        for c in cases:                                    # eager work between the replays: outputs and
            c[7].fill_(float(rep + 1))                     # workspaces overwritten with other values
            c[6].fill_(0x5A + rep)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for c in cases:
            assert np.array_equal(host(c[7]), c[8]), "replay %d differs" % rep
    del g


@pytest.mark.parametrize("M", [3, 17, 48])
def test_decode_odd_shapes(M):
    say("decode odd shapes M=%d" % M)
    N, K = 1000, 1500
    X = S.heavy(M, K, S.seed_for(2, 400 + M))
    W = S.latent_weights(N, K, S.seed_for(2, 401))
    p, a = pack(W)
    _check_linear(B.bitlinear_a4(dev(X, BF16), p, a, N, EPS, y_dtype=F32, want_acc=True),
                  O.bitlinear_a4(X, W, EPS, "f32"), F32)
    ref = O.bitlinear_a8_sparse(X, W, 700, EPS, "f32")
    _check_linear(B.bitlinear_a8_sparse(dev(X, BF16), 700, p, a, N, EPS, B.BL_W_GEMM, F32, True), ref, F32)
    if M <= 8:
        pk, ak = pack(W, B.BL_W_KMAJOR)
        _check_linear(B.bitlinear_a8_sparse(dev(X, BF16), 700, pk, ak, N, EPS, B.BL_W_KMAJOR, F32, True), ref, F32)


@pytest.mark.parametrize("M,N,K", [(1, 2064, 1504), (1, 4096, 2056), (1, 2050, 4096), (1, 2048, 256), (1, 2048, 8192),
                                   (2, 2064, 1500), (4, 2050, 4096)])
def test_decode_fused_int4(M, N, K):
    """One token with at least 128 output tiles: eq. 7 runs inside the GEMV launch (K with and
    without a ragged last tile, N ragged, the widest row it takes); two and four tokens, and a row
    that is only 8-byte aligned, take the two-launch path."""
    say("decode fused int4 M=%d N=%d K=%d" % (M, N, K))
    X = S.heavy(M, K, S.seed_for(2, 500 + M))
    W = S.latent_weights(N, K, S.seed_for(2, 501 + N))
    p, a = pack(W)
    for dt, name in ((F32, "f32"), (BF16, "bf16")):
        _check_linear(B.bitlinear_a4(dev(X, BF16), p, a, N, EPS, y_dtype=dt, want_acc=True),
                      O.bitlinear_a4(X, W, EPS, name), dt)


@pytest.mark.parametrize("M,N,K", [(1, 12288, 4096), (2, 37, 256), (3, 2050, 1000), (5, 11008, 4096), (8, 4112, 8192),
                                   (7, 1040, 2048), (8, 40000, 512), (1, 16, 8), (6, 200, 1504), (2, 16384, 8192)])
def test_decode_stream_int4_quantizer_inside(M, N, K):
    """Up to 8 bfloat16 tokens: eq. 7 runs inside the one persistent launch (every register variant of
    the in-kernel quantizer, ragged N and K, one to eight output tiles per workgroup, fewer tiles
    than waves, more tiles than one round of loads)."""
    say("decode stream int4 (quantizer inside) M=%d N=%d K=%d" % (M, N, K))
    assert B.lib().bitlinear_workspace_bytes(B.BL_ACT_INT4_ABSMEAN, M, N, K) > 0
    X = S.heavy(M, K, S.seed_for(2, 520 + M))
    W = S.latent_weights(N, K, S.seed_for(2, 521 + N))
    p, a = pack(W)
    for dt, name in ((F32, "f32"), (BF16, "bf16")):
        _check_linear(B.bitlinear_a4(dev(X, BF16), p, a, N, EPS, y_dtype=dt, want_acc=True),
                      O.bitlinear_a4(X, W, EPS, name), dt)


@pytest.mark.parametrize("M,N,K,kind", [(9, 12288, 4096, "a4"), (16, 2050, 1000, "a4"), (12, 4096, 4096, "a8s"),
                                        (16, 11008, 4096, "a4"), (8, 4096, 11008, "a8s"), (5, 2064, 5460, "a8s"),
                                        (3, 1040, 2048, "a4f32"), (16, 300, 8192, "a8s")])
def test_decode_stream_codes_from_quantizer(M, N, K, kind):
    """2 to 16 tokens through the stand-alone quantizer and the persistent launch (INT4 nibbles
    expanded into LDS, INT8 codes copied), float32 inputs included."""
    say("decode stream (codes from the quantizer) M=%d N=%d K=%d %s" % (M, N, K, kind))
    W = S.latent_weights(N, K, S.seed_for(2, 541 + N))
    p, a = pack(W)
    if kind.startswith("a4"):
        X = S.heavy(M, K, S.seed_for(2, 540 + M))
        xd = dev(X, F32 if kind == "a4f32" else BF16)
        for dt, name in ((F32, "f32"), (BF16, "bf16")):
            _check_linear(B.bitlinear_a4(xd, p, a, N, EPS, y_dtype=dt, want_acc=True), O.bitlinear_a4(X, W, EPS, name), dt)
    else:
        X = S.glu_like(M, K, S.seed_for(2, 542 + M))
        for dt, name in ((F32, "f32"), (BF16, "bf16")):
            _check_linear(B.bitlinear_a8_sparse(dev(X, BF16), K // 2, p, a, N, EPS, B.BL_W_GEMM, dt, True),
                          O.bitlinear_a8_sparse(X, W, K // 2, EPS, name), dt)


@pytest.mark.parametrize("M,N,K,layout", [(1, 11008, 4096, B.BL_W_GEMM), (4, 11008, 4096, B.BL_W_GEMM),
                                          (8, 5460, 2048, B.BL_W_GEMM), (3, 37, 256, B.BL_W_GEMM),
                                          (2, 2050, 1000, B.BL_W_GEMM), (8, 16400, 512, B.BL_W_GEMM),
                                          (20, 1040, 2048, B.BL_W_GEMM), (130, 520, 1000, B.BL_W_MX2),
                                          (32, 11008, 4096, B.BL_W_GEMM), (64, 11008, 4096, B.BL_W_GEMM),
                                          (17, 37, 256, B.BL_W_GEMM), (33, 2050, 1000, B.BL_W_GEMM), (12, 11008, 4096, B.BL_W_GEMM),
                                          (16, 2050, 1000, B.BL_W_GEMM), (9, 37, 256, B.BL_W_GEMM),
                                          (50, 5460, 2048, B.BL_W_GEMM), (64, 1030, 8192, B.BL_W_GEMM),
                                          (70, 300, 512, B.BL_W_GEMM), (300, 5460, 2048, B.BL_W_MX2),
                                          (257, 330, 1504, B.BL_W_MX4), (513, 333, 256, B.BL_W_MX2),
                                          (2048, 5460, 2048, B.BL_W_MX2)])
def test_gate_up(M, N, K, layout):
    """Gate and up projection on one quantized input (eq. 5-7): G, U and H = bf16(U * max(G, 0)^2)
    against the oracle's two linears and its GLU, bit for bit -- the one-launch form for up to 8
    tokens, and the composed form (decode kernels, int8 GEMM, block-float GEMM) for the rest; every
    combination of outputs the entry point can be asked for."""
    say("gate/up M=%d N=%d K=%d layout=%d" % (M, N, K, layout))
    X = S.heavy(M, K, S.seed_for(2, 800 + M))
    Wg = S.latent_weights(N, K, S.seed_for(2, 801 + N))
    Wu = S.latent_weights(N, K, S.seed_for(2, 802 + K))
    g = O.bitlinear_a4(X, Wg, EPS, "f32")["y"]
    u = O.bitlinear_a4(X, Wu, EPS, "f32")["y"]
    h_ref = O.relu2_glu(g, u)
    pg, ag = pack(Wg, layout)
    pu, au = pack(Wu, layout)
    Xd = dev(X, BF16)
    r = B.bitlinear_a4_gate_up(Xd, pg, ag, pu, au, N, EPS, layout)
    assert np.array_equal(host(r["G"]), g) and np.array_equal(host(r["U"]), u)
    assert np.array_equal(host(r["H"]), h_ref)
    r = B.bitlinear_a4_gate_up(Xd, pg, ag, pu, au, N, EPS, layout, want=("H",))
    assert np.array_equal(host(r["H"]), h_ref)
    r = B.bitlinear_a4_gate_up(Xd, pg, ag, pu, au, N, EPS, layout, want=("G", "U"), gu_dtype=BF16)
    assert np.array_equal(host(r["G"]), O.bf16_round(g)) and np.array_equal(host(r["U"]), O.bf16_round(u))
    r = B.bitlinear_a4_gate_up(Xd, pg, ag, pu, au, N, EPS, layout, want=("U", "H"), gu_dtype=BF16)
    assert np.array_equal(host(r["U"]), O.bf16_round(u)) and np.array_equal(host(r["H"]), h_ref)


@pytest.mark.parametrize("kind,N,K,topk", [("heavy", 2050, 1500, 700), ("glu", 2048, 5460, 2730),
                                           ("glu", 4096, 8640, 4320), ("ties", 2064, 1000, 500),
                                           ("ties", 2048, 4096, 1), ("heavy", 300, 16384, 8192),
                                           ("ties", 2064, 9000, 3), ("glu", 16, 256, 100), ("heavy", 4096, 4096, 4096)])
def test_decode_fused_topk_int8(kind, N, K, topk):
    """One token with at least 128 output tiles: eq. 1 + eq. 3 run inside the GEMV launch, for every
    register-block count of the selection, ragged K and N, ties at the threshold."""
    say("decode fused topk %s N=%d K=%d topk=%d" % (kind, N, K, topk))
    W = S.latent_weights(N, K, S.seed_for(2, 601 + N))
    p, a = pack(W)
    for row in (0, 1, 2, 3):                              # "ties": all-zero row, all-equal row, -0.0 row
        X = _x(kind, 4, K, S.seed_for(2, 600 + K), BF16)[row:row + 1]
        ref = O.bitlinear_a8_sparse(X, W, topk, EPS, "f32")
        _check_linear(B.bitlinear_a8_sparse(dev(X, BF16), topk, p, a, N, EPS, B.BL_W_GEMM, F32, True), ref, F32)


@pytest.mark.parametrize("M,N,K,gdt", [(1, 11008, 4096, F32), (4, 11008, 4096, BF16), (2, 1000, 8192, F32),
                                       (3, 5460, 2048, F32), (1, 37, 256, BF16), (2, 2050, 1000, F32)])
def test_up_gated(M, N, K, gdt):
    """Gate-first up projection (decode): H = bf16(U * max(G, 0)^2) with the rows of the up weights
    read only where some token's gate is open, against the oracle's dense up projection followed
    by its ReLU^2 GLU (zeros compare equal whatever their sign)."""
    say("up gated M=%d N=%d K=%d %s" % (M, N, K, gdt))
    X = S.heavy(M, K, S.seed_for(2, 700 + M))
    Wg = S.latent_weights(N, K, S.seed_for(2, 701 + N))
    Wu = S.latent_weights(N, K, S.seed_for(2, 702 + K))
    g = O.bitlinear_a4(X, Wg, EPS, "f32" if gdt == F32 else "bf16")["y"]
    u = O.bitlinear_a4(X, Wu, EPS, "f32")["y"]
    h_ref = O.relu2_glu(g, u)
    pu, au = pack(Wu, B.BL_W_ROWS)
    G = dev(g, gdt)
    assert np.array_equal(host(G).astype(np.float32), g.astype(np.float32))
    Hh = B.bitlinear_a4_up_gated(dev(X, BF16), pu, au, N, G, EPS)
    assert np.array_equal(host(Hh), h_ref)
    closed = ~(g > 0).any(axis=0)
    assert closed.any() or N < 64                          # the case does skip rows
    assert not host(Hh)[:, closed].any()


def test_linears_seeded_shape_sweep():
    """16 seeded draws of (M, N, K) between 1 and ~700 / 900 / 3000: every linear on every weight
    layout it takes, accumulators bit-exact (all kernel choices by token count, ragged everything)."""
    rng = np.random.default_rng(S.seed_for(0, 777))
    for it in range(16):
        M = int(rng.choice([1, 2, 5, 16, 17, 40, 64, 65, int(rng.integers(66, 700))]))
        N = int(rng.integers(1, 900)) if it % 3 else int(rng.choice([2048, 2064, 4096]))
        K = int(rng.integers(1, 3000))
        topk = int(rng.integers(1, K + 1))
        say("shape sweep %d: M=%d N=%d K=%d topk=%d" % (it, M, N, K, topk))
        X = S.heavy(M, K, S.seed_for(0, 6000 + it))
        W = S.latent_weights(N, K, S.seed_for(0, 7000 + it))
        ref4 = O.bitlinear_a4(X, W, EPS, "bf16")
        ref8 = O.bitlinear_a8_sparse(X, W, topk, EPS, "bf16")
        Xd = dev(X, BF16)
        p, a = pack(W)
        _check_linear(B.bitlinear_a4(Xd, p, a, N, EPS, y_dtype=BF16, want_acc=True), ref4, BF16)
        _check_linear(B.bitlinear_a8_sparse(Xd, topk, p, a, N, EPS, B.BL_W_GEMM, BF16, True), ref8, BF16)
        for wl in (B.BL_W_MX4, B.BL_W_MX2):
            pm, am = pack(W, wl)
            _check_linear(B.bitlinear_a4(Xd, pm, am, N, EPS, y_dtype=BF16, want_acc=True, layout=wl), ref4, BF16)
        if M <= 8:
            pk, ak = pack(W, B.BL_W_KMAJOR)
            _check_linear(B.bitlinear_a8_sparse(Xd, topk, pk, ak, N, EPS, B.BL_W_KMAJOR, BF16, True), ref8, BF16)


def test_maximum_width():
    """The widest rows the library takes (BL_MAX_K channels): every quantizer and both INT4 GEMMs."""
    K = 32768                                              # BL_MAX_K of the public header
    say("maximum width K=%d" % K)
    M, N = 40, 48
    X = S.heavy(M, K, S.seed_for(0, 90))
    W = S.latent_weights(N, K, S.seed_for(0, 91))
    ref4 = O.bitlinear_a4(X, W, EPS, "f32")
    for layout in (B.BL_W_GEMM, B.BL_W_MX4, B.BL_W_MX2):
        p, a = pack(W, layout)
        _check_linear(B.bitlinear_a4(dev(X, BF16), p, a, N, EPS, y_dtype=F32, want_acc=True, layout=layout), ref4, F32)
    p, a = pack(W)
    ref8 = O.bitlinear_a8_sparse(X, W, K // 2, EPS, "f32")
    _check_linear(B.bitlinear_a8_sparse(dev(X, BF16), K // 2, p, a, N, EPS, B.BL_W_GEMM, F32, True), ref8, F32)
    codes_ref, e_ref = O.quant_fp4(X)
    r = B.quantize_act(dev(X, BF16), B.BL_ACT_FP4_E2M1_B32)
    assert np.array_equal(decode_fp4(host(r["q"]), M, K), codes_ref)


# ------------------------------------------------------------------ full prefill size (config 3), sampled rows
@pytest.mark.parametrize("M,N,K,dtype", [(16, 512, 256, F32), (300, 520, 1000, BF16), (130, 2048, 5460, BF16),
                                         (257, 5460, 2048, BF16), (1100, 1100, 768, BF16),
                                         (70, 1030, 300, BF16), (33, 257, 4096, F32), (600, 1500, 256, BF16)])
@pytest.mark.parametrize("wl", [B.BL_W_MX4, B.BL_W_MX2])
def test_a4_block_float_gemm(M, N, K, dtype, wl):
    """The INT4 linear on the 6-bit x 4-bit matrix instruction (BL_W_MX4 / BL_W_MX2 weights): accumulators
    bit-exact against the integer oracle, for several tiles, ragged M / N / K, every store path
    (N % 8 == 0, N % 4 == 0, odd N) and a single K block."""
    say("a4 block-float M=%d N=%d K=%d %s" % (M, N, K, dtype))
    X = S.heavy(M, K, S.seed_for(1, M + N))
    W = S.latent_weights(N, K, S.seed_for(1, K + N + 1))
    p, a = pack(W, wl)
    ref = O.bitlinear_a4(X, W, EPS, "bf16" if dtype == BF16 else "f32")
    _check_linear(B.bitlinear_a4(dev(X, BF16), p, a, N, EPS, y_dtype=dtype, want_acc=True, layout=wl),
                  ref, dtype)
    # the kernel variant without accumulator output (the one a caller normally runs)
    Y = B.bitlinear_a4(dev(X, BF16), p, a, N, EPS, y_dtype=dtype, layout=wl)
    assert np.array_equal(host(Y), ref["y"])


@pytest.mark.parametrize("name,N,K,kind", [("qkv", 12288, 4096, "a4"), ("o", 4096, 4096, "a8s"),
                                           ("gate", 11008, 4096, "a4"), ("down", 4096, 11008, "a8s")])
def test_config3_prefill_sampled_rows(name, N, K, kind):
    """M = 16384 in the launch configuration the benchmark times; the oracle checks 128 sampled
    token rows in full (all N, full K) plus every activation code of those rows."""
    say("config 3 prefill %s" % name)
    M = 16384
    T, alpha, packs = _decode_weights(name, N, K)
    p, a = packs[B.BL_W_GEMM]
    X = (S.glu_like(M, K, S.seed_for(3, 2)) if name == "down"
         else S.heavy(M, K, S.seed_for(3, 3 if name == "o" else 1)))
    rows = np.random.default_rng(S.seed_for(3, 9)).choice(M, 128, replace=False)
    rows[:2] = (0, M - 1)
    Xd = dev(X, BF16)
    if kind == "a4":
        Y, acc = B.bitlinear_a4(Xd, p, a, N, EPS, y_dtype=BF16, want_acc=True)
        q, d = O.quant_int4(X[rows], EPS)
        # and on the block-float path, in the launch configuration the benchmark times
        for wl in (B.BL_W_MX2, B.BL_W_MX4):
            pm, am = packs[wl]
            Ym = B.bitlinear_a4(Xd, pm, am, N, EPS, y_dtype=BF16, layout=wl)
            assert torch.equal(Ym, Y)
    else:
        Y, acc = B.bitlinear_a8_sparse(Xd, K // 2, p, a, N, EPS, B.BL_W_GEMM, BF16, True)
        q, d, _ = O.quant_topk_int8(X[rows], K // 2, EPS)
    acc_ref = O.matmul_int(q, T)
    idx = torch.from_numpy(rows).cuda()
    assert np.array_equal(host(acc[idx]), acc_ref)
    y_ref = O.rescale(acc_ref, d, alpha, "bf16")
    assert_close_rel(host(Y[idx]), y_ref)
    assert np.array_equal(host(Y[idx]), y_ref)


def test_config3_gate_up_glu_sampled_rows():
    """The FFN's gate and up projection as one GEMM with eq. 5 in its epilogue, at M = 16384 in the launch
    configuration the benchmark times: H on 128 sampled token rows against the oracle's two linears and
    its GLU, bit for bit."""
    say("config 3 gate/up GEMM with the GLU epilogue")
    M, N, K = 16384, 11008, 4096
    Tg, ag_ref, packs_g = _decode_weights("gate", N, K)
    Tu, au_ref, packs_u = _decode_weights("up", N, K)
    X = S.heavy(M, K, S.seed_for(3, 1))
    rows = np.random.default_rng(S.seed_for(3, 9)).choice(M, 128, replace=False)
    rows[:2] = (0, M - 1)
    q, d = O.quant_int4(X[rows], EPS)
    g = O.rescale(O.matmul_int(q, Tg), d, ag_ref, "f32")
    u = O.rescale(O.matmul_int(q, Tu), d, au_ref, "f32")
    h_ref = O.relu2_glu(g, u)
    pg, ag = packs_g[B.BL_W_MX2]
    pu, au = packs_u[B.BL_W_MX2]
    r = B.bitlinear_a4_gate_up(dev(X, BF16), pg, ag, pu, au, N, EPS, B.BL_W_MX2, want=("H",))
    assert np.array_equal(host(r["H"][torch.from_numpy(rows).cuda()]), h_ref)


@pytest.mark.parametrize("name,N,K,kind", [("qkv", 12288, 4096, "a4"), ("down", 4096, 11008, "a8s")])
def test_config3_full_size_properties(name, N, K, kind):
    """M = 16384 in the benchmark's launch configuration, every output checked through properties the
    equations imply at any size: a permutation of the tokens permutes the output rows bit for bit
    (every row meets every tile position), and a power-of-two gain on the input with eps = 0 comes
    out as the same gain on the output, exactly."""
    say("config 3 full-size properties %s" % name)
    M = 16384
    T, alpha, packs = _decode_weights(name, N, K)
    wl = B.BL_W_MX2 if kind == "a4" else B.BL_W_GEMM
    p, a = packs[wl]
    X = S.heavy(M, K, S.seed_for(3, 1)) if kind == "a4" else S.glu_like(M, K, S.seed_for(3, 2))
    Xd = dev(X, BF16)

    def run(x, eps):
        if kind == "a4":
            return B.bitlinear_a4(x, p, a, N, eps, y_dtype=BF16, layout=wl)
        return B.bitlinear_a8_sparse(x, K // 2, p, a, N, eps, wl, BF16, False)

    Y = run(Xd, EPS)
    perm = torch.from_numpy(np.random.default_rng(S.seed_for(3, 11)).permutation(M)).cuda()
    Yp = run(Xd[perm].contiguous(), EPS)
    assert torch.equal(Yp, Y[perm])
    del Yp
    Y0 = run(Xd, 0.0)
    Y4 = run((Xd.float() * 4.0).to(torch.bfloat16), 0.0)
    assert torch.equal(Y4.float(), Y0.float() * 4.0)
    assert torch.isfinite(Y0.float()).all() and float(Y0.float().abs().max()) > 0


# ------------------------------------------------------------------ error paths (no kernel runs)
def test_argument_errors():
    say("argument errors")
    X = dev(np.zeros((4, 64), np.float32))
    p, a = pack(S.latent_weights(32, 64, 1))
    with pytest.raises(B.BitlinearError) as e:
        B.bitlinear_a8_sparse(X, 0, p, a, 32)
    assert e.value.status == -1
    with pytest.raises(B.BitlinearError) as e:
        B.bitlinear_a8_sparse(X, 65, p, a, 32)
    assert e.value.status == -1
    with pytest.raises(B.BitlinearError) as e:
        B.bitlinear_a4(X, p, a, 32, ws=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -4
    with pytest.raises(B.BitlinearError) as e:
        Xu = torch.zeros(4 * 64 + 4, device="cuda")[1:257].view(4, 64)      # 4-byte offset
        B.bitlinear_a4(Xu, p, a, 32)
    assert e.value.status == -3
    Hd = dev(np.zeros((2, 3, 64), np.float32))
    with pytest.raises(B.BitlinearError) as e:
        B.quantize_heads(Hd, 5)                                             # 3 or 4 bits only
    assert e.value.status == -1
    L = B.lib()
    qb = torch.empty(64, dtype=torch.uint8, device="cuda")
    sb = torch.empty(8, dtype=torch.float32, device="cuda")
    assert L.quantize_heads(Hd.data_ptr(), B.BL_F32, 2, 3, 12, 4, 1e-5, qb.data_ptr(), sb.data_ptr(), None) == -2   # D % 8
    assert L.quantize_heads_bytes(4, 2, 3, 12) == 0 and L.quantize_heads_bytes(3, 2, 3, 64) == 2 * 3 * 24


# ------------------------------------------------------------------ FP4 variant (config 4)
# Float32 accumulation of at most 32768 exact products in an order the matrix instruction does not
# define: each addition errs by at most 2^-24 of the running sum, and on outputs above the median
# magnitude the sum of |terms| is a few hundred times |y| at most; measured below 1e-6.  bfloat16
# outputs add half an ulp, up to 2^-8 of the value.
FP4_REL_F32 = 1e-4
FP4_REL_BF16 = 2.0 ** -8 + 1e-4


def _check_fp4(Y, ref, rows=None):
    """FP4 path: float32 accumulation inside the matrix instruction, so tolerance only:
    1e-3 of the sum of |terms| of each output (plus bf16 rounding when the output is bf16)."""
    y = host(Y).astype(np.float64)
    deq = np.abs(O.fp4_dequant(ref["codes"], ref["e"]))
    bound = 1e-3 * float(ref["alpha"]) * (deq @ np.abs(ref["T"]).astype(np.float64).T)
    if Y.dtype == BF16:
        bound = bound + np.abs(ref["y"]) * 2.0 ** -8
    err = np.abs(y - ref["y"])
    assert np.all(err <= bound + 1e-30), "max err/bound %g" % (err / (bound + 1e-30)).max()
    # achieved accuracy where the result is not a near-cancellation: outputs above the median magnitude
    big = np.abs(ref["y"]) > np.median(np.abs(ref["y"]))
    rel = float((err[big] / np.abs(ref["y"][big])).max()) if big.any() else 0.0
    say("fp4 max relative error on outputs above the median magnitude: %.3g (%s output)"
        % (rel, "bf16" if Y.dtype == BF16 else "f32"))
    assert rel <= (FP4_REL_BF16 if Y.dtype == BF16 else FP4_REL_F32)
    return rel


@pytest.mark.parametrize("layout", [B.BL_W_GEMM, B.BL_W_MX4, B.BL_W_MX2])
@pytest.mark.parametrize("M,N,K,dtype", [(16, 512, 256, F32), (130, 200, 992, BF16), (300, 1100, 3200, BF16),
                                         (257, 1030, 288, BF16), (600, 257, 1504, BF16)])
def test_fp4_linear(M, N, K, dtype, layout):
    """Both FP4 GEMMs: 2-bit weights on the 16x16x128 instruction, and E2M1 weights in LDS tile
    order on the 32x32x64 instruction (the prefill kernel; ragged M / N / K, every store path)."""
    say("fp4 linear M=%d N=%d K=%d layout=%d" % (M, N, K, layout))
    X = S.heavy(M, K, S.seed_for(4, M + N)) if dtype == BF16 else S.gauss_outlier(M, K, 4, 20.0, S.seed_for(4, M))
    W = S.latent_weights(N, K, S.seed_for(4, N + K))
    ref = O.bitlinear_fp4(X, W, EPS)
    p, a = pack(W, layout)
    for ydt in (F32, BF16):
        Y = B.bitlinear_a4(dev(X, dtype), p, a, N, EPS, act_fp4=True, y_dtype=ydt, layout=layout)
        _check_fp4(Y, ref)
    # an exactly representable case must be exact: integers up to 6 times ternary weights
    Xi = np.random.default_rng(5).integers(-6, 7, (M, K)).astype(np.float32)
    Xi[np.abs(Xi) == 5] = 4
    Xi[:, ::32] = 6                                         # every block has scale 2^0
    refi = O.bitlinear_fp4(Xi, W, EPS)
    Yi = B.bitlinear_a4(dev(Xi, dtype), p, a, N, EPS, act_fp4=True, y_dtype=F32, layout=layout)
    acc_exact = refi["y"] / np.float64(refi["alpha"])       # integers
    assert np.array_equal(host(Yi), (acc_exact.astype(np.float32) * refi["alpha"]).astype(np.float32))


@pytest.mark.parametrize("name,N,K", [("qkv", 9600, 3200), ("o", 3200, 3200), ("gate", 8640, 3200)])
def test_config4_fp4_sampled_rows(name, N, K):
    """3B-like FP4 variant at M = 8192, 64 sampled token rows against the float64 oracle."""
    say("config 4 fp4 %s" % name)
    M = 8192
    X = S.heavy(M, K, S.seed_for(4, 1))
    W = S.latent_weights(N, K, S.seed_for(4, 2 + len(name)))
    p, a = pack(W)
    rows = np.random.default_rng(S.seed_for(4, 9)).choice(M, 64, replace=False)
    rows[:2] = (0, M - 1)
    Y = B.bitlinear_a4(dev(X, BF16), p, a, N, EPS, act_fp4=True, y_dtype=F32)
    ref = O.bitlinear_fp4(X[rows], W, EPS)
    _check_fp4(Y[torch.from_numpy(rows).cuda()], ref)
    # and on the prefill kernel (E2M1 weights in LDS tile order), in the launch configuration the
    # FP4 / INT4 comparison is timed in
    pm, am = pack(W, B.BL_W_MX2)
    Ym = B.bitlinear_a4(dev(X, BF16), pm, am, N, EPS, act_fp4=True, y_dtype=F32, layout=B.BL_W_MX2)
    _check_fp4(Ym[torch.from_numpy(rows).cuda()], ref)
    # the INT4 path on identical inputs (the comparison the paper makes): both are reported
    # against the product of the raw activations with the same ternary weights; with
    # heavy-tailed outlier channels the FP4 grid, which never clips, must be the closer one
    Yi = host(B.bitlinear_a4(dev(X, BF16), p, a, N, EPS, y_dtype=F32)[torch.from_numpy(rows).cuda()])
    full = X[rows].astype(np.float64) @ (ref["T"].astype(np.float64) * np.float64(ref["alpha"])).T
    rel_fp4 = np.linalg.norm(host(Y[torch.from_numpy(rows).cuda()]) - full) / np.linalg.norm(full)
    rel_int4 = np.linalg.norm(Yi - full) / np.linalg.norm(full)
    say("relative error vs unquantized activations: fp4 %.4f, int4 %.4f" % (rel_fp4, rel_int4))
    assert rel_fp4 < rel_int4 and rel_fp4 < 0.2


def test_config4_down_int8_sampled_rows():
    """The down projection of the 3B-like variant stays on top-50 % + INT8 (config 4): 8640 -> 3200 at
    M = 8192, 64 sampled token rows against the integer oracle, bit for bit."""
    say("config 4 down (top-4320 + INT8)")
    M, N, K = 8192, 3200, 8640
    X = S.glu_like(M, K, S.seed_for(4, 31))
    W = S.latent_weights(N, K, S.seed_for(4, 32))
    T, alpha = O.ternarize(W, EPS)
    p, a = pack(W)
    rows = np.random.default_rng(S.seed_for(4, 33)).choice(M, 64, replace=False)
    rows[:2] = (0, M - 1)
    Y, acc = B.bitlinear_a8_sparse(dev(X, BF16), K // 2, p, a, N, EPS, B.BL_W_GEMM, BF16, True)
    q, d, _ = O.quant_topk_int8(X[rows], K // 2, EPS)
    acc_ref = O.matmul_int(q, T)
    idx = torch.from_numpy(rows).cuda()
    assert np.array_equal(host(acc[idx]), acc_ref)
    y_ref = O.rescale(acc_ref, d, alpha, "bf16")
    assert_close_rel(host(Y[idx]), y_ref)
    assert np.array_equal(host(Y[idx]), y_ref)


# ------------------------------------------------------------------ straight-through backward (Section 2.2)
def _ste_bounds(dYh, q, d, T, alpha, M, N):
    """Per-element error bounds of the bfloat16 / float32-accumulate gradient GEMMs against the exact
    sums: float32 accumulation of J terms in any order is within (J + 2) 2^-24 of the sum of the terms'
    magnitudes; dW's left operand bf16(dY d_m) carries one more relative 2^-8 per term (bfloat16's unit roundoff)."""
    absY = np.abs(dYh)
    sx = np.float64(alpha) * (absY @ np.abs(T).astype(np.float64))
    sw = absY.T @ (np.abs(q).astype(np.float64) * d.astype(np.float64)[:, None])
    Mc = (M + 63) // 64 * 64
    return (N + 2) * 2.0 ** -24 * sx, (2.0 ** -8 + (Mc + 3) * 2.0 ** -24) * sw


@pytest.mark.parametrize("M,N,K,kind", [(200, 264, 392, "a4"), (130, 72, 520, "a8"), (64, 128, 256, "a4"),
                                        (1, 8, 8, "a8"), (300, 1032, 136, "a8"), (257, 520, 1000, "a4"),
                                        (100, 5460, 2048, "a4"), (96, 2048, 5460, "a8"), (70, 100, 1000, "a8"),
                                        (33, 52, 300, "a4"), (5, 3, 20, "a8")])
def test_ste_backward(M, N, K, kind):
    """dX = dY . Q_w(W) and dW = dY^T . Q(X) (the quantizers and Top_k passed over) against the oracle's
    float64 sums, element by element, within the bounds the arithmetic gives; several tiles, ragged edges."""
    say("ste backward M=%d N=%d K=%d %s" % (M, N, K, kind))
    X = S.heavy(M, K, S.seed_for(5, 10 + M))
    W = S.latent_weights(N, K, S.seed_for(5, 11 + N))
    rng = np.random.default_rng(S.seed_for(5, 12 + K))
    dYh = S.snap_bf16((rng.standard_normal((M, N)) * 0.01).astype(np.float32))
    if kind == "a4":
        lay = O.bitlinear_a4(X, W, EPS)
        mode, topk = B.BL_ACT_INT4_ABSMEAN, 0
    else:
        lay = O.bitlinear_a8_sparse(X, W, max(1, K // 2), EPS)
        mode, topk = B.BL_ACT_TOPK_INT8_ABSMAX, max(1, K // 2)
    dX_ref, dW_ref = O.ste_backward(dYh, lay["q"], lay["d"], lay["T"], lay["alpha"])
    bx, bw = _ste_bounds(dYh.astype(np.float64), lay["q"], lay["d"], lay["T"], lay["alpha"], M, N)
    pk, ak = pack(W, B.BL_W_KMAJOR)
    qa = B.quantize_act(dev(X, BF16), mode, topk, EPS)
    dY = dev(dYh, BF16)
    dX, dW = B.bitlinear_backward(dY, qa["q"], qa["scale"], mode, K, pk, ak, dx_dtype=F32)
    ex = np.abs(host(dX).astype(np.float64) - dX_ref)
    ew = np.abs(host(dW).astype(np.float64) - dW_ref)
    assert np.all(ex <= bx + 1e-30), float((ex / (bx + 1e-30)).max())
    assert np.all(ew <= bw + 1e-30), float((ew / (bw + 1e-30)).max())
    # the sums are not trivially small against their bounds: the check would catch a dropped tile
    assert np.abs(dX_ref).max() > 20 * bx.max() and np.abs(dW_ref).max() > 5 * bw.max()
    # bfloat16 dX: one more rounding; dX alone and dW alone
    dXb, none = B.bitlinear_backward(dY, qa["q"], qa["scale"], mode, K, pk, ak, want_dw=False, dx_dtype=BF16)
    assert none is None
    eb = np.abs(host(dXb).astype(np.float64) - dX_ref)
    assert np.all(eb <= bx + 2.0 ** -8 * np.abs(dX_ref) + 1e-30)
    none, dW2 = B.bitlinear_backward(dY, qa["q"], qa["scale"], mode, K, pk, ak, want_dx=False)
    assert none is None and np.array_equal(host(dW2), host(dW))
    # masked channels still receive a gradient (the estimator passes over Top_k)
    if kind == "a8" and K >= 8:
        assert np.abs(host(dX)[~lay["mask"]]).max() > 0


def test_ste_backward_rejects():
    """Shapes and layouts the backward entry point does not take are refused before any launch."""
    L = B.lib()
    z = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    p = z.data_ptr()
    assert L.bitlinear_backward(p, 4, 8, 8, p, p, 0, p, B.BL_W_GEMM, p, p, 0, None, p, 1 << 16, None) == -6      # layout
    assert L.bitlinear_backward(p, 4, 8, 8, p, p, 2, p, B.BL_W_KMAJOR, p, p, 0, None, p, 1 << 16, None) == -6    # FP4 codes
    assert L.bitlinear_backward(p, 4, 8, 8, p, p, 0, p, B.BL_W_KMAJOR, p, None, 0, None, p, 1 << 16, None) == -1  # no output
    assert L.bitlinear_backward(p, 4, 8, 8, p, p, 0, p, B.BL_W_KMAJOR, p, p, 0, None, p, 16, None) == -4         # workspace


def test_ste_backward_7b_sampled_rows():
    """The qkv projection's backward at 7B width on 2048 tokens: sampled rows of dX and of dW against the
    oracle's float64 sums (the oracle computes each sampled row on its own)."""
    M, N, K = 2048, 12288, 4096
    say("ste backward 7B qkv, M=%d" % M)
    X = S.heavy(M, K, S.seed_for(5, 100))
    W = S.latent_weights(N, K, S.seed_for(5, 101))
    rng = np.random.default_rng(S.seed_for(5, 102))
    dYh = S.snap_bf16((rng.standard_normal((M, N)) * 0.01).astype(np.float32))
    T, alpha = O.ternarize(W, EPS)
    q, d = O.quant_int4(X, EPS)
    pk, ak = pack(W, B.BL_W_KMAJOR)
    qa = B.quantize_act(dev(X, BF16), B.BL_ACT_INT4_ABSMEAN, 0, EPS)
    dX, dW = B.bitlinear_backward(dev(dYh, BF16), qa["q"], qa["scale"], B.BL_ACT_INT4_ABSMEAN, K, pk, ak, dx_dtype=F32)
    dXh, dWh = host(dX).astype(np.float64), host(dW).astype(np.float64)
    dY64 = dYh.astype(np.float64)
    rows_m = rng.choice(M, 24, replace=False)
    ref, _ = O.ste_backward(dY64[rows_m], q[rows_m], d[rows_m], T, alpha)
    bx = (N + 2) * 2.0 ** -24 * np.float64(alpha) * (np.abs(dY64[rows_m]) @ np.abs(T).astype(np.float64))
    assert np.all(np.abs(dXh[rows_m] - ref) <= bx)
    rows_n = rng.choice(N, 24, replace=False)
    _, refw = O.ste_backward(dY64[:, rows_n], q, d, T[rows_n], alpha)
    bw = (2.0 ** -8 + (M + 3) * 2.0 ** -24) * (np.abs(dY64[:, rows_n]).T @ (np.abs(q).astype(np.float64) * d.astype(np.float64)[:, None]))
    assert np.all(np.abs(dWh[rows_n] - refw) <= bw)
    assert np.abs(ref).max() > 20 * bx.max() and np.abs(refw).max() > 5 * bw.max()
