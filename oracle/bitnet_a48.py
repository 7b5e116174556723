"""CPU oracle for the quantized linear layers of BitNet a4.8 (arXiv 2411.04965).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
kernels are checked against.  It must never be imported by the product package;
only tests, the smoke check and the benchmark's CPU-baseline leg may call it.
It shares no code with the HIP path.

Every function writes out one equation of the paper, in the paper's notation:

    X  activations [M, K] (one token per row),  W latent weights [N, K],
    Y = Q(X) . Q_w(W)^T  [M, N]                               (eq. 1 and eq. 6)

Arithmetic conventions (the paper fixes none of them; these are the readings
this build takes, each one listed in the design notes):

  * statistics (mean |.|, max |.|) are per token for activations and per matrix
    for weights;
  * a mean is the float64 sum divided in float64, rounded once to float32;
  * every other floating-point step is one IEEE float32 operation, never fused;
  * round() is round-half-to-even;
  * activations are multiplied by a precomputed scale c/(stat+eps), weights are
    divided by (alpha+eps), as the equations are printed;
  * Top_k keeps exactly k entries per token, ties go to the lower index.

Parity pins: every function here is pinned by tests/test_oracle_*.py against
hand-worked vectors, closed forms, brute force and invariants.  Nothing in
this file is "parity unpinned".
"""
import numpy as np

F32 = np.float32
SQRT7 = F32(np.sqrt(7.0))  # 0x402953FD
C127 = F32(127.0)
DEFAULT_EPS = 1e-5


# --------------------------------------------------------------------------
# small helpers
# --------------------------------------------------------------------------
def round_clip(x, a, b):
    """RoundClip(X, a, b) = min(max(round(X), a), b)   (eq. 4)."""
    return np.minimum(np.maximum(np.rint(x), a), b)


def bf16_round(x):
    """Round float32 values to the nearest bfloat16 (ties to even); float32 out."""
    u = np.ascontiguousarray(x, dtype=F32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(F32)


def _mean_abs_f32(x, axis=None):
    """mean(|x|): float64 sum, float64 divide, one rounding to float32."""
    a = np.abs(np.asarray(x, dtype=F32)).astype(np.float64)
    n = a.size if axis is None else a.shape[axis]
    return (a.sum(axis=axis) / np.float64(n)).astype(F32)


# --------------------------------------------------------------------------
# weights (eq. 2)
# --------------------------------------------------------------------------
def ternarize(W, eps=DEFAULT_EPS):
    """Q_w(W) = alpha * RoundClip(W / (alpha + eps), -1, 1), alpha = mean|W|  (eq. 2).

    Returns (T int8 [N, K] in {-1, 0, 1}, alpha float32 scalar)."""
    W = np.asarray(W, dtype=F32)
    alpha = _mean_abs_f32(W)
    t = F32(alpha + F32(eps))
    T = round_clip(W / t, -1, 1).astype(np.int8)
    return T, F32(alpha)


# --------------------------------------------------------------------------
# activations
# --------------------------------------------------------------------------
def quant_int4(X, eps=DEFAULT_EPS):
    """Q_INT4(X) = beta/sqrt7 * RoundClip(sqrt7/(beta+eps) * X, -8, 7), beta = mean|X|  (eq. 7).

    Per token.  Returns (q int8 [M, K] in [-8, 7], d float32 [M] = beta/sqrt7)."""
    X = np.asarray(X, dtype=F32)
    beta = _mean_abs_f32(X, axis=1)                       # [M]
    s = (SQRT7 / (beta + F32(eps)).astype(F32)).astype(F32)
    q = round_clip((X * s[:, None]).astype(F32), -8, 7).astype(np.int8)
    d = (beta / SQRT7).astype(F32)
    return q, d


def quant_int4_variant(X, eps=DEFAULT_EPS, kind="absmean2"):
    """The two other INT4 quantizers of the ablations (Section 4.3), per token.

    "absmean2": eq. 7 with beta = 2 mean|X| (used there for the inputs to the down projection);
    "absmax":   the absmax form of eq. 3 at 4 bits, gamma/7 * RoundClip(7/(gamma+eps) * X, -8, 7),
                gamma = max|X| (the paper names the quantizer without printing it).
    Returns (q int8 [M, K] in [-8, 7], d float32 [M] = the dequantization scale)."""
    X = np.asarray(X, dtype=F32)
    if kind == "absmean2":
        beta = (F32(2) * _mean_abs_f32(X, axis=1)).astype(F32)
        s = (SQRT7 / (beta + F32(eps)).astype(F32)).astype(F32)
        d = (beta / SQRT7).astype(F32)
    elif kind == "absmax":
        gamma = np.max(np.abs(X), axis=1).astype(F32)
        s = (F32(7) / (gamma + F32(eps)).astype(F32)).astype(F32)
        d = (gamma / F32(7)).astype(F32)
    else:
        raise ValueError(kind)
    q = round_clip((X * s[:, None]).astype(F32), -8, 7).astype(np.int8)
    return q, d


def topk_mask(X, k_sel):
    """M = Top_k(|X|) per token  (eq. 1): exactly k_sel ones per row.

    Magnitudes are compared as float32 values (so -0 equals +0); among equal
    magnitudes the lower channel index wins."""
    X = np.asarray(X, dtype=F32)
    M_, K = X.shape
    assert 1 <= k_sel <= K
    key = np.abs(X).view(np.uint32).astype(np.int64)      # order-preserving for finite |x|
    order = np.argsort(-key, axis=1, kind="stable")       # descending, stable -> lower index first
    mask = np.zeros((M_, K), dtype=bool)
    np.put_along_axis(mask, order[:, :k_sel], True, axis=1)
    return mask


def quant_int8(X, eps=DEFAULT_EPS):
    """Q_INT8(X) = gamma/127 * RoundClip(127/(gamma+eps) * X, -128, 127), gamma = max|X|  (eq. 3).

    Per token.  Returns (q int8 [M, K], d float32 [M] = gamma/127)."""
    X = np.asarray(X, dtype=F32)
    gamma = np.abs(X).max(axis=1).astype(F32)
    s = (C127 / (gamma + F32(eps)).astype(F32)).astype(F32)
    q = round_clip((X * s[:, None]).astype(F32), -128, 127).astype(np.int8)
    d = (gamma / C127).astype(F32)
    return q, d


def quant_topk_int8(X, k_sel, eps=DEFAULT_EPS):
    """Q_INT8(X) (.) M with M = Top_k(|X|)  (eq. 1, eq. 3).

    Returns (q int8 [M, K] with zeros outside the mask, d float32 [M], mask bool [M, K])."""
    q, d = quant_int8(X, eps)
    mask = topk_mask(X, k_sel)
    return np.where(mask, q, np.int8(0)).astype(np.int8), d, mask


def quant_heads(X, bits, eps=DEFAULT_EPS):
    """Low-bit attention states (Section 4.2, "Low-bit Attention"; Table 3): every head vector of a
    token (post-RoPE query, key or value) is quantized on its own with the absmax function, to
    `bits` = 4 or 3 bits, and stored as an unsigned integer.

    Reading (the paper gives one sentence and no formula): the absmax form of eq. 3 with
    Q_b = 2^(bits-1) - 1 levels on each side,
        q = RoundClip(Q_b / (gamma + eps) * x, -Q_b, Q_b),  gamma = max|x| over the head,
    stored with the offset 2^(bits-1):  code = q + 2^(bits-1), in [1, 2^bits - 1];
    the value it stands for is (code - 2^(bits-1)) * gamma / Q_b.  (Which tokens get which width -
    the paper keeps the first token's heads at 4 bits in the 3-bit cache - is the caller's choice.)

    X [T, H, D] -> (codes uint8 [T, H, D], d float32 [T, H] = gamma / Q_b)."""
    assert bits in (3, 4)
    X = np.asarray(X, dtype=F32)
    Qb = F32(2 ** (bits - 1) - 1)
    gamma = np.abs(X).max(axis=2).astype(F32)
    s = (Qb / (gamma + F32(eps)).astype(F32)).astype(F32)
    q = round_clip((X * s[:, :, None]).astype(F32), -float(Qb), float(Qb)).astype(np.int16)
    codes = (q + 2 ** (bits - 1)).astype(np.uint8)
    d = (gamma / Qb).astype(F32)
    return codes, d


def dequant_heads(codes, d, bits):
    """Value a low-bit attention code stands for (Section 4.2; the reading of quant_heads):
    (code - 2^(bits-1)) * d, one float32 multiply.  codes uint8 [T, H, D], d float32 [T, H]."""
    assert bits in (3, 4)
    q = codes.astype(np.int16) - 2 ** (bits - 1)
    return (q.astype(F32) * np.asarray(d, dtype=F32)[:, :, None]).astype(F32)


def _pack_bits_le(codes, bits):
    """One head's codes -> bytes of its little-endian bit stream (code j in bits bits*j ...)."""
    acc = 0
    for j, c in enumerate(int(v) for v in codes):
        acc |= c << (bits * j)
    n = (len(codes) * bits + 7) // 8
    return [(acc >> (8 * i)) & 255 for i in range(n)]


def kv_cache_pack(X, eps=DEFAULT_EPS):
    """The 3-bit key / value cache of Table 3 ("4-bit Q, 3-bit KV": "the heads of the bos token"
    stay at 4 bits, Section 4.2): token 0 of the sequence is quantized per head to 4 bits, every later
    token to 3 bits, all with quant_heads.  Byte layout (this build's; the paper defines none):
    token 0 takes H * D / 2 bytes, every later token H * 3 D / 8 bytes, tokens in order, heads in
    order inside a token, a head's codes as a little-endian bit stream (code j in bits bits*j ...).

    X [T, H, D] (D % 8 == 0) -> (bytes uint8 [H*D/2 + (T-1)*H*3D/8], d float32 [T, H])."""
    X = np.asarray(X, dtype=F32)
    T, H, D = X.shape
    assert D % 8 == 0
    out = []
    d = np.zeros((T, H), dtype=F32)
    for t in range(T):
        bits = 4 if t == 0 else 3
        c, dt = quant_heads(X[t:t + 1], bits, eps)
        d[t] = dt[0]
        for h in range(H):
            out.extend(_pack_bits_le(c[0, h], bits))
    return np.array(out, dtype=np.uint8), d


def kv_cache_unpack(raw, d, T, H, D):
    """Inverse of kv_cache_pack's layout followed by dequant_heads: float32 values [T, H, D]."""
    raw = [int(v) for v in np.asarray(raw, dtype=np.uint8)]
    out = np.zeros((T, H, D), dtype=F32)
    pos = 0
    for t in range(T):
        bits = 4 if t == 0 else 3
        nb = D * bits // 8
        codes = np.zeros((1, H, D), dtype=np.uint8)
        for h in range(H):
            acc = 0
            for i in range(nb):
                acc |= raw[pos + i] << (8 * i)
            pos += nb
            for j in range(D):
                codes[0, h, j] = (acc >> (bits * j)) & (2 ** bits - 1)
        out[t] = dequant_heads(codes, d[t:t + 1], bits)[0]
    return out


# E2M1 magnitudes by 3-bit code (1 sign, 2 exponent, 1 mantissa bit).
E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float64)
FP4_BLOCK = 32


E1M2_GRID = np.arange(8, dtype=np.float64) / 4.0           # 0, 0.25, ..., 1.75


def quant_fp4(X, fmt="e2m1"):
    """FP4 MinMax quantizer (eq. 8-9) with one power-of-two scale per block of
    32 consecutive channels of a token.  fmt = "e2m1" (E = 2, M = 1, the format
    the paper adopts) or "e1m2" (E = 1, M = 2, the other arm of Section 4.3's
    4-bit comparison).

    Reading of eq. 8-9 for power-of-two scales: the bias b is an integer per
    block, chosen as the largest one for which the block maximum does not clip,
    i.e. the scale 2^e is the smallest power of two with max|x| / 2^e <= top,
    top = (2 - 2^-M) 2^(2^E - 2) = 6 for E2M1 and 1.75 for E1M2 (exponent bias 1
    in both).  Within a block every value is rounded to the nearest value of the
    format (ties to the even code).  A value that rounds to zero is stored as +0.
    E1M2's values are the uniform grid j / 4, j = 0..7 (one subnormal and one
    normal binade).

    Returns (codes uint8 [M, K] = sign<<3 | code3,  e int16 [M, K/32] block exponents;
    the E8M0 scale byte is e + 127)."""
    assert fmt in ("e2m1", "e1m2")
    X = np.asarray(X, dtype=F32)
    M_, K = X.shape
    assert K % FP4_BLOCK == 0
    xb = X.reshape(M_, K // FP4_BLOCK, FP4_BLOCK).astype(np.float64)
    a = np.abs(xb).max(axis=2)                             # [M, K/32]
    mant, ex = np.frexp(a)                                 # a = mant * 2^ex, mant in [0.5, 1)
    if fmt == "e2m1":
        # a = (2 mant) * 2^(ex-1);  smallest e with a / 2^e <= 6 = 1.5 * 2^2
        e = np.where(2.0 * mant <= 1.5, ex - 1 - 2, ex - 1 - 1)
    else:
        # smallest e with a / 2^e <= 1.75 = 1.75 * 2^0
        e = np.where(2.0 * mant <= 1.75, ex - 1, ex)
    e = np.where(a == 0.0, 0, e)
    e = np.clip(e, -127, 127).astype(np.int64)
    v = np.ldexp(xb, -e[:, :, None])                       # exact
    av = np.abs(v)
    if fmt == "e2m1":
        grid = E2M1_GRID
        step = np.where(av < 2.0, 0.5, np.where(av < 4.0, 1.0, 2.0))
        r = np.minimum(np.rint(av / step) * step, 6.0)     # RNE on the local step == ties to even code
    else:
        grid = E1M2_GRID
        r = np.minimum(np.rint(av * 4.0) / 4.0, 1.75)      # one step everywhere
    code3 = np.searchsorted(grid, r).astype(np.uint8)
    assert np.all(grid[code3] == r)
    sign = ((v < 0) & (code3 != 0)).astype(np.uint8)
    codes = (sign << 3 | code3).reshape(M_, K)
    return codes, e.astype(np.int16)


def fp4_dequant(codes, e, fmt="e2m1"):
    """float64 values encoded by quant_fp4's output."""
    M_, K = codes.shape
    mag = (E2M1_GRID if fmt == "e2m1" else E1M2_GRID)[codes & 7]
    val = np.where(codes & 8, -mag, mag).reshape(M_, K // FP4_BLOCK, FP4_BLOCK)
    return np.ldexp(val, e.astype(np.int64)[:, :, None]).reshape(M_, K)


# --------------------------------------------------------------------------
# matmul and rescale
# --------------------------------------------------------------------------
def matmul_int(q, T):
    """acc[m, n] = sum_k q[m, k] * T[n, k], exact integers (int32).

    Evaluated as a float64 matrix product: every partial sum is an integer far
    below 2^53, so the result is exact whatever the summation order."""
    acc = q.astype(np.float64) @ T.astype(np.float64).T
    out = acc.astype(np.int64)
    assert np.all(out == acc) and np.abs(out).max(initial=0) < 2 ** 31
    return out.astype(np.int32)


def rescale(acc, d, alpha, out_dtype="f32"):
    """y = (float(acc) * d_m) * alpha, two float32 multiplies in this order;
    then an optional rounding to bfloat16 (returned as float32 values)."""
    y = (acc.astype(F32) * np.asarray(d, dtype=F32)[:, None]).astype(F32)
    y = (y * F32(alpha)).astype(F32)
    if out_dtype == "bf16":
        y = bf16_round(y)
    return y


def relu2_glu(g, u):
    """ReLU^2 GLU combine  h = u (.) ReLU(g)^2  (eq. 5), float32 steps, bf16 result."""
    g = np.asarray(g, dtype=F32)
    u = np.asarray(u, dtype=F32)
    r = np.maximum(g, F32(0))
    rr = (r * r).astype(F32)
    return bf16_round((u * rr).astype(F32))


def swish_glu(g, u):
    """Swish GLU combine  h = u (.) g sigmoid(g), the activation Section 4.3
    compares squared ReLU with.  Evaluated in float64 from the float32 inputs
    and rounded once, from float64, to bfloat16 (returned as float32 values): the
    definition itself, so a float32 implementation may differ from it by one bfloat16 ulp
    where its few-ulp float32 error straddles a rounding boundary."""
    g = np.asarray(g, dtype=F32).astype(np.float64)
    u = np.asarray(u, dtype=F32).astype(np.float64)
    with np.errstate(over="ignore"):
        h = u * (g / (1.0 + np.exp(-g)))
    # nearest bfloat16 of the float64 value, ties to even: a power-of-two ulp makes h / ulp exact
    _, ex = np.frexp(h)                                    # |h| in [2^(ex-1), 2^ex)
    ulp = np.ldexp(1.0, np.maximum(ex - 1, -126) - 7)
    return (np.rint(h / ulp) * ulp).astype(F32)


# --------------------------------------------------------------------------
# the linear layers
# --------------------------------------------------------------------------
def bitlinear_a4(X, W, eps=DEFAULT_EPS, out_dtype="f32"):
    """Y = Q_INT4(X) . Q_w(W)^T  (eq. 6).  Returns a dict of every intermediate."""
    T, alpha = ternarize(W, eps)
    q, d = quant_int4(X, eps)
    acc = matmul_int(q, T)
    return dict(T=T, alpha=alpha, q=q, d=d, acc=acc, y=rescale(acc, d, alpha, out_dtype))


def bitlinear_a8_sparse(X, W, k_sel, eps=DEFAULT_EPS, out_dtype="f32"):
    """Y = (Q_INT8(X) (.) Top_k(|X|)) . Q_w(W)^T  (eq. 1)."""
    T, alpha = ternarize(W, eps)
    q, d, mask = quant_topk_int8(X, k_sel, eps)
    acc = matmul_int(q, T)
    return dict(T=T, alpha=alpha, q=q, d=d, mask=mask, acc=acc,
                y=rescale(acc, d, alpha, out_dtype))


def bitlinear_fp4(X, W, eps=DEFAULT_EPS):
    """Y = Q_FP4(X) . Q_w(W)^T, float64 accumulation (the FP4 variant of eq. 6)."""
    T, alpha = ternarize(W, eps)
    codes, e = quant_fp4(X)
    xhat = fp4_dequant(codes, e)
    y = np.float64(alpha) * (xhat @ T.astype(np.float64).T)
    return dict(T=T, alpha=alpha, codes=codes, e=e, y=y)


def ffn_block(X, W_gate, W_up, W_down, k_sel, eps=DEFAULT_EPS):
    """One FFN block: INT4 -> gate/up, ReLU^2 GLU, top-k + INT8 -> down."""
    g = bitlinear_a4(X, W_gate, eps, "f32")
    u = bitlinear_a4(X, W_up, eps, "f32")
    h = relu2_glu(g["y"], u["y"])
    dn = bitlinear_a8_sparse(h, W_down, k_sel, eps, "bf16")
    return dict(gate=g, up=u, h=h, down=dn)


# --------------------------------------------------------------------------
# training: straight-through backward of a quantized linear
# --------------------------------------------------------------------------
def ste_backward(dY, q, d, T, alpha):
    """Gradients of Y = Q(X) . Q_w(W)^T under the straight-through estimator
    (Section 2.2, "Gradient approximation"): the quantizers of the activations
    and of the weights and the Top_k mask are passed over in the backward pass,
    i.e. dL/dX := dL/dQ(X) and dL/dW := dL/dQ_w(W).  With the dequantized
    operands  Xq = d_m * q[m, k]  (masked entries are zeros of q)  and
    Wq = alpha * T[n, k]  the layer is the plain product Y = Xq . Wq^T, hence

        dX[m, k] = sum_n dY[m, n] * Wq[n, k]         (does not depend on X or on the mask)
        dW[n, k] = sum_m dY[m, n] * Xq[m, k]         (the gradient for the latent weight)

    Everything in float64 (the paper fixes no precision for the backward pass
    beyond "mixed precision training")."""
    dY = np.asarray(dY, dtype=np.float64)
    Xq = np.asarray(d, dtype=np.float64)[:, None] * np.asarray(q, dtype=np.float64)
    Wq = np.float64(alpha) * np.asarray(T, dtype=np.float64)
    dX = dY @ Wq
    dW = dY.T @ Xq
    return dX, dW

