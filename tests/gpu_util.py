"""Helpers shared by the GPU parity tests (host <-> device plumbing, format decoders).

The decoders below are written from the format description in include/bitlinear.h, in
numpy, so that packed bytes coming back from the GPU are checked against the documented
layout and not only against the library's own unpack kernels."""
import numpy as np
import torch

from paper_2411_04965_amd import binding as B

EPS = 1e-5
REL_TOL = 1e-3          # spec tolerance on rescaled outputs


def dev(x, dtype=torch.float32):
    """numpy float32 array -> device tensor (bf16 conversion is exact for bf16-valued data)."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
    return t.to(dtype).contiguous()


def host(t):
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.cpu().numpy()


def decode_w_gemm(packed, N, K):
    """BL_W_GEMM bytes -> int8 [N, K]."""
    Kp = (K + 255) // 256 * 256
    Np = (N + 15) // 16 * 16
    words = np.frombuffer(packed.tobytes(), dtype="<u4").reshape(Np // 16, Kp // 256, 4, 16, 4)
    # [nt, kt, g, i, t] ; field f of a word holds channel 16 t + 4 (f % 4) + f // 4
    f = np.arange(16)
    fields = (words[..., None] >> (2 * f)) & 3                      # [nt, kt, g, i, t, f]
    T = np.where(fields == 3, -1, fields).astype(np.int8)
    assert not (fields == 2).any()
    kk = 4 * (f % 4) + f // 4
    out = np.zeros((Np // 16, 16, Kp // 256, 4, 4, 16), dtype=np.int8)   # [nt, i, kt, g, t, kk]
    out[..., kk] = np.transpose(T, (0, 3, 1, 2, 4, 5))
    full = out.reshape(Np, Kp)
    assert not full[N:].any() and not full[:, K:].any()
    return full[:N, :K]


def decode_w_kmajor(packed, N, K):
    """BL_W_KMAJOR bytes -> int8 [N, K]."""
    Np = (N + 511) // 512 * 512
    words = np.frombuffer(packed.tobytes(), dtype="<u4").reshape(Np // 512, K, 32)
    f = np.arange(16)
    fields = (words[..., None] >> (2 * f)) & 3                      # [cb, k, d, f]
    assert not (fields == 2).any()
    T = np.where(fields == 3, -1, fields).astype(np.int8)
    full = np.transpose(T, (0, 2, 3, 1)).reshape(Np, K)             # n = 512 cb + 16 d + f
    assert not full[N:].any()
    return full[:N]


def decode_int4(q, M, K):
    Kp = (K + 255) // 256 * 256
    b = np.frombuffer(q.tobytes(), dtype=np.uint8).reshape(M, Kp // 8, 4)
    lo = (b & 15).astype(np.int8)
    hi = (b >> 4).astype(np.int8)
    lo = np.where(lo > 7, lo - 16, lo)
    hi = np.where(hi > 7, hi - 16, hi)
    full = np.concatenate([lo, hi], axis=2).reshape(M, Kp)         # k0+b then k0+4+b
    assert not full[:, K:].any()
    return full[:, :K].astype(np.int8)


def decode_w_mx4(packed, N, K):
    """BL_W_MX4 bytes -> int8 [N, K]."""
    Kp = (K + 255) // 256 * 256
    Np = (N + 31) // 32 * 32
    b = np.frombuffer(packed.tobytes(), dtype=np.uint8).reshape(Np // 32, Kp // 128, 32, 4, 16)
    r = np.arange(32)
    u = np.arange(4)
    piece = u[None, :] ^ ((r[:, None] >> 2) & 3)                    # [r, u] -> piece that holds unit u
    units = b[:, :, r[:, None], piece, :]                           # [nb, kb, r, u, 16]
    nib = np.stack([units & 15, units >> 4], axis=-1).reshape(Np // 32, Kp // 128, 32, 4, 32)
    assert np.isin(nib, (0, 2, 10)).all()
    T = np.where(nib == 2, 1, np.where(nib == 10, -1, 0)).astype(np.int8)
    full = np.transpose(T, (0, 2, 1, 3, 4)).reshape(Np, Kp)         # n = 32 nb + r, k = 128 kb + 32 u + i
    assert not full[N:].any() and not full[:, K:].any()
    return full[:N, :K]


def decode_w_mx2(packed, N, K):
    """BL_W_MX2 bytes -> int8 [N, K]: 1 KB blocks of 32 outputs x 128 channels, 2-bit codes."""
    Kp = (K + 255) // 256 * 256
    Np = (N + 31) // 32 * 32
    w = np.frombuffer(packed.tobytes(), dtype="<u4").reshape(Np // 32, Kp // 128, 32, 4, 2)
    r = np.arange(32)
    u = np.arange(4)
    piece = u[None, :] ^ ((r[:, None] >> 3) & 3)                    # [r, u] -> piece that holds unit u
    units = w[:, :, r[:, None], piece, :]                           # [nb, kb, r, u, 2 words]
    j = np.arange(8, dtype=np.uint32)
    nib = (units[..., None] >> (4 * j)) & 15                        # s_j s_8+j m_j m_8+j
    lo = np.where(nib & 2, np.where(nib & 8, -1, 1), 0)             # channels 0..7 of the word's 16
    hi = np.where(nib & 1, np.where(nib & 4, -1, 1), 0)             # channels 8..15
    assert not ((nib & 8) & ~((nib & 2) << 2)).any() and not ((nib & 4) & ~((nib & 1) << 2)).any()   # no -0
    T = np.concatenate([lo, hi], axis=-1).reshape(Np // 32, Kp // 128, 32, 4, 32).astype(np.int8)
    full = np.transpose(T, (0, 2, 1, 3, 4)).reshape(Np, Kp)
    assert not full[N:].any() and not full[:, K:].any()
    return full[:N, :K]


def decode_w_rows(packed, N, K):
    """BL_W_ROWS bytes -> int8 [N, K]: row n = Kp/4 bytes, channel k in bits 2 (k % 16) of word k / 16."""
    Kp = (K + 255) // 256 * 256
    w = np.frombuffer(packed.tobytes(), dtype="<u4").reshape(N, Kp // 16)
    f = np.arange(16, dtype=np.uint32)
    c = ((w[:, :, None] >> (2 * f)) & 3).reshape(N, Kp).astype(np.int8)
    T = np.where(c == 3, -1, c).astype(np.int8)
    assert not (c == 2).any() and not T[:, K:].any()
    return T[:, :K]


def decode_int4_mx6(q, M, K):
    """INT4 levels in the MX6 form (E3M2 codes, 32-token blocks) -> int8 [M, K]."""
    Kp = (K + 255) // 256 * 256
    Mp = (M + 31) // 32 * 32
    b = np.frombuffer(q.tobytes(), dtype=np.uint8).reshape(Mp // 32, Kp // 128, 3072)
    P = b[:, :, :2048].reshape(Mp // 32, Kp // 128, 32, 4, 16)
    Q = b[:, :, 2048:].reshape(Mp // 32, Kp // 128, 32, 4, 8)
    r = np.arange(32)
    u = np.arange(4)
    pp = u[None, :] ^ ((r[:, None] >> 2) & 3)
    qq = u[None, :] ^ ((r[:, None] >> 3) & 3)
    stream = np.concatenate([P[:, :, r[:, None], pp, :], Q[:, :, r[:, None], qq, :]], axis=-1)   # [mb, kb, r, u, 24]
    bits = np.unpackbits(stream, axis=-1, bitorder="little").reshape(Mp // 32, Kp // 128, 32, 4, 32, 6)
    code = (bits * (1 << np.arange(6))).sum(-1)
    code = np.transpose(code, (0, 2, 1, 3, 4)).reshape(Mp, Kp)[:M]  # rows past M are never written
    e, mant, sign = (code >> 2) & 7, code & 3, code >> 5
    mag = np.where(e == 0, 0.0, (1 + mant / 4.0) * 2.0 ** (e - 3.0))
    assert np.array_equal(mag, np.round(mag)) and mag.max() <= 8
    assert not (code == 32).any(), "-0 code"
    full = np.where(sign == 1, -mag, mag)
    assert not full[:, K:].any()
    return full[:, :K].astype(np.int8)


def decode_int8(q, M, K):
    Kp = (K + 255) // 256 * 256
    full = np.frombuffer(q.tobytes(), dtype=np.int8).reshape(M, Kp)
    assert not full[:, K:].any()
    return full[:, :K]


def decode_fp4(q, M, K):
    Kp = (K + 255) // 256 * 256
    words = np.frombuffer(q.tobytes(), dtype="<u4").reshape(M, Kp // 16, 2)
    j = np.arange(8)
    nib = (words[..., None] >> (4 * j)) & 15                        # [M, grp, word, j]
    out = np.zeros((M, Kp // 16, 16), dtype=np.uint8)
    kk = 8 * (j % 2) + j // 2
    out[:, :, kk] = nib[:, :, 0, :]
    out[:, :, 4 + kk] = nib[:, :, 1, :]
    full = out.reshape(M, Kp)
    assert not full[:, K:].any()
    return full[:, :K]


def decode_fp4_mx(q, sc, M, K):
    """FP4 MX form (32-token blocks, natural nibble order; scales 128 bytes per block) ->
    nibble codes uint8 [M, K] and E8M0 bytes uint8 [M, Kp/32]."""
    Kp = (K + 255) // 256 * 256
    Mp = (M + 31) // 32 * 32
    b = np.frombuffer(q.tobytes(), dtype=np.uint8).reshape(Mp // 32, Kp // 128, 32, 4, 16)
    r = np.arange(32)
    u = np.arange(4)
    piece = u[None, :] ^ ((r[:, None] >> 2) & 3)                    # [r, u] -> piece that holds unit u
    units = b[:, :, r[:, None], piece, :]                           # [mb, kb, r, u, 16]
    nib = np.stack([units & 15, units >> 4], axis=-1).reshape(Mp // 32, Kp // 128, 32, 4, 32)
    full = np.transpose(nib, (0, 2, 1, 3, 4)).reshape(Mp, Kp)       # m = 32 mb + r, k = 128 kb + 32 u + i
    assert not full[:M, K:].any()
    e = np.frombuffer(sc.tobytes(), dtype=np.uint8).reshape(Mp // 32, Kp // 128, 32, 4)
    e = np.transpose(e, (0, 2, 1, 3)).reshape(Mp, Kp // 32)
    return full[:M, :K], e[:M]


def assert_close_rel(y_gpu, y_ref, tol=REL_TOL):
    """|gpu - ref| <= tol * |ref| element-wise (plus a denormal-sized floor)."""
    y_gpu = np.asarray(y_gpu, dtype=np.float64)
    y_ref = np.asarray(y_ref, dtype=np.float64)
    err = np.abs(y_gpu - y_ref)
    bound = tol * np.abs(y_ref) + 1e-30
    bad = err > bound
    assert not bad.any(), "max rel err %g at %s" % ((err / (np.abs(y_ref) + 1e-30)).max(),
                                                     np.argwhere(bad)[:5].tolist())


def pack(W, layout=B.BL_W_GEMM, dtype=torch.float32):
    return B.pack_ternary(dev(W, dtype), EPS, layout)


def decode_heads(q, T, H, D, bits):
    """Packed head codes (little-endian bit stream per head, `bits` bits per code) -> uint8 [T, H, D]."""
    b = np.frombuffer(q.tobytes(), dtype=np.uint8).reshape(T * H, D * bits // 8)
    bitsarr = np.unpackbits(b, axis=1, bitorder="little").reshape(T * H, D, bits)
    w = (1 << np.arange(bits)).astype(np.uint8)
    return (bitsarr * w).sum(axis=2).astype(np.uint8).reshape(T, H, D)
