"""Thin ctypes binding of libbitlinear.so (the C ABI declared in include/bitlinear.h).

Argument marshalling only: every function allocates its outputs with torch (device
memory), passes raw device pointers and the current HIP stream, and checks the status
code.  No arithmetic of the method happens here, and there is no fallback: if the
library has not been built, loading fails loudly.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "lib", "libbitlinear.so")

BL_F32, BL_BF16 = 0, 1
BL_ACT_INT4_ABSMEAN, BL_ACT_TOPK_INT8_ABSMAX, BL_ACT_FP4_E2M1_B32, BL_ACT_INT4_ABSMEAN_MX6 = 0, 1, 2, 3
BL_ACT_FP4_E2M1_B32_MX = 4
BL_ACT_INT4_ABSMEAN2, BL_ACT_INT4_ABSMAX = 5, 6
BL_ACT_FP4_E1M2_B32 = 7
BL_W_GEMM, BL_W_KMAJOR, BL_W_MX4, BL_W_ROWS, BL_W_MX2 = 0, 1, 2, 3, 4
BL_DECODE_MAX_M = 64
DEFAULT_EPS = 1e-5

_lib = None

_vp, _i64, _f32, _sz, _int = ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_size_t, ctypes.c_int

_SIGNATURES = {
    "bl_padded_k": (_i64, [_i64]),
    "pack_ternary_bytes": (_sz, [_i64, _i64, _int]),
    "pack_ternary_workspace_bytes": (_sz, [_i64, _i64]),
    "pack_ternary": (_int, [_vp, _int, _i64, _i64, _f32, _int, _vp, _vp, _vp, _sz, _vp]),
    "quantize_act_bytes": (_sz, [_int, _i64, _i64]),
    "quantize_act": (_int, [_vp, _int, _i64, _i64, _int, _i64, _f32, _vp, _vp, _vp, _vp, _vp]),
    "bitlinear_workspace_bytes": (_sz, [_int, _i64, _i64, _i64]),
    "bitlinear_a4": (_int, [_vp, _int, _i64, _i64, _vp, _int, _vp, _i64, _f32, _int, _vp, _int,
                            _vp, _vp, _sz, _vp]),
    "bitlinear_a8_sparse": (_int, [_vp, _int, _i64, _i64, _i64, _vp, _int, _vp, _i64, _f32, _vp,
                                   _int, _vp, _vp, _sz, _vp]),
    "bitlinear_a8_sparse_static": (_int, [_vp, _int, _i64, _i64, _i64, _vp, _int, _vp, _i64, _f32, _vp,
                                          _int, _vp, _vp]),
    "bitlinear_gemm": (_int, [_vp, _vp, _int, _i64, _i64, _vp, _int, _vp, _i64, _vp, _int, _vp,
                              _vp, _sz, _vp]),
    "relu2_glu": (_int, [_vp, _vp, _int, _i64, _i64, _vp, _vp]),
    "swish_glu": (_int, [_vp, _vp, _int, _i64, _i64, _vp, _vp]),
    "quantize_heads_bytes": (_sz, [_int, _i64, _i64, _i64]),
    "quantize_heads": (_int, [_vp, _int, _i64, _i64, _i64, _int, _f32, _vp, _vp, _vp]),
    "dequantize_heads": (_int, [_vp, _vp, _i64, _i64, _i64, _int, _vp, _int, _vp]),
    "kv_cache_bytes": (_sz, [_i64, _i64, _i64]),
    "kv_cache_append": (_int, [_vp, _int, _i64, _i64, _i64, _i64, _f32, _vp, _vp, _vp]),
    "kv_cache_read": (_int, [_vp, _vp, _i64, _i64, _i64, _i64, _vp, _int, _vp]),
    "quantize_act_glu": (_int, [_vp, _vp, _int, _i64, _i64, _i64, _f32, _vp, _vp, _vp, _vp]),
    "bitlinear_gate_up_workspace_bytes": (_sz, [_i64, _i64, _i64, _int]),
    "bitlinear_a4_gate_up": (_int, [_vp, _int, _i64, _i64, _vp, _vp, _vp, _vp, _int, _i64, _f32, _vp, _vp, _int,
                                    _vp, _vp, _sz, _vp]),
    "bitlinear_gemm_glu": (_int, [_vp, _vp, _i64, _i64, _vp, _vp, _vp, _vp, _int, _i64, _vp, _vp]),
    "bitlinear_a4_up_gated": (_int, [_vp, _i64, _i64, _vp, _vp, _i64, _f32, _vp, _int, _vp, _vp]),
    "bitlinear_backward_workspace_bytes": (_sz, [_i64, _i64, _i64]),
    "bitlinear_backward": (_int, [_vp, _i64, _i64, _i64, _vp, _vp, _int, _vp, _int, _vp, _vp, _int, _vp, _vp, _sz, _vp]),
    "unpack_ternary": (_int, [_vp, _i64, _i64, _int, _vp, _vp]),
    "unpack_act": (_int, [_vp, _int, _i64, _i64, _vp, _vp]),
    "bl_noop": (_int, [_vp]),
    "bl_status_string": (ctypes.c_char_p, [_int]),
}


def lib():
    """Load the native library once; raise if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libbitlinear.so is not built (%s). Run `python -m paper_2411_04965_amd.build` "
                "first; there is no fallback path." % LIB_PATH)
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


class BitlinearError(RuntimeError):
    def __init__(self, fn, status):
        self.status = status
        msg = lib().bl_status_string(status).decode()
        super().__init__("%s failed: %s (%d)" % (fn, msg, status))


def _check(fn, status):
    if status != 0:
        raise BitlinearError(fn, status)


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _dt(t):
    if t.dtype == torch.float32:
        return BL_F32
    if t.dtype == torch.bfloat16:
        return BL_BF16
    raise TypeError("float32 or bfloat16 tensor expected, got %s" % t.dtype)


def _ptr(t):
    return None if t is None else t.data_ptr()


def _dev(t):
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("contiguous device tensor expected")
    return t


def noop():
    """Enqueue the library's empty kernel on the current stream (launch-floor measurements)."""
    _check("bl_noop", lib().bl_noop(_stream()))


def padded_k(K):
    return lib().bl_padded_k(K)


def pack_ternary(W, eps=DEFAULT_EPS, layout=BL_W_GEMM):
    """W [N, K] (device, fp32/bf16) -> (packed uint8 tensor, alpha float32[1])."""
    _dev(W)
    N, K = W.shape
    L = lib()
    packed = torch.empty(L.pack_ternary_bytes(N, K, layout), dtype=torch.uint8, device=W.device)
    alpha = torch.empty(1, dtype=torch.float32, device=W.device)
    wsb = L.pack_ternary_workspace_bytes(N, K)
    ws = torch.empty(wsb, dtype=torch.uint8, device=W.device)
    _check("pack_ternary", L.pack_ternary(_ptr(W), _dt(W), N, K, eps, layout, _ptr(packed),
                                          _ptr(alpha), _ptr(ws), wsb, _stream()))
    return packed, alpha


def unpack_ternary(packed, N, K, layout=BL_W_GEMM):
    T = torch.empty((N, K), dtype=torch.int8, device=packed.device)
    _check("unpack_ternary", lib().unpack_ternary(_ptr(packed), N, K, layout, _ptr(T), _stream()))
    return T


def quantize_act(X, mode, topk=0, eps=DEFAULT_EPS, want_rowsum=False, want_sel=False):
    """X [M, K] -> dict(q=packed codes uint8, scale, rowsum, sel)."""
    _dev(X)
    M, K = X.shape
    L = lib()
    q = torch.empty(L.quantize_act_bytes(mode, M, K), dtype=torch.uint8, device=X.device)
    if mode in (BL_ACT_FP4_E2M1_B32, BL_ACT_FP4_E1M2_B32):
        scale = torch.empty(M * (L.bl_padded_k(K) // 32), dtype=torch.uint8, device=X.device)
    elif mode == BL_ACT_FP4_E2M1_B32_MX:
        scale = torch.empty((M + 31) // 32 * 32 * (L.bl_padded_k(K) // 32), dtype=torch.uint8, device=X.device)
    else:
        scale = torch.empty(M, dtype=torch.float32, device=X.device)
    rowsum = torch.empty(M, dtype=torch.int32, device=X.device) if want_rowsum else None
    sel = torch.empty((M, topk), dtype=torch.int32, device=X.device) if want_sel else None
    _check("quantize_act", L.quantize_act(_ptr(X), _dt(X), M, K, mode, topk, eps, _ptr(q),
                                          _ptr(scale), _ptr(rowsum), _ptr(sel), _stream()))
    return dict(q=q, scale=scale, rowsum=rowsum, sel=sel)


def unpack_act(q, mode, M, K):
    codes = torch.empty((M, K), dtype=torch.int8, device=q.device)
    _check("unpack_act", lib().unpack_act(_ptr(q), mode, M, K, _ptr(codes), _stream()))
    return codes


def workspace(mode, M, N, K, device):
    n = lib().bitlinear_workspace_bytes(mode, M, N, K)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def _out(M, N, y_dtype, device, want_acc):
    Y = torch.empty((M, N), dtype=y_dtype, device=device)
    acc = torch.empty((M, N), dtype=torch.int32, device=device) if want_acc else None
    return Y, acc


def bitlinear_a4(X, W_packed, alpha, N, eps=DEFAULT_EPS, act_fp4=False, y_dtype=torch.bfloat16,
                 want_acc=False, ws=None, out=None, layout=BL_W_GEMM):
    _dev(X)
    M, K = X.shape
    if act_fp4:
        mode = BL_ACT_FP4_E2M1_B32_MX if layout in (BL_W_MX4, BL_W_MX2) else BL_ACT_FP4_E2M1_B32
    else:
        mode = BL_ACT_INT4_ABSMEAN_MX6 if layout in (BL_W_MX4, BL_W_MX2) else BL_ACT_INT4_ABSMEAN
    if ws is None:
        ws = workspace(mode, M, N, K, X.device)
    Y, acc = _out(M, N, y_dtype, X.device, want_acc) if out is None else (out, None)
    _check("bitlinear_a4", lib().bitlinear_a4(
        _ptr(X), _dt(X), M, K, _ptr(W_packed), layout, _ptr(alpha), N, eps, int(act_fp4),
        _ptr(Y), _dt(Y), _ptr(acc), _ptr(ws), ws.numel(), _stream()))
    return (Y, acc) if want_acc else Y


def bitlinear_a8_sparse(X, topk, W_packed, alpha, N, eps=DEFAULT_EPS, layout=BL_W_GEMM,
                        y_dtype=torch.bfloat16, want_acc=False, ws=None, out=None):
    _dev(X)
    M, K = X.shape
    if ws is None:
        ws = workspace(BL_ACT_TOPK_INT8_ABSMAX, M, N, K, X.device)
    Y, acc = _out(M, N, y_dtype, X.device, want_acc) if out is None else (out, None)
    _check("bitlinear_a8_sparse", lib().bitlinear_a8_sparse(
        _ptr(X), _dt(X), M, K, topk, _ptr(W_packed), layout, _ptr(alpha), N, eps, _ptr(Y),
        _dt(Y), _ptr(acc), _ptr(ws), ws.numel(), _stream()))
    return (Y, acc) if want_acc else Y


def bitlinear_a8_sparse_static(X, topk, W_packed, alpha, N, out, eps=DEFAULT_EPS, layout=BL_W_GEMM, acc=None):
    """bitlinear_a8_sparse on the library's static scratch: the caller brings the output (and the
    accumulator buffer if wanted); nothing is allocated here or in the library."""
    M, K = X.shape
    _check("bitlinear_a8_sparse_static", lib().bitlinear_a8_sparse_static(
        _ptr(X), _dt(X), M, K, topk, _ptr(W_packed), layout, _ptr(alpha), N, eps, _ptr(out), _dt(out),
        _ptr(acc), _stream()))
    return out


def bitlinear_gemm(q, scale, mode, M, K, W_packed, alpha, N, layout=BL_W_GEMM,
                   y_dtype=torch.bfloat16, want_acc=False, ws=None, out=None):
    if ws is None:
        ws = workspace(mode, M, N, K, q.device)
    Y, acc = _out(M, N, y_dtype, q.device, want_acc) if out is None else (out, None)
    _check("bitlinear_gemm", lib().bitlinear_gemm(
        _ptr(q), _ptr(scale), mode, M, K, _ptr(W_packed), layout, _ptr(alpha), N, _ptr(Y),
        _dt(Y), _ptr(acc), _ptr(ws), ws.numel(), _stream()))
    return (Y, acc) if want_acc else Y


def quantize_act_glu(G, U, topk, eps=DEFAULT_EPS, want_rowsum=False):
    """Rows of bf16(U * max(G, 0)^2) -> top-K + INT8 codes, without writing the rows out."""
    _dev(G), _dev(U)
    assert G.shape == U.shape and G.dtype == U.dtype
    M, K = G.shape
    L = lib()
    q = torch.empty(L.quantize_act_bytes(BL_ACT_TOPK_INT8_ABSMAX, M, K), dtype=torch.uint8, device=G.device)
    scale = torch.empty(M, dtype=torch.float32, device=G.device)
    rowsum = torch.empty(M, dtype=torch.int32, device=G.device) if want_rowsum else None
    _check("quantize_act_glu", L.quantize_act_glu(_ptr(G), _ptr(U), _dt(G), M, K, topk, eps, _ptr(q),
                                                  _ptr(scale), _ptr(rowsum), _stream()))
    return dict(q=q, scale=scale, rowsum=rowsum)


def bitlinear_a4_gate_up(X, W_gate, alpha_gate, W_up, alpha_up, N, eps=DEFAULT_EPS, layout=BL_W_GEMM,
                         want=("G", "U", "H"), gu_dtype=torch.float32, ws=None, out=None):
    """Gate and up projection on one quantized input.  Returns a dict with the tensors named in
    `want` (G, U of gu_dtype; H = bf16(U * max(G, 0)^2)); `out` may bring preallocated ones."""
    _dev(X)
    M, K = X.shape
    out = dict(out or {})
    for k in want:
        if k not in out:
            out[k] = torch.empty((M, N), dtype=torch.bfloat16 if k == "H" else gu_dtype, device=X.device)
    if ws is None:
        ws = torch.empty(max(lib().bitlinear_gate_up_workspace_bytes(M, N, K, layout), 16), dtype=torch.uint8,
                         device=X.device)
    G, U, H = out.get("G"), out.get("U"), out.get("H")
    gdt = _dt(G) if G is not None else (_dt(U) if U is not None else BL_F32)
    _check("bitlinear_a4_gate_up", lib().bitlinear_a4_gate_up(
        _ptr(X), _dt(X), M, K, _ptr(W_gate), _ptr(alpha_gate), _ptr(W_up), _ptr(alpha_up), layout, N, eps,
        _ptr(G), _ptr(U), gdt, _ptr(H), _ptr(ws), ws.numel(), _stream()))
    return out


def gemm_a4_glu_prequantized(L, q, scale, M, K, Wg, Wu, layout, N, H, stream):
    """Raw call of bitlinear_gemm_glu on preallocated buffers (Wg, Wu = (packed, alpha) pairs); returns the status."""
    return L.bitlinear_gemm_glu(q.data_ptr(), scale.data_ptr(), M, K, Wg[0].data_ptr(), Wg[1].data_ptr(),
                                Wu[0].data_ptr(), Wu[1].data_ptr(), layout, N, H.data_ptr(), stream)


def bitlinear_a4_up_gated(X, W_rows, alpha, N, G, eps=DEFAULT_EPS):
    """Gate-first up projection: H = bf16(U * max(G, 0)^2), U computed only where a gate is open."""
    _dev(X), _dev(G)
    assert X.dtype == torch.bfloat16
    M, K = X.shape
    H = torch.empty((M, N), dtype=torch.bfloat16, device=X.device)
    _check("bitlinear_a4_up_gated", lib().bitlinear_a4_up_gated(
        _ptr(X), M, K, _ptr(W_rows), _ptr(alpha), N, eps, _ptr(G), _dt(G), _ptr(H), _stream()))
    return H


def relu2_glu(G, U):
    _dev(G), _dev(U)
    M, N = G.shape
    H = torch.empty((M, N), dtype=torch.bfloat16, device=G.device)
    _check("relu2_glu", lib().relu2_glu(_ptr(G), _ptr(U), _dt(G), M, N, _ptr(H), _stream()))
    return H


def quantize_heads(X, bits, eps=DEFAULT_EPS):
    """X [T, H, D] -> (packed codes uint8 [T * H * D * bits / 8], scale float32 [T, H])."""
    _dev(X)
    T, H, D = X.shape
    L = lib()
    q = torch.empty(L.quantize_heads_bytes(bits, T, H, D), dtype=torch.uint8, device=X.device)
    scale = torch.empty((T, H), dtype=torch.float32, device=X.device)
    _check("quantize_heads", L.quantize_heads(_ptr(X), _dt(X), T, H, D, bits, eps, _ptr(q), _ptr(scale), _stream()))
    return q, scale


def dequantize_heads(q, scale, T, H, D, bits, out_dtype=torch.float32):
    out = torch.empty((T, H, D), dtype=out_dtype, device=q.device)
    _check("dequantize_heads", lib().dequantize_heads(_ptr(q), _ptr(scale), T, H, D, bits, _ptr(out), _dt(out), _stream()))
    return out


def kv_cache_new(T_max, H, D, device):
    """Empty mixed-width key / value cache for T_max positions: (codes uint8, scales float32 [T_max, H])."""
    return (torch.zeros(lib().kv_cache_bytes(T_max, H, D), dtype=torch.uint8, device=device),
            torch.zeros((T_max, H), dtype=torch.float32, device=device))


def kv_cache_append(X, pos0, cache, scales, eps=DEFAULT_EPS):
    _dev(X)
    T, H, D = X.shape
    _check("kv_cache_append", lib().kv_cache_append(_ptr(X), _dt(X), T, H, D, pos0, eps, _ptr(cache), _ptr(scales), _stream()))


def kv_cache_read(cache, scales, pos0, T, H, D, out_dtype=torch.float32):
    out = torch.empty((T, H, D), dtype=out_dtype, device=cache.device)
    _check("kv_cache_read", lib().kv_cache_read(_ptr(cache), _ptr(scales), pos0, T, H, D, _ptr(out), _dt(out), _stream()))
    return out


def bitlinear_backward(dY, q, scale, mode, K, W_kmajor, alpha, want_dx=True, want_dw=True,
                       dx_dtype=torch.bfloat16, ws=None):
    """Straight-through backward (Section 2.2): dY [M, N] bfloat16 and the forward's codes -> (dX, dW)."""
    _dev(dY)
    M, N = dY.shape
    L = lib()
    if ws is None:
        ws = torch.empty(max(L.bitlinear_backward_workspace_bytes(M, N, K), 16), dtype=torch.uint8, device=dY.device)
    dX = torch.empty((M, K), dtype=dx_dtype, device=dY.device) if want_dx else None
    dW = torch.empty((N, K), dtype=torch.float32, device=dY.device) if want_dw else None
    _check("bitlinear_backward", L.bitlinear_backward(
        _ptr(dY), M, N, K, _ptr(q), _ptr(scale), mode, _ptr(W_kmajor), BL_W_KMAJOR, _ptr(alpha), _ptr(dX),
        BL_F32 if dx_dtype == torch.float32 else BL_BF16, _ptr(dW), _ptr(ws), ws.numel(), _stream()))
    return dX, dW


def swish_glu(G, U):
    _dev(G), _dev(U)
    M, N = G.shape
    H = torch.empty((M, N), dtype=torch.bfloat16, device=G.device)
    _check("swish_glu", lib().swish_glu(_ptr(G), _ptr(U), _dt(G), M, N, _ptr(H), _stream()))
    return H
