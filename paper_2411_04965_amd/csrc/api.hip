// C ABI of the library: argument validation and kernel dispatch.  See include/bitlinear.h for
// the contract of every entry point.
#include "common.h"

#include <mutex>

static inline size_t ws_align(size_t x) { return (x + 255) & ~(size_t)255; }

static bool valid_dtype(int d) { return d == BL_F32 || d == BL_BF16; }
static bool valid_layout(int l) { return l >= BL_W_GEMM && l <= BL_W_MX2; }
static bool mx_layout(int l) { return l == BL_W_MX4 || l == BL_W_MX2; }
static bool valid_mode(int m) { return m >= BL_ACT_INT4_ABSMEAN && m <= BL_ACT_FP4_E1M2_B32; }
static bool int4_nibble_mode(int m) {
  return m == BL_ACT_INT4_ABSMEAN || m == BL_ACT_INT4_ABSMEAN2 || m == BL_ACT_INT4_ABSMAX;
}
static bool mx_mode(int m) { return m == BL_ACT_INT4_ABSMEAN_MX6 || m == BL_ACT_FP4_E2M1_B32_MX; }
static bool fp4_mode(int m) {
  return m == BL_ACT_FP4_E2M1_B32 || m == BL_ACT_FP4_E2M1_B32_MX || m == BL_ACT_FP4_E1M2_B32;
}

static int check_sizes(int64_t M, int64_t N, int64_t K) {
  if (M < 1 || N < 1 || K < 1) return BL_EINVAL;
  if (K > BL_MAX_K) return BL_ESHAPE;
  const int64_t lim = (int64_t)1 << 40;
  if (M > lim / N || N > lim / K || M > ((int64_t)1 << 31) - 1 || N > ((int64_t)1 << 31) - 1) return BL_ESHAPE;
  return BL_OK;
}

extern "C" int64_t bl_padded_k(int64_t K) { return bl_round_up(K, BL_KPAD); }

// Every elementwise launcher runs 256 threads per workgroup, one element (or block of 32) each.
static bool elementwise_grid_ok(int64_t n) { return bl_grid_ok((n + 255) / 256); }

int bl_num_cus() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  std::atomic<int>& slot = cached[dev & 63];
  int cus = slot.load(std::memory_order_relaxed);
  if (cus == 0) {
    int v = 0;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 256;
    cus = v;
    slot.store(cus, std::memory_order_relaxed);
  }
  return cus;
}

__global__ void bl_noop_kernel() {}

extern "C" int bl_noop(void* stream) {
  bl_noop_kernel<<<1, 64, 0, (hipStream_t)stream>>>();
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

extern "C" const char* bl_status_string(int status) {
  switch (status) {
    case BL_OK: return "ok";
    case BL_EINVAL: return "invalid argument";
    case BL_ESHAPE: return "unsupported size";
    case BL_EALIGN: return "pointer not 16-byte aligned";
    case BL_EWORKSPACE: return "workspace missing or too small";
    case BL_EHIP: return "HIP launch failed";
    case BL_EUNSUPPORTED: return "not implemented for these arguments";
    case BL_ESCRATCH: return "request needs more scratch memory than the library's static buffer holds";
    default: return "unknown status";
  }
}

// ---------------------------------------------------------------- weights
extern "C" size_t pack_ternary_bytes(int64_t N, int64_t K, bl_w_layout layout) {
  if (N < 1 || K < 1) return 0;
  if (layout == BL_W_GEMM) return (size_t)(bl_round_up(N, 16) * bl_round_up(K, BL_KPAD) / 4);
  if (layout == BL_W_KMAJOR) return (size_t)(bl_round_up(N, 512) / 4 * K);
  if (layout == BL_W_MX4) return (size_t)(bl_round_up(N, 32) * bl_round_up(K, BL_KPAD) / 2);
  if (layout == BL_W_MX2) return (size_t)(bl_round_up(N, 32) * bl_round_up(K, BL_KPAD) / 4);
  if (layout == BL_W_ROWS) return (size_t)(N * bl_round_up(K, BL_KPAD) / 4);
  return 0;
}

extern "C" int pack_ternary(const void* W, bl_dtype w_dtype, int64_t N, int64_t K, float eps,
                            bl_w_layout layout, void* packed_out, float* alpha_out,
                            void* workspace, size_t workspace_bytes, void* stream) {
  if (!W || !packed_out || !alpha_out) return BL_EINVAL;
  if (!valid_dtype(w_dtype) || !valid_layout(layout) || !(eps >= 0.0f)) return BL_EINVAL;
  int rc = check_sizes(1, N, K);
  if (rc) return rc;
  if (!bl_aligned16(W) || !bl_aligned16(packed_out)) return BL_EALIGN;
  if (!workspace || workspace_bytes < pack_ternary_workspace_bytes(N, K)) return BL_EWORKSPACE;
  if (!bl_aligned16(workspace)) return BL_EALIGN;
  return bl_launch_pack_ternary(W, w_dtype, N, K, eps, layout, packed_out, alpha_out, workspace,
                                (hipStream_t)stream);
}

extern "C" int unpack_ternary(const void* packed, int64_t N, int64_t K, bl_w_layout layout,
                              int8_t* T_out, void* stream) {
  if (!packed || !T_out || !valid_layout(layout)) return BL_EINVAL;
  int rc = check_sizes(1, N, K);
  if (rc) return rc;
  if (!elementwise_grid_ok(N * K)) return BL_ESHAPE;
  return bl_launch_unpack_ternary(packed, N, K, layout, T_out, (hipStream_t)stream);
}

// ---------------------------------------------------------------- activations
extern "C" size_t quantize_act_bytes(bl_act_mode mode, int64_t M, int64_t K) {
  if (M < 1 || K < 1) return 0;
  const int64_t Kp = bl_round_up(K, BL_KPAD);
  switch (mode) {
    case BL_ACT_INT4_ABSMEAN:
    case BL_ACT_INT4_ABSMEAN2:
    case BL_ACT_INT4_ABSMAX: return (size_t)(M * Kp / 2);
    case BL_ACT_TOPK_INT8_ABSMAX: return (size_t)(M * Kp);
    case BL_ACT_FP4_E2M1_B32:
    case BL_ACT_FP4_E1M2_B32: return (size_t)(M * Kp / 2);
    case BL_ACT_INT4_ABSMEAN_MX6: return (size_t)(bl_round_up(M, 32) * Kp / 4 * 3);
    case BL_ACT_FP4_E2M1_B32_MX: return (size_t)(bl_round_up(M, 32) * Kp / 2);
    default: return 0;
  }
}

static size_t act_scale_bytes(bl_act_mode mode, int64_t M, int64_t K) {
  if (mode == BL_ACT_FP4_E2M1_B32 || mode == BL_ACT_FP4_E1M2_B32)
    return (size_t)(M * (bl_round_up(K, BL_KPAD) / 32));
  if (mode == BL_ACT_FP4_E2M1_B32_MX) return (size_t)(bl_round_up(M, 32) * (bl_round_up(K, BL_KPAD) / 32));
  return (size_t)M * sizeof(float);
}

extern "C" int quantize_act(const void* X, bl_dtype x_dtype, int64_t M, int64_t K,
                            bl_act_mode mode, int64_t topk, float eps, void* q_out,
                            void* scale_out, int32_t* rowsum_out, int32_t* sel_idx_out,
                            void* stream) {
  if (!X || !q_out || !scale_out) return BL_EINVAL;
  if (!valid_dtype(x_dtype) || !valid_mode(mode) || !(eps >= 0.0f)) return BL_EINVAL;
  int rc = check_sizes(M, 1, K);
  if (rc) return rc;
  if (mode == BL_ACT_TOPK_INT8_ABSMAX && (topk < 1 || topk > K)) return BL_EINVAL;
  if (mode != BL_ACT_TOPK_INT8_ABSMAX && sel_idx_out) return BL_EINVAL;
  if (fp4_mode(mode) && rowsum_out) return BL_EINVAL;
  if (fp4_mode(mode) && !elementwise_grid_ok(M * (bl_round_up(K, BL_KPAD) / 32))) return BL_ESHAPE;
  if (!bl_aligned16(X) || !bl_aligned16(q_out)) return BL_EALIGN;
  return bl_launch_quantize(X, x_dtype, M, K, mode, topk, eps, q_out, scale_out, rowsum_out,
                            sel_idx_out, (hipStream_t)stream);
}

extern "C" int quantize_act_glu(const void* G, const void* U, bl_dtype in_dtype, int64_t M, int64_t K,
                                int64_t topk, float eps, void* q_out, float* scale_out,
                                int32_t* rowsum_out, void* stream) {
  if (!G || !U || !q_out || !scale_out) return BL_EINVAL;
  if (!valid_dtype(in_dtype) || !(eps >= 0.0f)) return BL_EINVAL;
  int rc = check_sizes(M, 1, K);
  if (rc) return rc;
  if (topk < 1 || topk > K) return BL_EINVAL;
  if (!bl_aligned16(G) || !bl_aligned16(U) || !bl_aligned16(q_out)) return BL_EALIGN;
  return bl_launch_quantize_glu(G, U, in_dtype, M, K, topk, eps, q_out, scale_out, rowsum_out,
                                (hipStream_t)stream);
}

extern "C" int unpack_act(const void* q, bl_act_mode mode, int64_t M, int64_t K,
                          int8_t* codes_out, void* stream) {
  if (!q || !codes_out || !valid_mode(mode)) return BL_EINVAL;
  if (int4_nibble_mode(mode)) mode = BL_ACT_INT4_ABSMEAN;
  int rc = check_sizes(M, 1, K);
  if (rc) return rc;
  if (!elementwise_grid_ok(M * K)) return BL_ESHAPE;
  return bl_launch_unpack_act(q, mode, M, K, codes_out, (hipStream_t)stream);
}

// ---------------------------------------------------------------- attention states (Section 4.2)
extern "C" size_t quantize_heads_bytes(int bits, int64_t T, int64_t H, int64_t D) {
  if ((bits != 3 && bits != 4) || T < 1 || H < 1 || D < 8 || D % 8 != 0) return 0;
  return (size_t)(T * H * (D / 8) * bits);
}

extern "C" int quantize_heads(const void* X, bl_dtype x_dtype, int64_t T, int64_t H, int64_t D, int bits,
                              float eps, void* q_out, float* scale_out, void* stream) {
  if (!X || !q_out || !scale_out) return BL_EINVAL;
  if (!valid_dtype(x_dtype) || (bits != 3 && bits != 4) || !(eps >= 0.0f)) return BL_EINVAL;
  if (T < 1 || H < 1 || D < 1) return BL_EINVAL;
  if (D % 8 != 0 || D > BL_MAX_K) return BL_ESHAPE;
  const int64_t lim = (int64_t)1 << 40;
  if (T > lim / H || T * H > lim / D) return BL_ESHAPE;
  // the kernels take 4 or 16 heads per workgroup: bound the grid by the smaller
  if (!bl_grid_ok((T * H + 3) / 4)) return BL_ESHAPE;
  if (!bl_aligned16(X) || !bl_aligned16(q_out)) return BL_EALIGN;
  return bl_launch_quantize_heads(X, x_dtype, T * H, D, bits, eps, q_out, scale_out, (hipStream_t)stream);
}

extern "C" int dequantize_heads(const void* q, const float* scale, int64_t T, int64_t H, int64_t D, int bits,
                                void* out, bl_dtype out_dtype, void* stream) {
  if (!q || !scale || !out) return BL_EINVAL;
  if (!valid_dtype(out_dtype) || (bits != 3 && bits != 4)) return BL_EINVAL;
  if (T < 1 || H < 1 || D < 1) return BL_EINVAL;
  if (D % 8 != 0 || D > BL_MAX_K) return BL_ESHAPE;
  const int64_t lim = (int64_t)1 << 40;
  if (T > lim / H || T * H > lim / D) return BL_ESHAPE;
  if (!bl_aligned16(out)) return BL_EALIGN;
  return bl_launch_dequantize_heads(q, scale, T * H, D, bits, out, out_dtype, (hipStream_t)stream);
}

// The 3-bit key / value cache with the first token's heads at 4 bits (Table 3): byte offset of the
// token at sequence position `pos`.
static int64_t kv_token_offset(int64_t pos, int64_t H, int64_t D) {
  return pos == 0 ? 0 : H * (D / 2) + (pos - 1) * H * (3 * D / 8);
}

extern "C" size_t kv_cache_bytes(int64_t T, int64_t H, int64_t D) {
  if (T < 1 || H < 1 || D < 8 || D % 8 != 0) return 0;
  return (size_t)kv_token_offset(T, H, D);
}

static int kv_check(int64_t T, int64_t H, int64_t D, int64_t pos0) {
  if (T < 1 || H < 1 || D < 1 || pos0 < 0) return BL_EINVAL;
  // D % 32: every token's codes then start on a 4-byte boundary, which the quantizer's stores need
  if (D % 32 != 0 || D > BL_MAX_K) return BL_ESHAPE;
  const int64_t lim = (int64_t)1 << 40;
  if (pos0 > lim - T || (pos0 + T) > lim / H || (pos0 + T) * H > lim / D) return BL_ESHAPE;
  if (!bl_grid_ok((T * H + 3) / 4)) return BL_ESHAPE;
  return BL_OK;
}

extern "C" int kv_cache_append(const void* X, bl_dtype x_dtype, int64_t T, int64_t H, int64_t D, int64_t pos0,
                               float eps, void* cache, float* scales, void* stream) {
  if (!X || !cache || !scales) return BL_EINVAL;
  if (!valid_dtype(x_dtype) || !(eps >= 0.0f)) return BL_EINVAL;
  int rc = kv_check(T, H, D, pos0);
  if (rc) return rc;
  if (!bl_aligned16(X) || !bl_aligned16(cache)) return BL_EALIGN;
  const size_t esz = x_dtype == BL_BF16 ? 2 : 4;
  const unsigned char* x = (const unsigned char*)X;
  unsigned char* c = (unsigned char*)cache;
  int64_t t = 0;
  if (pos0 == 0) {                                         // the sequence's first token: 4 bits
    rc = bl_launch_quantize_heads(x, x_dtype, H, D, 4, eps, c, scales, (hipStream_t)stream);
    if (rc) return rc;
    t = 1;
  }
  if (t < T)
    rc = bl_launch_quantize_heads(x + (size_t)t * H * D * esz, x_dtype, (T - t) * H, D, 3, eps,
                                  c + kv_token_offset(pos0 + t, H, D), scales + (pos0 + t) * H, (hipStream_t)stream);
  return rc;
}

extern "C" int kv_cache_read(const void* cache, const float* scales, int64_t pos0, int64_t T, int64_t H, int64_t D,
                             void* out, bl_dtype out_dtype, void* stream) {
  if (!cache || !scales || !out) return BL_EINVAL;
  if (!valid_dtype(out_dtype)) return BL_EINVAL;
  int rc = kv_check(T, H, D, pos0);
  if (rc) return rc;
  if (!bl_aligned16(out)) return BL_EALIGN;
  const size_t esz = out_dtype == BL_BF16 ? 2 : 4;
  const unsigned char* c = (const unsigned char*)cache;
  unsigned char* o = (unsigned char*)out;
  int64_t t = 0;
  if (pos0 == 0) {
    rc = bl_launch_dequantize_heads(c, scales, H, D, 4, o, out_dtype, (hipStream_t)stream);
    if (rc) return rc;
    t = 1;
  }
  if (t < T)
    rc = bl_launch_dequantize_heads(c + kv_token_offset(pos0 + t, H, D), scales + (pos0 + t) * H, (T - t) * H, D, 3,
                                    o + (size_t)t * H * D * esz, out_dtype, (hipStream_t)stream);
  return rc;
}

// ---------------------------------------------------------------- ReLU^2 GLU (eq. 5)
template <typename RawT>
__global__ __launch_bounds__(256) void relu2_glu_kernel(const RawT* __restrict__ G,
                                                        const RawT* __restrict__ U, int64_t n,
                                                        uint16_t* __restrict__ H) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float g, u;
  if (sizeof(RawT) == 2) {
    g = bl_bf16_to_f32((uint16_t)G[i]);
    u = bl_bf16_to_f32((uint16_t)U[i]);
  } else {
    g = __uint_as_float((u32)G[i]);
    u = __uint_as_float((u32)U[i]);
  }
  const float r = fmaxf(g, 0.0f);
  const float rr = r * r;
  H[i] = bl_f32_to_bf16_rne(u * rr);
}

// Swish GLU (Section 4.3): h = u * (g * sigmoid(g)), float32 steps, one bfloat16 rounding
template <typename RawT>
__global__ __launch_bounds__(256) void swish_glu_kernel(const RawT* __restrict__ G,
                                                        const RawT* __restrict__ U, int64_t n,
                                                        uint16_t* __restrict__ H) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n) return;
  float g, u;
  if (sizeof(RawT) == 2) {
    g = bl_bf16_to_f32((uint16_t)G[i]);
    u = bl_bf16_to_f32((uint16_t)U[i]);
  } else {
    g = __uint_as_float((u32)G[i]);
    u = __uint_as_float((u32)U[i]);
  }
  const float sg = 1.0f / (1.0f + expf(-g));               // expf(-g) = inf for g < -88.7: sg = 0, h = -0
  const float sw = g * sg;
  H[i] = bl_f32_to_bf16_rne(u * sw);
}

// ---------------------------------------------------------------- linear layers
// Workspace layout: [codes | scales | stage-2 scratch], each part 256-byte aligned.
static size_t stage2_ws_bytes(bl_act_mode mode, int64_t M, int64_t N, int64_t K) {
  if (fp4_mode(mode) || mx_mode(mode) || M > BL_DECODE_MAX_M) return 0;
  size_t a = bl_gemm_decode_ws_bytes(M, N, K);
  if (mode == BL_ACT_TOPK_INT8_ABSMAX && M <= BL_SPARSE_MAX_M) {
    const size_t b = bl_gemv_sparse_ws_bytes(M, N, K);
    if (b > a) a = b;
  }
  return a;
}

extern "C" size_t bitlinear_workspace_bytes(bl_act_mode mode, int64_t M, int64_t N, int64_t K) {
  if (!valid_mode(mode) || M < 1 || N < 1 || K < 1) return 0;
  return ws_align(quantize_act_bytes(mode, M, K)) + ws_align(act_scale_bytes(mode, M, K)) +
         ws_align(stage2_ws_bytes(mode, M, N, K));
}

static int gemm_dispatch(const void* q, const void* scale, bl_act_mode mode, int64_t M, int64_t K,
                         const void* W_packed, bl_w_layout layout, const float* alpha, int64_t N,
                         void* Y, bl_dtype y_dtype, int32_t* acc_out, void* ws, size_t ws_bytes,
                         hipStream_t s) {
  // the block-float forms of activations and weights go together and with nothing else
  if (layout == BL_W_ROWS) return BL_EUNSUPPORTED;       // only the gate-first up projection reads rows
  if (mode == BL_ACT_FP4_E1M2_B32) return BL_EUNSUPPORTED;   // a quantizer format only: no MFMA operand type
  if (int4_nibble_mode(mode)) mode = BL_ACT_INT4_ABSMEAN;   // same codes, same rescale
  if (mx_mode(mode) != mx_layout(layout)) return BL_EINVAL;
  if (mode == BL_ACT_INT4_ABSMEAN_MX6)
    return bl_launch_gemm_a4_mx(q, (const float*)scale, M, K, W_packed, layout == BL_W_MX2, alpha, N, Y, y_dtype,
                                acc_out, s);
  if (mode == BL_ACT_FP4_E2M1_B32_MX) {
    if (acc_out) return BL_EINVAL;
    return bl_launch_gemm_fp4_mx(q, (const uint8_t*)scale, M, K, W_packed, layout == BL_W_MX2, alpha, N, Y,
                                 y_dtype, s);
  }
  if (mode == BL_ACT_FP4_E2M1_B32) {
    if (layout != BL_W_GEMM || acc_out) return BL_EINVAL;
    return bl_launch_gemm_fp4(q, (const uint8_t*)scale, M, K, W_packed, alpha, N, Y, y_dtype, s);
  }
  if (layout == BL_W_KMAJOR) {
    if (mode != BL_ACT_TOPK_INT8_ABSMAX) return BL_EUNSUPPORTED;
    if (M > BL_SPARSE_MAX_M) return BL_EUNSUPPORTED;
    if (!ws || ws_bytes < bl_gemv_sparse_ws_bytes(M, N, K)) return BL_EWORKSPACE;
    return bl_launch_gemv_sparse(q, (const float*)scale, M, K, W_packed, alpha, N, Y, y_dtype,
                                 acc_out, ws, s);
  }
  if (M <= BL_DECODE_MAX_M) {
    const size_t need = bl_gemm_decode_ws_bytes(M, N, K);
    if (need && (!ws || ws_bytes < need)) return BL_EWORKSPACE;
    return bl_launch_gemm_decode(q, (const float*)scale, mode, M, K, W_packed, alpha, N, Y,
                                 y_dtype, acc_out, ws, s);
  }
  return bl_launch_gemm_prefill(q, (const float*)scale, mode, M, K, W_packed, alpha, N, Y,
                                y_dtype, acc_out, s);
}

extern "C" int bitlinear_gemm(const void* q, const void* scale, bl_act_mode mode, int64_t M,
                              int64_t K, const void* W_packed, bl_w_layout layout,
                              const float* alpha, int64_t N, void* Y, bl_dtype y_dtype,
                              int32_t* acc_out, void* workspace, size_t workspace_bytes,
                              void* stream) {
  if (!q || !scale || !W_packed || !alpha || !Y) return BL_EINVAL;
  if (!valid_mode(mode) || !valid_layout(layout) || !valid_dtype(y_dtype)) return BL_EINVAL;
  int rc = check_sizes(M, N, K);
  if (rc) return rc;
  if (!bl_aligned16(q) || !bl_aligned16(W_packed) || !bl_aligned16(Y) ||
      (acc_out && !bl_aligned16(acc_out)) || (workspace && !bl_aligned16(workspace)))
    return BL_EALIGN;
  // scales: float32 per token, or E8M0 block scales that the FP4 GEMMs fetch four at a time
  if (reinterpret_cast<uintptr_t>(scale) & 3) return BL_EALIGN;
  return gemm_dispatch(q, scale, mode, M, K, W_packed, layout, alpha, N, Y, y_dtype, acc_out,
                       workspace, workspace_bytes, (hipStream_t)stream);
}

static int linear_common(const void* X, bl_dtype x_dtype, int64_t M, int64_t K, bl_act_mode mode,
                         int64_t topk, const void* W_packed, bl_w_layout layout,
                         const float* alpha, int64_t N, float eps, void* Y, bl_dtype y_dtype,
                         int32_t* acc_out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!X || !W_packed || !alpha || !Y) return BL_EINVAL;
  if (!valid_dtype(x_dtype) || !valid_dtype(y_dtype) || !valid_layout(layout) || !(eps >= 0.0f))
    return BL_EINVAL;
  int rc = check_sizes(M, N, K);
  if (rc) return rc;
  if (mode == BL_ACT_TOPK_INT8_ABSMAX && (topk < 1 || topk > K)) return BL_EINVAL;
  if (!bl_aligned16(X) || !bl_aligned16(W_packed) || !bl_aligned16(Y) ||
      (acc_out && !bl_aligned16(acc_out)))
    return BL_EALIGN;
  if (!workspace || workspace_bytes < bitlinear_workspace_bytes(mode, M, N, K)) return BL_EWORKSPACE;
  if (!bl_aligned16(workspace)) return BL_EALIGN;
  // reject what the second stage would reject, before the first kernel is enqueued
  if (mode == BL_ACT_FP4_E2M1_B32 && (layout != BL_W_GEMM || acc_out)) return BL_EINVAL;
  if (mode == BL_ACT_FP4_E2M1_B32_MX && acc_out) return BL_EINVAL;
  if (mx_mode(mode) != mx_layout(layout)) return BL_EINVAL;
  if (layout == BL_W_KMAJOR && (mode != BL_ACT_TOPK_INT8_ABSMAX || M > BL_SPARSE_MAX_M)) return BL_EUNSUPPORTED;
  if (layout == BL_W_ROWS) return BL_EUNSUPPORTED;

  // a few tokens: quantizer and product in one launch
  if (mode == BL_ACT_INT4_ABSMEAN && layout == BL_W_GEMM && x_dtype == BL_BF16 &&
      bl_gemv_stream_ok(M, N, K, true))
    return bl_launch_gemv_stream_a4(X, M, K, eps, W_packed, alpha, N, Y, y_dtype, acc_out,
                                    (hipStream_t)stream);

  if (mode == BL_ACT_TOPK_INT8_ABSMAX && layout == BL_W_GEMM && x_dtype == BL_BF16 &&
      bl_gemv_stream_topk_ok(M, N, K))
    return bl_launch_gemv_stream_topk(X, K, topk, eps, W_packed, alpha, N, Y, y_dtype, acc_out,
                                      (hipStream_t)stream);

  unsigned char* p = (unsigned char*)workspace;
  void* codes = p;
  p += ws_align(quantize_act_bytes(mode, M, K));
  void* scales = p;
  p += ws_align(act_scale_bytes(mode, M, K));
  void* ws2 = p;
  const size_t ws2_bytes = workspace_bytes - (size_t)(p - (unsigned char*)workspace);
  rc = bl_launch_quantize(X, x_dtype, M, K, mode, topk, eps, codes, scales, nullptr, nullptr,
                          (hipStream_t)stream);
  if (rc) return rc;
  return gemm_dispatch(codes, scales, mode, M, K, W_packed, layout, alpha, N, Y, y_dtype, acc_out,
                       ws2, ws2_bytes, (hipStream_t)stream);
}

extern "C" int bitlinear_a4(const void* X, bl_dtype x_dtype, int64_t M, int64_t K,
                            const void* W_packed, bl_w_layout layout, const float* alpha,
                            int64_t N, float eps, int act_fp4, void* Y, bl_dtype y_dtype,
                            int32_t* acc_out, void* workspace, size_t workspace_bytes,
                            void* stream) {
  if (act_fp4 != 0 && act_fp4 != 1) return BL_EINVAL;
  if (layout != BL_W_GEMM && !mx_layout(layout)) return valid_layout(layout) ? BL_EUNSUPPORTED : BL_EINVAL;
  const bl_act_mode int4_mode = mx_layout(layout) ? BL_ACT_INT4_ABSMEAN_MX6 : BL_ACT_INT4_ABSMEAN;
  const bl_act_mode fp4_mode_ = mx_layout(layout) ? BL_ACT_FP4_E2M1_B32_MX : BL_ACT_FP4_E2M1_B32;
  return linear_common(X, x_dtype, M, K, act_fp4 ? fp4_mode_ : int4_mode, 0,
                       W_packed, layout, alpha, N, eps, Y, y_dtype, acc_out, workspace,
                       workspace_bytes, stream);
}

extern "C" int bitlinear_a8_sparse(const void* X, bl_dtype x_dtype, int64_t M, int64_t K,
                                   int64_t topk, const void* W_packed, bl_w_layout layout,
                                   const float* alpha, int64_t N, float eps, void* Y,
                                   bl_dtype y_dtype, int32_t* acc_out, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  return linear_common(X, x_dtype, M, K, BL_ACT_TOPK_INT8_ABSMAX, topk, W_packed, layout, alpha,
                       N, eps, Y, y_dtype, acc_out, workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------- the entry point that allocates nothing
// Scratch memory of bitlinear_a8_sparse_static: lives in the library's device image, one copy per
// GPU, from load to process end.  The name below is a host-side stand-in: device code and HIP calls
// get the array's address on the current device from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char scratch[BL_STATIC_SCRATCH_BYTES];

static int static_scratch_ptr(void** out) {
  static std::mutex mu;
  static void* ptrs[64] = {nullptr};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return BL_EHIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptrs[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BL_EHIP;
    ptrs[dev] = p;
  }
  *out = ptrs[dev];
  return BL_OK;
}

extern "C" int bitlinear_a8_sparse_static(const void* X, bl_dtype x_dtype, int64_t M, int64_t K, int64_t topk,
                                          const void* W_packed, bl_w_layout layout, const float* alpha,
                                          int64_t N, float eps, void* Y, bl_dtype y_dtype, int32_t* acc_out,
                                          void* stream) {
  if (M < 1 || N < 1 || K < 1) return BL_EINVAL;
  if (M > BL_DECODE_MAX_M) return BL_ESCRATCH;
  const size_t need = bitlinear_workspace_bytes(BL_ACT_TOPK_INT8_ABSMAX, M, N, K);
  if (need > (size_t)BL_STATIC_SCRATCH_BYTES) return BL_ESCRATCH;
  void* ws = nullptr;
  const int rc = static_scratch_ptr(&ws);
  if (rc) return rc;
  // (nothing in the scratch has to start at zero: codes, scales and every partial sum that is read
  // are written by this call's own kernels first)
  return linear_common(X, x_dtype, M, K, BL_ACT_TOPK_INT8_ABSMAX, topk, W_packed, layout, alpha, N, eps, Y,
                       y_dtype, acc_out, ws, (size_t)BL_STATIC_SCRATCH_BYTES, stream);
}

// ---------------------------------------------------------------- gate and up projection on one quantized input
extern "C" size_t bitlinear_gate_up_workspace_bytes(int64_t M, int64_t N, int64_t K, bl_w_layout layout) {
  if (M < 1 || N < 1 || K < 1) return 0;
  const bl_act_mode mode = mx_layout(layout) ? BL_ACT_INT4_ABSMEAN_MX6 : BL_ACT_INT4_ABSMEAN;
  return bitlinear_workspace_bytes(mode, M, N, K) + 2 * ws_align((size_t)M * N * sizeof(float));
}

extern "C" int bitlinear_a4_gate_up(const void* X, bl_dtype x_dtype, int64_t M, int64_t K, const void* W_gate,
                                    const float* alpha_gate, const void* W_up, const float* alpha_up,
                                    bl_w_layout layout, int64_t N, float eps, void* G, void* U, bl_dtype gu_dtype,
                                    void* H, void* workspace, size_t workspace_bytes, void* stream) {
  if (!X || !W_gate || !alpha_gate || !W_up || !alpha_up || (!G && !U && !H)) return BL_EINVAL;
  if (!valid_dtype(x_dtype) || !valid_dtype(gu_dtype) || !valid_layout(layout) || !(eps >= 0.0f)) return BL_EINVAL;
  if (layout != BL_W_GEMM && !mx_layout(layout)) return BL_EUNSUPPORTED;
  int rc = check_sizes(M, N, K);
  if (rc) return rc;
  if (!bl_aligned16(X) || !bl_aligned16(W_gate) || !bl_aligned16(W_up) || (G && !bl_aligned16(G)) ||
      (U && !bl_aligned16(U)) || (H && !bl_aligned16(H)))
    return BL_EALIGN;
  hipStream_t s = (hipStream_t)stream;
  // a few tokens: quantizer, both products and the combine in one launch, no workspace
  if (layout == BL_W_GEMM && x_dtype == BL_BF16 && bl_gemv_stream_pair_ok(M, N, K, H != nullptr))
    return bl_launch_gemv_stream_gate_up(X, M, K, eps, W_gate, alpha_gate, W_up, alpha_up, N, G, U, gu_dtype, H, s);

  // composed: quantize once, two products, then the combine on float32 G and U
  const bl_act_mode mode = mx_layout(layout) ? BL_ACT_INT4_ABSMEAN_MX6 : BL_ACT_INT4_ABSMEAN;
  const size_t base = bitlinear_workspace_bytes(mode, M, N, K);
  if (!workspace || workspace_bytes < base) return BL_EWORKSPACE;
  if (!bl_aligned16(workspace)) return BL_EALIGN;
  if (H && !elementwise_grid_ok(M * N)) return BL_ESHAPE;
  unsigned char* p = (unsigned char*)workspace;
  void* codes = p;
  p += ws_align(quantize_act_bytes(mode, M, K));
  void* scales = p;
  p += ws_align(act_scale_bytes(mode, M, K));
  void* ws2 = p;
  const size_t ws2_bytes = ws_align(stage2_ws_bytes(mode, M, N, K));
  p += ws2_bytes;
  // block-float weights and only H wanted: one GEMM over both matrices with eq. 5 in its epilogue
  if (mx_layout(layout) && H && !G && !U) {
    rc = bl_launch_quantize(X, x_dtype, M, K, mode, 0, eps, codes, scales, nullptr, nullptr, s);
    if (rc) return rc;
    return bl_launch_gemm_a4_mx_glu(codes, (const float*)scales, M, K, W_gate, alpha_gate, W_up, alpha_up,
                                    layout == BL_W_MX2, N, H, s);
  }
  // 9 to 16 tokens (or tokens that are not bfloat16), 2-bit tile weights, only H wanted: the stand-alone
  // quantizer, then both products and eq. 5 in one launch of the streaming kernel
  if (layout == BL_W_GEMM && H && !G && !U && bl_gemv_stream_glu_codes_ok(M, N, K)) {
    rc = bl_launch_quantize(X, x_dtype, M, K, mode, 0, eps, codes, scales, nullptr, nullptr, s);
    if (rc) return rc;
    return bl_launch_gemv_stream_glu_codes(codes, (const float*)scales, M, K, W_gate, alpha_gate, W_up, alpha_up, N, H, s);
  }
  // 17 to 64 tokens, 2-bit tile weights, only H wanted: both products and eq. 5 in one launch of the
  // kernel that keeps the tokens' codes in LDS
  if (layout == BL_W_GEMM && H && !G && !U && bl_gemm_decode_glu_ok(M, N, K)) {
    rc = bl_launch_quantize(X, x_dtype, M, K, mode, 0, eps, codes, scales, nullptr, nullptr, s);
    if (rc) return rc;
    return bl_launch_gemm_decode_glu(codes, (const float*)scales, M, K, W_gate, alpha_gate, W_up, alpha_up, N, H, s);
  }
  // when H is wanted the products are kept in float32 (eq. 5 combines them before any rounding)
  const bool need_f32 = H != nullptr && gu_dtype != BL_F32;
  void* Gt = G;
  void* Ut = U;
  bl_dtype tdt = gu_dtype;
  if (H && (!G || need_f32)) { Gt = p; p += ws_align((size_t)M * N * sizeof(float)); tdt = BL_F32; }
  if (H && (!U || need_f32)) { Ut = p; p += ws_align((size_t)M * N * sizeof(float)); tdt = BL_F32; }
  if ((size_t)(p - (unsigned char*)workspace) > workspace_bytes) return BL_EWORKSPACE;
  rc = bl_launch_quantize(X, x_dtype, M, K, mode, 0, eps, codes, scales, nullptr, nullptr, s);
  if (rc) return rc;
  if (H && need_f32) {
    // float32 copies for the combine, and the caller's own G / U in its dtype
    rc = gemm_dispatch(codes, scales, mode, M, K, W_gate, layout, alpha_gate, N, Gt, BL_F32, nullptr, ws2, ws2_bytes, s);
    if (rc) return rc;
    rc = gemm_dispatch(codes, scales, mode, M, K, W_up, layout, alpha_up, N, Ut, BL_F32, nullptr, ws2, ws2_bytes, s);
    if (rc) return rc;
    if (G) { rc = gemm_dispatch(codes, scales, mode, M, K, W_gate, layout, alpha_gate, N, G, gu_dtype, nullptr, ws2, ws2_bytes, s); if (rc) return rc; }
    if (U) { rc = gemm_dispatch(codes, scales, mode, M, K, W_up, layout, alpha_up, N, U, gu_dtype, nullptr, ws2, ws2_bytes, s); if (rc) return rc; }
  } else {
    if (Gt) { rc = gemm_dispatch(codes, scales, mode, M, K, W_gate, layout, alpha_gate, N, Gt, tdt, nullptr, ws2, ws2_bytes, s); if (rc) return rc; }
    if (Ut) { rc = gemm_dispatch(codes, scales, mode, M, K, W_up, layout, alpha_up, N, Ut, tdt, nullptr, ws2, ws2_bytes, s); if (rc) return rc; }
  }
  if (H) {
    const int64_t n = M * N;
    relu2_glu_kernel<u32><<<(unsigned)((n + 255) / 256), 256, 0, s>>>((const u32*)Gt, (const u32*)Ut, n, (uint16_t*)H);
    BL_HIP_CHECK_LAUNCH();
  }
  return BL_OK;
}

extern "C" int bitlinear_gemm_glu(const void* q, const float* scale, int64_t M, int64_t K, const void* W_gate,
                                  const float* alpha_gate, const void* W_up, const float* alpha_up,
                                  bl_w_layout layout, int64_t N, void* H, void* stream) {
  if (!q || !scale || !W_gate || !alpha_gate || !W_up || !alpha_up || !H) return BL_EINVAL;
  if (!valid_layout(layout)) return BL_EINVAL;
  if (!mx_layout(layout)) return BL_EUNSUPPORTED;
  int rc = check_sizes(M, N, K);
  if (rc) return rc;
  if (!bl_aligned16(q) || !bl_aligned16(W_gate) || !bl_aligned16(W_up) || !bl_aligned16(H)) return BL_EALIGN;
  if (reinterpret_cast<uintptr_t>(scale) & 3) return BL_EALIGN;
  return bl_launch_gemm_a4_mx_glu(q, scale, M, K, W_gate, alpha_gate, W_up, alpha_up, layout == BL_W_MX2, N, H,
                                  (hipStream_t)stream);
}

extern "C" int bitlinear_a4_up_gated(const void* X, int64_t M, int64_t K, const void* W_rows,
                                     const float* alpha, int64_t N, float eps, const void* G,
                                     bl_dtype g_dtype, void* H, void* stream) {
  if (!X || !W_rows || !alpha || !G || !H) return BL_EINVAL;
  if (!valid_dtype(g_dtype) || !(eps >= 0.0f)) return BL_EINVAL;
  int rc = check_sizes(M, N, K);
  if (rc) return rc;
  if (!bl_aligned16(X) || !bl_aligned16(W_rows)) return BL_EALIGN;
  // G and H are read and written one element at a time: natural alignment is all they need
  if ((reinterpret_cast<uintptr_t>(G) & (g_dtype == BL_F32 ? 3 : 1)) || (reinterpret_cast<uintptr_t>(H) & 1))
    return BL_EALIGN;
  return bl_launch_up_gated(X, M, K, eps, W_rows, alpha, N, G, g_dtype, H, (hipStream_t)stream);
}

extern "C" int swish_glu(const void* G, const void* U, bl_dtype in_dtype, int64_t M, int64_t N,
                         void* H, void* stream) {
  if (!G || !U || !H || !valid_dtype(in_dtype)) return BL_EINVAL;
  if (M < 1 || N < 1 || M > ((int64_t)1 << 40) / N) return BL_ESHAPE;
  const int64_t n = M * N;
  if (!elementwise_grid_ok(n)) return BL_ESHAPE;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  if (in_dtype == BL_BF16)
    swish_glu_kernel<uint16_t><<<blocks, 256, 0, (hipStream_t)stream>>>((const uint16_t*)G, (const uint16_t*)U, n, (uint16_t*)H);
  else
    swish_glu_kernel<u32><<<blocks, 256, 0, (hipStream_t)stream>>>((const u32*)G, (const u32*)U, n, (uint16_t*)H);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

extern "C" int relu2_glu(const void* G, const void* U, bl_dtype in_dtype, int64_t M, int64_t N,
                         void* H, void* stream) {
  if (!G || !U || !H || !valid_dtype(in_dtype)) return BL_EINVAL;
  if (M < 1 || N < 1 || M > ((int64_t)1 << 40) / N) return BL_ESHAPE;
  const int64_t n = M * N;
  if (!elementwise_grid_ok(n)) return BL_ESHAPE;
  const unsigned blocks = (unsigned)((n + 255) / 256);
  if (in_dtype == BL_BF16)
    relu2_glu_kernel<uint16_t><<<blocks, 256, 0, (hipStream_t)stream>>>((const uint16_t*)G, (const uint16_t*)U, n, (uint16_t*)H);
  else
    relu2_glu_kernel<u32><<<blocks, 256, 0, (hipStream_t)stream>>>((const u32*)G, (const u32*)U, n, (uint16_t*)H);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

// ---------------------------------------------------------------- straight-through backward (Section 2.2)
extern "C" size_t bitlinear_backward_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  if (M < 1 || N < 1 || K < 1 || M > ((int64_t)1 << 31) || N > ((int64_t)1 << 24) || K > BL_MAX_K) return 0;
  return bl_ste_workspace_bytes(M, N, K);
}

extern "C" int bitlinear_backward(const void* dY, int64_t M, int64_t N, int64_t K, const void* q, const float* scale,
                                  bl_act_mode mode, const void* W_packed, bl_w_layout layout, const float* alpha,
                                  void* dX, bl_dtype dx_dtype, float* dW, void* workspace, size_t workspace_bytes,
                                  void* stream) {
  if (!dY || !q || !scale || !W_packed || !alpha || !workspace || (!dX && !dW)) return BL_EINVAL;
  if (!valid_dtype(dx_dtype)) return BL_EINVAL;
  if (mode != BL_ACT_INT4_ABSMEAN && mode != BL_ACT_TOPK_INT8_ABSMAX) return BL_EUNSUPPORTED;
  if (layout != BL_W_KMAJOR) return BL_EUNSUPPORTED;
  if (M < 1 || N < 1 || K < 1) return BL_EINVAL;
  if (M > ((int64_t)1 << 30) || N > ((int64_t)1 << 24) || K > BL_MAX_K) return BL_ESHAPE;
  if (!bl_aligned16(dY) || !bl_aligned16(q) || !bl_aligned16(W_packed) || !bl_aligned16(workspace) ||
      (dX && !bl_aligned16(dX)) || (dW && !bl_aligned16(dW)) || (reinterpret_cast<uintptr_t>(scale) & 3))
    return BL_EALIGN;
  if (workspace_bytes < bl_ste_workspace_bytes(M, N, K)) return BL_EWORKSPACE;
  return bl_launch_ste_backward(dY, M, N, K, q, scale, mode == BL_ACT_INT4_ABSMEAN, W_packed, alpha, dX, dx_dtype, dW,
                                workspace, (hipStream_t)stream);
}

