// Shared device/host helpers of the gfx950 BitNet a4.8 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <type_traits>

#include "../../include/bitlinear.h"

#define BL_KPAD 256   // K padding unit of every packed format
#define BL_WAVE 64

#define BL_HIP_CHECK_LAUNCH()                         \
  do {                                                \
    if (hipGetLastError() != hipSuccess) return BL_EHIP; \
  } while (0)

static inline int64_t bl_round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }
static inline bool bl_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
// A one-dimensional grid holds at most 2^31 - 1 workgroups.
static inline bool bl_grid_ok(int64_t blocks) { return blocks >= 1 && blocks <= (int64_t)0x7FFFFFFF; }

// Compute units of the current device (cached per device; 256 if the query fails).
int bl_num_cus();

// Raise a kernel's dynamic LDS limit to `BYTES`, once per device and call site (a driver call,
// kept off the launch path after the first time).  Expands to a statement that returns BL_EHIP
// from the enclosing function when the driver refuses.
#define BL_SET_MAX_LDS_ONCE(KERN, BYTES)                                                          \
  do {                                                                                            \
    static std::atomic<unsigned long long> bl_done_{0};                                           \
    int bl_dev_ = 0;                                                                              \
    if (hipGetDevice(&bl_dev_) != hipSuccess) return BL_EHIP;                                     \
    const unsigned long long bl_bit_ = 1ull << (bl_dev_ & 63);                                    \
    if (!(bl_done_.load(std::memory_order_acquire) & bl_bit_)) {                                  \
      if (hipFuncSetAttribute((const void*)(KERN), hipFuncAttributeMaxDynamicSharedMemorySize,    \
                              (int)(BYTES)) != hipSuccess)                                        \
        return BL_EHIP;                                                                           \
      bl_done_.fetch_or(bl_bit_, std::memory_order_release);                                      \
    }                                                                                             \
  } while (0)

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int u32;

// bfloat16 <-> float32 on raw bits.
__device__ __forceinline__ float bl_bf16_to_f32(uint16_t b) { return __uint_as_float(((u32)b) << 16); }
__device__ __forceinline__ uint16_t bl_f32_to_bf16_rne(float f) {
  u32 u = __float_as_uint(f);
  u32 lsb = (u >> 16) & 1u;
  return (uint16_t)((u + 0x7FFFu + lsb) >> 16);   // finite inputs only
}

// Sum over a 64-lane wave (all lanes get the result).
__device__ __forceinline__ double bl_wave_sum_f64(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
// The same sum with DPP moves instead of LDS permutes (a third of the latency); exact sums only,
// the order of the additions differs.
__device__ __forceinline__ double bl_wave_sum_f64_dpp(double v) {
  // sum over the 64 lanes: 16-lane rows with DPP (two 32-bit moves per step), rows with readlane
  auto step = [&](auto ctrl) {
    constexpr int C = decltype(ctrl)::value;
    const u32 lo = (u32)__double_as_longlong(v), hi = (u32)(__double_as_longlong(v) >> 32);
    const u32 plo = (u32)__builtin_amdgcn_update_dpp(0, (int)lo, C, 0xF, 0xF, false);
    const u32 phi = (u32)__builtin_amdgcn_update_dpp(0, (int)hi, C, 0xF, 0xF, false);
    v += __longlong_as_double((long long)(((unsigned long long)phi << 32) | plo));
  };
  step(std::integral_constant<int, 0x121>{});    // row_ror:1
  step(std::integral_constant<int, 0x122>{});    // row_ror:2
  step(std::integral_constant<int, 0x124>{});    // row_ror:4
  step(std::integral_constant<int, 0x128>{});    // row_ror:8
  const u32 lo = (u32)__double_as_longlong(v), hi = (u32)(__double_as_longlong(v) >> 32);
  double t = 0.0;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const u32 a = (u32)__builtin_amdgcn_readlane((int)lo, 16 * r), b = (u32)__builtin_amdgcn_readlane((int)hi, 16 * r);
    t += __longlong_as_double((long long)(((unsigned long long)b << 32) | a));
  }
  return t;
}
__device__ __forceinline__ int bl_wave_sum_i32(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ u32 bl_wave_max_u32(u32 v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    u32 t = (u32)__shfl_xor((int)v, o, 64);
    v = t > v ? t : v;
  }
  return v;
}

// Tile index -> tile origin.  Blocks are dealt round-robin to the 8 XCDs, so tiles whose index
// is congruent mod 8 run on one XCD: give each XCD a contiguous range of the tile order, and
// walk that order in groups of 4 token tiles, so that the tiles an XCD works on at one time
// share activations and weights in its L2.
__device__ __forceinline__ void bl_tile_origin(int t, int n_tiles, int MT, int NTB, int BM, int BN,
                                               int& m0, int& n0) {
  const int q = n_tiles >> 3, rmd = n_tiles & 7, xcd = t & 7, loc = t >> 3;
  const int pid = xcd * q + min(xcd, rmd) + loc;
  constexpr int GM = 4;
  const int per_group = GM * NTB;
  const int group = pid / per_group, in_group = pid % per_group;
  const int first_m = group * GM;
  const int gsz = min(MT - first_m, GM);
  m0 = (first_m + in_group % gsz) * BM;
  n0 = (in_group / gsz) * BN;
}

// Internal launchers (one per source file); all return a bl_status.
int bl_launch_pack_ternary(const void* W, bl_dtype dt, int64_t N, int64_t K, float eps,
                           bl_w_layout layout, void* out, float* alpha, void* ws, hipStream_t s);
int bl_launch_unpack_ternary(const void* packed, int64_t N, int64_t K, bl_w_layout layout,
                             int8_t* T, hipStream_t s);
int bl_launch_quantize_glu(const void* G, const void* U, bl_dtype dt, int64_t M, int64_t K, int64_t topk,
                           float eps, void* q, void* scale, int32_t* rowsum, hipStream_t s);
int bl_launch_quantize(const void* X, bl_dtype dt, int64_t M, int64_t K, bl_act_mode mode,
                       int64_t topk, float eps, void* q, void* scale, int32_t* rowsum,
                       int32_t* sel_idx, hipStream_t s);
int bl_launch_unpack_act(const void* q, bl_act_mode mode, int64_t M, int64_t K, int8_t* codes,
                         hipStream_t s);
int bl_launch_quantize_heads(const void* X, bl_dtype dt, int64_t n_heads, int64_t D, int bits, float eps,
                             void* q, float* scale, hipStream_t s);
int bl_launch_dequantize_heads(const void* q, const float* scale, int64_t n_heads, int64_t D, int bits, void* out,
                               bl_dtype odt, hipStream_t s);
int bl_launch_gemm_prefill(const void* q, const float* scale, bl_act_mode mode, int64_t M,
                           int64_t K, const void* Wp, const float* alpha, int64_t N, void* Y,
                           bl_dtype ydt, int32_t* acc_out, hipStream_t s);
int bl_launch_gemm_decode(const void* q, const float* scale, bl_act_mode mode, int64_t M,
                          int64_t K, const void* Wp, const float* alpha, int64_t N, void* Y,
                          bl_dtype ydt, int32_t* acc_out, void* ws, hipStream_t s);
size_t bl_gemm_decode_ws_bytes(int64_t M, int64_t N, int64_t K);
bool bl_gemv_a4_fused_ok(int64_t M, int64_t N, int64_t K);
int bl_launch_up_gated(const void* X, int64_t M, int64_t K, float eps, const void* Wr, const float* alpha,
                       int64_t N, const void* G, bl_dtype gdt, void* H, hipStream_t s);
bool bl_gemv_a8_fused_ok(int64_t M, int64_t N, int64_t K);
int bl_launch_gemv_a8_fused(const void* X, int64_t K, int64_t topk, float eps, const void* Wp,
                            const float* alpha, int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out,
                            hipStream_t s);
int bl_launch_gemv_a4_fused(const void* X, int64_t M, int64_t K, float eps, const void* Wp,
                            const float* alpha, int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out,
                            hipStream_t s);
// one persistent launch for up to 16 tokens (gemv_stream.hip)
bool bl_gemv_stream_ok(int64_t M, int64_t N, int64_t K, bool quant_inside);
bool bl_gemv_stream_pair_ok(int64_t M, int64_t N, int64_t K, bool glu);
int bl_launch_gemv_stream(const void* q, const float* scale, bool a4, int64_t M, int64_t K, const void* Wp,
                          const float* alpha, int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out, hipStream_t s);
int bl_launch_gemv_stream_a4(const void* X, int64_t M, int64_t K, float eps, const void* Wp, const float* alpha,
                             int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out, hipStream_t s);
bool bl_gemv_stream_topk_ok(int64_t M, int64_t N, int64_t K);
int bl_launch_gemv_stream_topk(const void* X, int64_t K, int64_t topk, float eps, const void* Wp, const float* alpha,
                               int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out, hipStream_t s);
int bl_launch_gemv_stream_gate_up(const void* X, int64_t M, int64_t K, float eps, const void* Wg, const float* ag,
                                  const void* Wu, const float* au, int64_t N, void* G, void* U, bl_dtype ydt,
                                  void* H, hipStream_t s);
int bl_launch_gemv_sparse(const void* q, const float* scale, int64_t M, int64_t K,
                          const void* Wk, const float* alpha, int64_t N, void* Y, bl_dtype ydt,
                          int32_t* acc_out, void* ws, hipStream_t s);
size_t bl_gemv_sparse_ws_bytes(int64_t M, int64_t N, int64_t K);
int bl_launch_gemm_a4_mx(const void* q, const float* scale, int64_t M, int64_t K, const void* Wp, bool w2,
                         const float* alpha, int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out,
                         hipStream_t s);
int bl_launch_gemm_a4_mx_glu(const void* q, const float* scale, int64_t M, int64_t K, const void* Wg, const float* ag,
                             const void* Wu, const float* au, bool w2, int64_t N, void* H, hipStream_t s);
int bl_launch_gemm_fp4_mx(const void* q, const uint8_t* xscale, int64_t M, int64_t K, const void* Wp, bool w2,
                          const float* alpha, int64_t N, void* Y, bl_dtype ydt, hipStream_t s);
int bl_launch_gemm_fp4(const void* q, const uint8_t* scale, int64_t M, int64_t K, const void* Wp,
                       const float* alpha, int64_t N, void* Y, bl_dtype ydt, hipStream_t s);
size_t bl_ste_workspace_bytes(int64_t M, int64_t N, int64_t K);
int bl_launch_ste_backward(const void* dY, int64_t M, int64_t N, int64_t K, const void* q, const float* scale, bool a4,
                           const void* Wk, const float* alpha, void* dX, bl_dtype dx_dtype, float* dW, void* ws,
                           hipStream_t s);
bool bl_gemm_decode_glu_ok(int64_t M, int64_t N, int64_t K);
int bl_launch_gemm_decode_glu(const void* q, const float* scale, int64_t M, int64_t K, const void* Wg, const float* ag,
                              const void* Wu, const float* au, int64_t N, void* H, hipStream_t s);
bool bl_gemv_stream_glu_codes_ok(int64_t M, int64_t N, int64_t K);
int bl_launch_gemv_stream_glu_codes(const void* q, const float* scale, int64_t M, int64_t K, const void* Wg,
                                    const float* ag, const void* Wu, const float* au, int64_t N, void* H, hipStream_t s);

