// Low-bit attention states (Section 4.2 of the paper, "Low-bit Attention"; Table 3): every head
// vector of a token (post-RoPE query, key or value) is quantized on its own with the absmax
// function to 4 or 3 bits and stored as an unsigned integer:
//   gamma = max |x| over the head,  q = RoundClip(Q_b / (gamma + eps) * x, -Q_b, Q_b),
//   Q_b = 2^(bits-1) - 1,  code = q + 2^(bits-1),  scale = gamma / Q_b.
// HBM bound: 2 D bytes in (bfloat16), D bits / 8 bytes and one float out per head.
#include "common.h"

#define QH_THREADS 256

template <typename RawT>
__device__ __forceinline__ float qh_to_f32(RawT v) {
  return sizeof(RawT) == 2 ? __uint_as_float((u32)v << 16) : __uint_as_float((u32)v);
}

// maximum over the 16 lanes of a row, in every lane of the row
__device__ __forceinline__ u32 qh_row_max_dpp(u32 v) {
  v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
  v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
  v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x124, 0xF, 0xF, false));   // row_ror:4
  v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x128, 0xF, 0xF, false));   // row_ror:8
  return v;
}

template <typename RawT>
__device__ __forceinline__ void qh_load8(const RawT* p, float (&x)[8]) {
  if (sizeof(RawT) == 2) {
    const uint4 w = *reinterpret_cast<const uint4*>(p);
    const u32 ww[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      x[2 * e] = __uint_as_float(ww[e] << 16);
      x[2 * e + 1] = __uint_as_float(ww[e] & 0xFFFF0000u);
    }
  } else {
    const float4 a = reinterpret_cast<const float4*>(p)[0], b = reinterpret_cast<const float4*>(p)[1];
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
  }
}

// eight codes of `BITS` bits, code j in bits BITS j .. BITS j + BITS - 1
template <int BITS>
__device__ __forceinline__ u32 qh_codes8(const float (&x)[8], float s) {
  constexpr float QB = (float)((1 << (BITS - 1)) - 1);
  constexpr int OFF = 1 << (BITS - 1);
  u32 v = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float p = fminf(fmaxf(rintf(x[j] * s), -QB), QB);    // one float32 multiply
    v |= (u32)((int)p + OFF) << (BITS * j);
  }
  return v;
}

// One head per row of 16 lanes, lane j holding channels 8 j .. 8 j + 7: D <= 128, D % 8 == 0
// (3 bits: D % 32 == 0, so that the lanes of a quad fill whole words).
template <typename RawT, int BITS>
__global__ __launch_bounds__(QH_THREADS) void quant_heads_row_kernel(
    const RawT* __restrict__ X, int64_t n_heads, int D, float eps, unsigned char* __restrict__ q_out,
    float* __restrict__ scale_out) {
  const int64_t head = (int64_t)blockIdx.x * (QH_THREADS / 16) + (threadIdx.x >> 4);
  if (head >= n_heads) return;                            // whole rows leave together
  const int j = threadIdx.x & 15;
  const bool have = 8 * j < D;
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = 0.0f;
  if (have) qh_load8<RawT>(X + head * D + 8 * j, x);
  u32 mx = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) mx = max(mx, __float_as_uint(x[e]) & 0x7FFFFFFFu);
  mx = qh_row_max_dpp(mx);
  const float gamma = __uint_as_float(mx);
  constexpr float QB = (float)((1 << (BITS - 1)) - 1);
  const float s = QB / (gamma + eps);
  if (j == 0) scale_out[head] = gamma / QB;
  const u32 v = qh_codes8<BITS>(x, s);
  if (BITS == 4) {
    if (have) reinterpret_cast<u32*>(q_out + head * (D / 2))[j] = v;
  } else {
    // four lanes hold 4 x 24 bits = three words: lane jq of the quad builds word jq from its own
    // value and its right neighbour's
    const u32 nxt = (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x39, 0xF, 0xF, false);   // quad_perm [1,2,3,0]
    const int jq = j & 3;
    const u32 word = (v >> (8 * jq)) | (nxt << (24 - 8 * jq));
    if (have && jq < 3) reinterpret_cast<u32*>(q_out + head * (3 * D / 8) + (j >> 2) * 12)[jq] = word;
  }
}

// Any D % 8 == 0 up to BL_MAX_K: one wave per head, groups of 8 channels strided over the lanes,
// the head read twice (statistics, coding), the codes written byte by byte.
template <typename RawT, int BITS>
__global__ __launch_bounds__(QH_THREADS) void quant_heads_wave_kernel(
    const RawT* __restrict__ X, int64_t n_heads, int D, float eps, unsigned char* __restrict__ q_out,
    float* __restrict__ scale_out) {
  const int64_t head = (int64_t)blockIdx.x * (QH_THREADS / 64) + (threadIdx.x >> 6);
  if (head >= n_heads) return;                            // (no barriers in this kernel)
  const int lane = threadIdx.x & 63;
  const RawT* x = X + head * D;
  u32 mx = 0;
  for (int g = lane; g < D / 8; g += 64)
#pragma unroll
    for (int e = 0; e < 8; ++e) mx = max(mx, __float_as_uint(qh_to_f32<RawT>(x[8 * g + e])) & 0x7FFFFFFFu);
  mx = bl_wave_max_u32(mx);
  const float gamma = __uint_as_float(mx);
  constexpr float QB = (float)((1 << (BITS - 1)) - 1);
  const float s = QB / (gamma + eps);
  if (lane == 0) scale_out[head] = gamma / QB;
  unsigned char* out = q_out + head * (BITS * D / 8);
  for (int g = lane; g < D / 8; g += 64) {
    float v8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) v8[e] = qh_to_f32<RawT>(x[8 * g + e]);
    const u32 v = qh_codes8<BITS>(v8, s);
#pragma unroll
    for (int b = 0; b < BITS; ++b) out[BITS * g + b] = (unsigned char)(v >> (8 * b));
  }
}

int bl_launch_quantize_heads(const void* X, bl_dtype dt, int64_t n_heads, int64_t D64, int bits, float eps,
                             void* q, float* scale, hipStream_t s) {
  const int D = (int)D64;
  const bool rows = D <= 128 && (bits == 4 || D % 32 == 0);
  const unsigned grid = (unsigned)((n_heads + (rows ? QH_THREADS / 16 : QH_THREADS / 64) - 1) /
                                   (rows ? QH_THREADS / 16 : QH_THREADS / 64));
#define QH_GO(KERN)                                                                                          \
  do {                                                                                                       \
    if (dt == BL_BF16) {                                                                                     \
      if (bits == 4) KERN<uint16_t, 4><<<grid, QH_THREADS, 0, s>>>((const uint16_t*)X, n_heads, D, eps, (unsigned char*)q, scale); \
      else KERN<uint16_t, 3><<<grid, QH_THREADS, 0, s>>>((const uint16_t*)X, n_heads, D, eps, (unsigned char*)q, scale);           \
    } else {                                                                                                 \
      if (bits == 4) KERN<u32, 4><<<grid, QH_THREADS, 0, s>>>((const u32*)X, n_heads, D, eps, (unsigned char*)q, scale);           \
      else KERN<u32, 3><<<grid, QH_THREADS, 0, s>>>((const u32*)X, n_heads, D, eps, (unsigned char*)q, scale);                     \
    }                                                                                                        \
  } while (0)
  if (rows) QH_GO(quant_heads_row_kernel);
  else QH_GO(quant_heads_wave_kernel);
#undef QH_GO
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

// ---------------------------------------------------------------- reading the codes back
// value = (code - 2^(bits-1)) * scale, one float32 multiply (bfloat16 outputs: one rounding more).
// One thread per group of 8 channels: BITS bytes in, 8 values out.
template <typename OutT, int BITS>
__global__ __launch_bounds__(QH_THREADS) void dequant_heads_kernel(
    const unsigned char* __restrict__ q, const float* __restrict__ scale, int64_t n_groups, int gph,
    OutT* __restrict__ out) {
  const int64_t g = (int64_t)blockIdx.x * QH_THREADS + threadIdx.x;
  if (g >= n_groups) return;
  const float d = scale[g / gph];                          // gph = groups of 8 channels per head
  const unsigned char* p = q + g * BITS;
  u32 v = 0;
#pragma unroll
  for (int b = 0; b < BITS; ++b) v |= (u32)p[b] << (8 * b);
  constexpr int OFF = 1 << (BITS - 1);
  float x[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) x[j] = (float)((int)((v >> (BITS * j)) & ((1u << BITS) - 1u)) - OFF) * d;
  if (sizeof(OutT) == 2) {
    uint4 w;
    w.x = (u32)bl_f32_to_bf16_rne(x[0]) | ((u32)bl_f32_to_bf16_rne(x[1]) << 16);
    w.y = (u32)bl_f32_to_bf16_rne(x[2]) | ((u32)bl_f32_to_bf16_rne(x[3]) << 16);
    w.z = (u32)bl_f32_to_bf16_rne(x[4]) | ((u32)bl_f32_to_bf16_rne(x[5]) << 16);
    w.w = (u32)bl_f32_to_bf16_rne(x[6]) | ((u32)bl_f32_to_bf16_rne(x[7]) << 16);
    reinterpret_cast<uint4*>(out)[g] = w;
  } else {
    reinterpret_cast<float4*>(out)[2 * g] = make_float4(x[0], x[1], x[2], x[3]);
    reinterpret_cast<float4*>(out)[2 * g + 1] = make_float4(x[4], x[5], x[6], x[7]);
  }
}

int bl_launch_dequantize_heads(const void* q, const float* scale, int64_t n_heads, int64_t D, int bits, void* out,
                               bl_dtype odt, hipStream_t s) {
  const int64_t n_groups = n_heads * (D / 8);
  const int64_t blocks = (n_groups + QH_THREADS - 1) / QH_THREADS;
  if (!bl_grid_ok(blocks)) return BL_ESHAPE;
  const int gph = (int)(D / 8);
#define QH_DQ(T, B) dequant_heads_kernel<T, B><<<(unsigned)blocks, QH_THREADS, 0, s>>>((const unsigned char*)q, scale, n_groups, gph, (T*)out)
  if (odt == BL_BF16) { if (bits == 4) QH_DQ(uint16_t, 4); else QH_DQ(uint16_t, 3); }
  else { if (bits == 4) QH_DQ(float, 4); else QH_DQ(float, 3); }
#undef QH_DQ
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}
