// Per-token activation quantizers of BitNet a4.8:
//   INT4 absmean (eq. 7), Top_k + INT8 absmax (eq. 1, eq. 3), FP4 E2M1 MinMax with one
//   power-of-two scale per 32 channels (eq. 8-9).
// One workgroup handles one token: the row is read from HBM once, kept in LDS, and every
// later pass (statistics, selection, coding) runs out of LDS.
#include "common.h"

#define QA_THREADS 256
#define QA_WAVES (QA_THREADS / BL_WAVE)

// ---------------------------------------------------------------- raw element access
// Rows are handled as raw bit patterns: uint16_t = bfloat16, u32 = float32.
template <typename RawT> __device__ __forceinline__ float qa_to_f32(RawT r);
template <> __device__ __forceinline__ float qa_to_f32<uint16_t>(uint16_t r) { return bl_bf16_to_f32(r); }
template <> __device__ __forceinline__ float qa_to_f32<u32>(u32 r) { return __uint_as_float(r); }

template <typename RawT, int VEC> struct QaVec;
template <> struct QaVec<uint16_t, 8> { typedef uint4 type; };
template <> struct QaVec<uint16_t, 4> { typedef uint2 type; };
template <> struct QaVec<uint16_t, 1> { typedef uint16_t type; };
template <> struct QaVec<u32, 4> { typedef uint4 type; };
template <> struct QaVec<u32, 1> { typedef u32 type; };

// Copy one row of K raw elements from global memory into LDS (zero padded to Kp), VEC
// elements per load.  The row start must be aligned to VEC elements.
template <typename RawT, int VEC, int NT = QA_THREADS>
__device__ __forceinline__ void qa_stage_row(const RawT* __restrict__ x, int K, int Kp,
                                             RawT* __restrict__ row) {
  typedef typename QaVec<RawT, VEC>::type V;
  const V* xv = reinterpret_cast<const V*>(x);
  V* rv = reinterpret_cast<V*>(row);
  const int nv = K / VEC;                  // K % VEC == 0 by dispatch
  for (int i = threadIdx.x; i < nv; i += NT) rv[i] = xv[i];
  for (int i = K + threadIdx.x; i < Kp; i += NT) row[i] = (RawT)0;
}

// ---------------------------------------------------------------- INT4 absmean (eq. 7)
template <typename RawT, int VEC>
__global__ __launch_bounds__(QA_THREADS) void quant_int4_kernel(
    const RawT* __restrict__ X, int K, int Kp, float eps, u32* __restrict__ q_out,
    float* __restrict__ scale_out, int32_t* __restrict__ rowsum_out) {
  extern __shared__ __align__(16) unsigned char qa_smem[];
  RawT* row = reinterpret_cast<RawT*>(qa_smem);
  __shared__ double red[QA_WAVES];
  __shared__ int redi[QA_WAVES];
  const int64_t m = blockIdx.x;
  qa_stage_row<RawT, VEC>(X + m * (int64_t)K, K, Kp, row);
  __syncthreads();

  // beta = mean|x|: float64 sum (exact for bf16 data of any sane range), one rounding.
  double acc = 0.0;
  for (int i = threadIdx.x; i < Kp; i += QA_THREADS) acc += (double)fabsf(qa_to_f32<RawT>(row[i]));
  acc = bl_wave_sum_f64(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  double tot = 0.0;
#pragma unroll
  for (int w = 0; w < QA_WAVES; ++w) tot += red[w];
  const float beta = (float)(tot / (double)K);
  const float sqrt7 = 2.6457512f;            // float32(sqrt(7)) = 0x402953FD
  const float s = sqrt7 / (beta + eps);
  if (threadIdx.x == 0) scale_out[m] = beta / sqrt7;

  int sum = 0;
  u32* out = q_out + m * (int64_t)(Kp / 8);
  for (int w = threadIdx.x; w < Kp / 8; w += QA_THREADS) {
    int q[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float p = qa_to_f32<RawT>(row[8 * w + j]) * s;       // one float32 multiply
      p = fminf(fmaxf(rintf(p), -8.0f), 7.0f);
      q[j] = (int)p;
      sum += q[j];
    }
    u32 word = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b)
      word |= (((u32)q[b] & 15u) | (((u32)q[4 + b] & 15u) << 4)) << (8 * b);
    out[w] = word;
  }
  if (rowsum_out) {
    sum = bl_wave_sum_i32(sum);
    if ((threadIdx.x & 63) == 0) redi[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
      int t = 0;
      for (int w = 0; w < QA_WAVES; ++w) t += redi[w];
      rowsum_out[m] = t;
    }
  }
}

// ---------------------------------------------------------------- Top_k + INT8 absmax (eq. 1, 3)
// Selection key = bit pattern of |x| (monotone for finite values, -0 equals +0).  The k-th
// largest key tau is built bit by bit: a bit stays set if at least topk keys are >= the
// candidate.  Keys above tau are kept; among keys equal to tau the first r in channel order
// are kept, r = topk - #(key > tau).  Each wave owns a contiguous range of 256-element
// chunks, a lane owns 4 consecutive channels of a chunk, so channel order is
// (wave, chunk, lane, j) order and ranks come from ballots.
template <typename RawT> struct QaKey;
template <> struct QaKey<uint16_t> { static constexpr u32 mask = 0x7FFFu; static constexpr int bits = 15; };
template <> struct QaKey<u32> { static constexpr u32 mask = 0x7FFFFFFFu; static constexpr int bits = 31; };

template <typename RawT>
__device__ __forceinline__ void qa_load4(const RawT* row, int idx, u32 (&raw)[4]);
template <> __device__ __forceinline__ void qa_load4<uint16_t>(const uint16_t* row, int idx, u32 (&raw)[4]) {
  const uint2 v = *reinterpret_cast<const uint2*>(row + idx);
  raw[0] = v.x & 0xFFFFu; raw[1] = v.x >> 16; raw[2] = v.y & 0xFFFFu; raw[3] = v.y >> 16;
}
template <> __device__ __forceinline__ void qa_load4<u32>(const u32* row, int idx, u32 (&raw)[4]) {
  const uint4 v = *reinterpret_cast<const uint4*>(row + idx);
  raw[0] = v.x; raw[1] = v.y; raw[2] = v.z; raw[3] = v.w;
}

// NT threads per token: 256 when there are many tokens (several workgroups per CU), 1024 for
// decode-sized inputs, where the latency of one token's passes is what counts.
template <typename RawT, int VEC, int NT>
__global__ __launch_bounds__(NT) void quant_topk_int8_kernel(
    const RawT* __restrict__ X, int K, int Kp, int topk, float eps, u32* __restrict__ q_out,
    float* __restrict__ scale_out, int32_t* __restrict__ rowsum_out,
    int32_t* __restrict__ sel_idx_out) {
  constexpr int NW = NT / 64;
  extern __shared__ __align__(16) unsigned char qa_smem[];
  RawT* row = reinterpret_cast<RawT*>(qa_smem);
  __shared__ u32 sh_a[2][NW];
  __shared__ u32 sh_b[NW];
  __shared__ u32 sh_c[NW];
  constexpr u32 KMASK = QaKey<RawT>::mask;
  const int64_t m = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  qa_stage_row<RawT, VEC, NT>(X + m * (int64_t)K, K, Kp, row);
  __syncthreads();

  const int n_chunks = Kp / 256;
  const int per_wave = (n_chunks + NW - 1) / NW;
  const int c_begin = min(wave * per_wave, n_chunks), c_end = min(c_begin + per_wave, n_chunks);

  // gamma = max|x| (as a key)
  u32 kmax = 0;
  for (int c = c_begin; c < c_end; ++c) {
    u32 raw[4];
    qa_load4<RawT>(row, c * 256 + lane * 4, raw);
#pragma unroll
    for (int j = 0; j < 4; ++j) kmax = max(kmax, raw[j] & KMASK);
  }
  kmax = bl_wave_max_u32(kmax);
  if (lane == 0) sh_b[wave] = kmax;
  __syncthreads();
  kmax = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) kmax = max(kmax, sh_b[w]);
  const float gamma = sizeof(RawT) == 2 ? __uint_as_float(kmax << 16) : __uint_as_float(kmax);
  const float s = 127.0f / (gamma + eps);
  if (threadIdx.x == 0) scale_out[m] = gamma / 127.0f;

  // tau = topk-th largest key
  u32 tau = 0;
  int pass = 0;
  for (int bit = 31 - __clz((int)(kmax | 1u)); bit >= 0; --bit, ++pass) {
    const u32 cand = tau | (1u << bit);
    int cnt = 0;                          // wave-uniform: ballots, no cross-lane reduction
    for (int c = c_begin; c < c_end; ++c) {
      u32 raw[4];
      qa_load4<RawT>(row, c * 256 + lane * 4, raw);
#pragma unroll
      for (int j = 0; j < 4; ++j) cnt += __popcll(__ballot((raw[j] & KMASK) >= cand));
    }
    if (lane == 0) sh_a[pass & 1][wave] = (u32)cnt;
    __syncthreads();                      // one barrier per pass: slots alternate
    u32 total = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) total += sh_a[pass & 1][w];
    if (total >= (u32)topk) tau = cand;
  }

  // per-wave counts of keys above and equal to tau
  {
    int gt = 0, eq = 0;                   // wave-uniform
    for (int c = c_begin; c < c_end; ++c) {
      u32 raw[4];
      qa_load4<RawT>(row, c * 256 + lane * 4, raw);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const u32 key = raw[j] & KMASK;
        gt += __popcll(__ballot(key > tau));
        eq += __popcll(__ballot(key == tau));
      }
    }
    __syncthreads();                      // sh_b was read above by every thread
    if (lane == 0) { sh_b[wave] = (u32)gt; sh_c[wave] = (u32)eq; }
    __syncthreads();
  }
  int total_gt = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) total_gt += (int)sh_b[w];
  const int r = topk - total_gt;          // >= 1: how many keys equal to tau are kept
  int eq_base = 0, idx_base = 0;          // equal keys / kept channels before this wave
  for (int w = 0; w < wave; ++w) {
    const int eqw = (int)sh_c[w];
    idx_base += (int)sh_b[w] + max(0, min(r - eq_base, eqw));
    eq_base += eqw;
  }

  // codes
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  int sum = 0;
  u32* out = q_out + m * (int64_t)(Kp / 4);
  int32_t* sel = sel_idx_out ? sel_idx_out + m * (int64_t)topk : nullptr;
  for (int c = c_begin; c < c_end; ++c) {
    u32 raw[4];
    qa_load4<RawT>(row, c * 256 + lane * 4, raw);
    bool keep[4], eqf[4];
    uint64_t any_eq = 0;
    uint64_t beq[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const u32 key = raw[j] & KMASK;
      keep[j] = key > tau;
      eqf[j] = key == tau;
      beq[j] = __ballot(eqf[j]);
      any_eq |= beq[j];
    }
    if (any_eq) {                          // wave-uniform
      int before = 0, in_chunk = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        before += __popcll(beq[j] & lt_mask);
        in_chunk += __popcll(beq[j]);
      }
      int rank = eq_base + before;         // equal keys in lower channels
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (eqf[j]) { keep[j] = rank < r; ++rank; }
      }
      eq_base += in_chunk;
    }
    u32 word = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float p = qa_to_f32<RawT>((RawT)raw[j]) * s;          // one float32 multiply
      p = fminf(fmaxf(rintf(p), -128.0f), 127.0f);
      const int q = keep[j] ? (int)p : 0;
      sum += q;
      word |= ((u32)q & 255u) << (8 * j);
    }
    out[c * 64 + lane] = word;
    if (sel) {                             // ascending channel list of the mask
      uint64_t bk[4];
      int before = 0, in_chunk = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        bk[j] = __ballot(keep[j]);
        before += __popcll(bk[j] & lt_mask);
        in_chunk += __popcll(bk[j]);
      }
      int pos = idx_base + before;
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (keep[j] && pos < topk) sel[pos++] = c * 256 + lane * 4 + j;
      idx_base += in_chunk;
    }
  }
  if (rowsum_out) {
    sum = bl_wave_sum_i32(sum);
    __syncthreads();
    if (lane == 0) sh_a[0][wave] = (u32)sum;
    __syncthreads();
    if (threadIdx.x == 0) {
      int t = 0;
      for (int w = 0; w < NW; ++w) t += (int)sh_a[0][w];
      rowsum_out[m] = t;
    }
  }
}

// ---------------------------------------------------------------- FP4 E2M1, block of 32 (eq. 8-9)
// One thread per block of 32 channels.
template <typename RawT>
__global__ __launch_bounds__(QA_THREADS) void quant_fp4_kernel(
    const RawT* __restrict__ X, int64_t M, int K, int Kp, u32* __restrict__ q_out,
    uint8_t* __restrict__ scale_out) {
  const int bpr = Kp / 32;
  const int64_t id = (int64_t)blockIdx.x * QA_THREADS + threadIdx.x;
  if (id >= M * bpr) return;
  const int64_t m = id / bpr;
  const int blk = (int)(id % bpr);
  const RawT* x = X + m * (int64_t)K + blk * 32;
  float v[32];
  float a = 0.0f;
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    v[j] = (blk * 32 + j < K) ? qa_to_f32<RawT>(x[j]) : 0.0f;
    a = fmaxf(a, fabsf(v[j]));
  }
  // smallest e with a / 2^e <= 6 = 1.5 * 2^2
  int e = 0;
  if (a != 0.0f) {
    const u32 ab = __float_as_uint(a);
    const int be = (int)(ab >> 23);                       // biased exponent (0 for subnormals)
    const u32 mant = ab & 0x7FFFFFu;
    e = (be - 127) - ((mant <= 0x400000u) ? 2 : 1);
    if (be == 0) e = -127;                                // subnormal maximum: below the clamp
    e = max(-127, min(127, e));
  }
  scale_out[m * bpr + blk] = (uint8_t)(e + 127);
  u32 nib[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const float sv = ldexpf(v[j], -e);                    // exact
    const float av = fabsf(sv);
    float r;
    if (av < 2.0f) r = rintf(av * 2.0f) * 0.5f;
    else if (av < 4.0f) r = rintf(av);
    else r = rintf(av * 0.5f) * 2.0f;
    r = fminf(r, 6.0f);
    int code;
    if (r < 2.0f) code = (int)(r * 2.0f);
    else if (r < 4.0f) code = (int)r + 2;
    else code = (int)(r * 0.5f) + 4;
    nib[j] = (u32)code | ((sv < 0.0f && code != 0) ? 8u : 0u);
  }
  u32* out = q_out + m * (int64_t)(Kp / 8) + blk * 4;
#pragma unroll
  for (int h = 0; h < 2; ++h) {                           // two groups of 16 channels
    u32 w0 = 0, w1 = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int kk = 8 * (j & 1) + (j >> 1);
      w0 |= nib[16 * h + kk] << (4 * j);
      w1 |= nib[16 * h + 4 + kk] << (4 * j);
    }
    out[2 * h] = w0;
    out[2 * h + 1] = w1;
  }
}

// ---------------------------------------------------------------- format helper
__global__ __launch_bounds__(QA_THREADS) void unpack_act_kernel(const u32* __restrict__ q, int mode,
                                                                int64_t M, int K, int Kp,
                                                                int8_t* __restrict__ codes) {
  const int64_t id = (int64_t)blockIdx.x * QA_THREADS + threadIdx.x;
  if (id >= M * K) return;
  const int64_t m = id / K;
  const int k = (int)(id % K);
  int v;
  if (mode == BL_ACT_INT4_ABSMEAN) {
    const u32 word = q[m * (Kp / 8) + (k >> 3)];
    const int kk = k & 7;
    const u32 nibv = (word >> (8 * (kk & 3) + 4 * (kk >> 2))) & 15u;
    v = (int)(nibv << 28) >> 28;
  } else if (mode == BL_ACT_TOPK_INT8_ABSMAX) {
    const u32 word = q[m * (Kp / 4) + (k >> 2)];
    v = (int)(int8_t)((word >> (8 * (k & 3))) & 255u);
  } else {
    const int kk = k & 15;
    const int wsel = (kk >> 2) & 1;
    const int base = kk - 4 * wsel;                       // 0..3 or 8..11
    const int j = 2 * (base & 7) + (base >> 3);
    const u32 word = q[m * (Kp / 8) + (k >> 4) * 2 + wsel];
    v = (int)((word >> (4 * j)) & 15u);
  }
  codes[id] = (int8_t)v;
}

// ---------------------------------------------------------------- dispatch
template <typename RawT, int VEC>
static int qa_run_row_kernels(const RawT* X, int64_t M, int K, int Kp, bl_act_mode mode, int topk,
                              float eps, void* q, void* scale, int32_t* rowsum, int32_t* sel,
                              hipStream_t s) {
  const size_t smem = (size_t)Kp * sizeof(RawT);
  if (mode == BL_ACT_INT4_ABSMEAN) {
    auto kern = quant_int4_kernel<RawT, VEC>;
    if (smem > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return BL_EHIP;
    kern<<<(unsigned)M, QA_THREADS, smem, s>>>(X, K, Kp, eps, (u32*)q, (float*)scale, rowsum);
  } else if (M <= 64) {
    auto kern = quant_topk_int8_kernel<RawT, VEC, 1024>;
    if (smem > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return BL_EHIP;
    kern<<<(unsigned)M, 1024, smem, s>>>(X, K, Kp, topk, eps, (u32*)q, (float*)scale, rowsum, sel);
  } else {
    auto kern = quant_topk_int8_kernel<RawT, VEC, QA_THREADS>;
    if (smem > 48 * 1024 &&
        hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess)
      return BL_EHIP;
    kern<<<(unsigned)M, QA_THREADS, smem, s>>>(X, K, Kp, topk, eps, (u32*)q, (float*)scale, rowsum, sel);
  }
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

int bl_launch_quantize(const void* X, bl_dtype dt, int64_t M, int64_t K64, bl_act_mode mode,
                       int64_t topk, float eps, void* q, void* scale, int32_t* rowsum,
                       int32_t* sel_idx, hipStream_t s) {
  const int K = (int)K64, Kp = (int)bl_round_up(K64, BL_KPAD);
  if (mode == BL_ACT_FP4_E2M1_B32) {
    const int64_t n = M * (Kp / 32);
    const int64_t blocks = (n + QA_THREADS - 1) / QA_THREADS;
    if (dt == BL_BF16)
      quant_fp4_kernel<uint16_t><<<(unsigned)blocks, QA_THREADS, 0, s>>>((const uint16_t*)X, M, K, Kp, (u32*)q, (uint8_t*)scale);
    else
      quant_fp4_kernel<u32><<<(unsigned)blocks, QA_THREADS, 0, s>>>((const u32*)X, M, K, Kp, (u32*)q, (uint8_t*)scale);
    BL_HIP_CHECK_LAUNCH();
    return BL_OK;
  }
  if (dt == BL_BF16) {
    const uint16_t* x = (const uint16_t*)X;
    if (K % 8 == 0) return qa_run_row_kernels<uint16_t, 8>(x, M, K, Kp, mode, (int)topk, eps, q, scale, rowsum, sel_idx, s);
    if (K % 4 == 0) return qa_run_row_kernels<uint16_t, 4>(x, M, K, Kp, mode, (int)topk, eps, q, scale, rowsum, sel_idx, s);
    return qa_run_row_kernels<uint16_t, 1>(x, M, K, Kp, mode, (int)topk, eps, q, scale, rowsum, sel_idx, s);
  }
  const u32* x = (const u32*)X;
  if (K % 4 == 0) return qa_run_row_kernels<u32, 4>(x, M, K, Kp, mode, (int)topk, eps, q, scale, rowsum, sel_idx, s);
  return qa_run_row_kernels<u32, 1>(x, M, K, Kp, mode, (int)topk, eps, q, scale, rowsum, sel_idx, s);
}

int bl_launch_unpack_act(const void* q, bl_act_mode mode, int64_t M, int64_t K, int8_t* codes,
                         hipStream_t s) {
  const int64_t blocks = (M * K + QA_THREADS - 1) / QA_THREADS;
  unpack_act_kernel<<<(unsigned)blocks, QA_THREADS, 0, s>>>((const u32*)q, (int)mode, M, (int)K,
                                                           (int)bl_round_up(K, BL_KPAD), codes);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}
