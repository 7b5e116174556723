// Per-token activation quantizers of BitNet a4.8:
//   INT4 absmean (eq. 7), Top_k + INT8 absmax (eq. 1, eq. 3), FP4 E2M1 MinMax with one
//   power-of-two scale per 32 channels (eq. 8-9).
// A token is read from HBM once.  INT4: one workgroup per token, the row kept in LDS.  Top_k + INT8:
// the row in registers (four waves per token, or one wave per token for many tokens of moderate
// width; topk_regs.h), optionally formed on the fly as the ReLU^2 GLU product of two rows (eq. 5);
// an LDS-resident kernel for everything the register kernels do not take (float32 rows, index
// lists, very wide rows).  FP4: one thread per block of 32 channels.
#include "common.h"
#include "topk_regs.h"

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
// E3M2 code (sign, 3 exponent bits with bias 3, 2 mantissa bits) of an INT4 level -8..7: every
// level is exact in that format.  Magnitudes 0..8 -> 00, 0C, 10, 12, 14, 15, 16, 17, 18.
__device__ __forceinline__ u32 qa_e3m2_of_level(int q) {
  const unsigned long long lut = 0x00ull | (0x0Cull << 6) | (0x10ull << 12) | (0x12ull << 18) |
                                 (0x14ull << 24) | (0x15ull << 30) | (0x16ull << 36) |
                                 (0x17ull << 42) | (0x18ull << 48);
  const int a = q < 0 ? -q : q;
  return ((u32)(lut >> (6 * a)) & 63u) | (q < 0 ? 32u : 0u);
}

// The same code from the level as a float (an integer value in [-8, 7]): its exponent field minus
// 124 and its top two mantissa bits are the five magnitude bits (the low five bits of bits >> 21,
// with bit 4 flipped), the sign moves from bit 31 to bit 5, and zero of either sign is code 0.
__device__ __forceinline__ u32 qa_e3m2_of_levelf(float p) {
  const u32 b = __float_as_uint(p);
  const u32 c = (((b >> 21) & 31u) ^ 16u) | ((b >> 26) & 32u);
  return (b << 1) != 0u ? c : 0u;
}

// MX6: the same levels, written as E3M2 codes in the tile order of the block-float GEMM (blocks of
// 32 tokens x 128 channels, 3072 bytes; see the format notes of the public header) instead of
// packed nibbles.
// stat: 0 = eq. 7 (beta = mean |x|), 1 = beta = 2 mean |x|, 2 = absmax with 7 levels (ablation
// quantizers of Section 4.3)
template <typename RawT, int VEC, bool MX6>
__global__ __launch_bounds__(QA_THREADS) void quant_int4_kernel(
    const RawT* __restrict__ X, int K, int Kp, float eps, u32* __restrict__ q_out,
    float* __restrict__ scale_out, int32_t* __restrict__ rowsum_out, int stat) {
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
  float beta = (float)(tot / (double)K);
  const float sqrt7 = 2.6457512f;            // float32(sqrt(7)) = 0x402953FD
  float s, d;
  if (stat == 2) {
    // gamma = max |x| (bit patterns of non-negative floats order like integers)
    __shared__ u32 redm[QA_WAVES];
    u32 mx = 0;
    for (int i = threadIdx.x; i < Kp; i += QA_THREADS) mx = max(mx, __float_as_uint(fabsf(qa_to_f32<RawT>(row[i]))));
    mx = bl_wave_max_u32(mx);
    if ((threadIdx.x & 63) == 0) redm[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = 0;
#pragma unroll
    for (int w = 0; w < QA_WAVES; ++w) mx = max(mx, redm[w]);
    const float gamma = __uint_as_float(mx);
    s = 7.0f / (gamma + eps);
    d = gamma / 7.0f;
  } else {
    if (stat == 1) beta = 2.0f * beta;
    s = sqrt7 / (beta + eps);
    d = beta / sqrt7;
  }
  if (threadIdx.x == 0) scale_out[m] = d;

  int sum = 0;
  if (MX6) {
    // one thread per half unit: 16 channels = 96 bits of the unit's 192-bit stream
    unsigned char* blk = reinterpret_cast<unsigned char*>(q_out) + (m >> 5) * (int64_t)(Kp / 128) * 3072;
    const int r = (int)(m & 31);
    for (int h = threadIdx.x; h < Kp / 16; h += QA_THREADS) {
      u32 w3[3] = {0u, 0u, 0u};
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        float p = qa_to_f32<RawT>(row[16 * h + j]) * s;     // one float32 multiply
        p = fminf(fmaxf(rintf(p), -8.0f), 7.0f);
        const int q = (int)p;
        sum += q;
        const u32 c = qa_e3m2_of_level(q);
        const int bit = 6 * j;
        w3[bit >> 5] |= c << (bit & 31);
        if ((bit & 31) > 26) w3[(bit >> 5) + 1] |= c >> (32 - (bit & 31));
      }
      const int kb = h >> 3, u = (h >> 1) & 3;
      unsigned char* b = blk + (int64_t)kb * 3072;
      u32* pp = reinterpret_cast<u32*>(b + r * 64 + ((u ^ ((r >> 2) & 3)) << 4));
      if ((h & 1) == 0) {                                   // stream bytes 0..11
        pp[0] = w3[0]; pp[1] = w3[1]; pp[2] = w3[2];
      } else {                                              // stream bytes 12..15 and 16..23
        pp[3] = w3[0];
        u32* qq = reinterpret_cast<u32*>(b + 2048 + r * 32 + ((u ^ ((r >> 3) & 3)) << 3));
        qq[0] = w3[1]; qq[1] = w3[2];
      }
    }
  }
  u32* out = q_out + m * (int64_t)(Kp / 8);
  for (int w = threadIdx.x; !MX6 && w < Kp / 8; w += QA_THREADS) {
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

// The same quantizer for bfloat16 rows of up to 16384 channels without the trip through LDS: a
// thread keeps its half units (16 channels = two 16-byte loads each; half units tid, tid + 256, ...)
// in registers between the statistics and the coding; one barrier.  K % 8 == 0 by dispatch.
template <bool MX6, int NV>
__global__ __launch_bounds__(QA_THREADS) void quant_int4_regs_kernel(
    const uint16_t* __restrict__ X, int64_t M, int K, int Kp, float eps, u32* __restrict__ q_out,
    float* __restrict__ scale_out, int32_t* __restrict__ rowsum_out, int stat) {
  __shared__ double red[QA_WAVES];
  __shared__ u32 redm[QA_WAVES];
  __shared__ int redi[QA_WAVES];
  // Workgroups go to the eight XCDs in turn.  Tokens that share 128-byte lines of the blocked 6-bit
  // output (neighbours within a block of 32) are given to one XCD, so that its L2 can put the lines
  // together before they go to memory: workgroup 8 j + x works on token x * ceil(M / 8) + j.
  int64_t m = blockIdx.x;
  if (MX6) {
    m = (int64_t)(blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    if (m >= M) return;                          // (whole workgroup, before any barrier)
  }
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint4* xv = reinterpret_cast<const uint4*>(X + m * (int64_t)K);
  const int nv = K >> 3;                         // 16-byte pieces of the row
  uint4 v[NV][2];
#pragma unroll
  for (int j = 0; j < NV; ++j)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int pc = 2 * (tid + QA_THREADS * j) + i;
      v[j][i] = make_uint4(0u, 0u, 0u, 0u);
      if (pc < nv) v[j][i] = xv[pc];
    }
  // statistics: float64 sum of |x| (exact for bfloat16 data), maximum of |x| as a bit pattern
  double acc = 0.0;
  u32 mx = 0;
  if (stat == 2) {                               // (uniform) only the maximum is needed
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const u32 w4[4] = {v[j][i].x, v[j][i].y, v[j][i].z, v[j][i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = max(mx, max((w4[e] << 16) & 0x7FFFFFFFu, w4[e] & 0x7FFF0000u));
      }
    mx = bl_wave_max_u32(mx);
  } else {                                       // only the sum
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const u32 w4[4] = {v[j][i].x, v[j][i].y, v[j][i].z, v[j][i].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          acc += (double)fabsf(__uint_as_float(w4[e] << 16));
          acc += (double)fabsf(__uint_as_float(w4[e] & 0xFFFF0000u));
        }
      }
    acc = bl_wave_sum_f64_dpp(acc);
  }
  if (lane == 0) { red[wave] = acc; redm[wave] = mx; }
  __syncthreads();
  double tot = 0.0;
  u32 gmx = 0;
#pragma unroll
  for (int w = 0; w < QA_WAVES; ++w) { tot += red[w]; gmx = max(gmx, redm[w]); }
  float beta = (float)(tot / (double)K);
  const float sqrt7 = 2.6457512f;            // float32(sqrt(7)) = 0x402953FD
  float s, d;
  if (stat == 2) {
    const float gamma = __uint_as_float(gmx);
    s = 7.0f / (gamma + eps);
    d = gamma / 7.0f;
  } else {
    if (stat == 1) beta = 2.0f * beta;
    s = sqrt7 / (beta + eps);
    d = beta / sqrt7;
  }
  if (tid == 0) scale_out[m] = d;

  int sum = 0;
  unsigned char* blk = reinterpret_cast<unsigned char*>(q_out) + (m >> 5) * (int64_t)(Kp / 128) * 3072;
  const int r = (int)(m & 31);
  u32* out = q_out + m * (int64_t)(Kp / 8);
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int h = tid + QA_THREADS * j;          // half unit: channels 16 h .. 16 h + 15
    if (h < Kp / 16) {
      // The 16 levels as int8 bytes, four to a word.  RoundClip as round(clamp(v)) (the bounds are
      // integers, so this equals clamp(round(v))): one float32 multiply, the clamp, and the rounding as the
      // float32 addition of 1.5 * 2^23 (round to nearest even at integer spacing), whose low byte is the level.
      u32 lv[4];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const u32 w4[4] = {v[j][i].x, v[j][i].y, v[j][i].z, v[j][i].w};
#pragma unroll
        for (int e = 0; e < 4; e += 2) {
          u32 rb[4];
#pragma unroll
          for (int t = 0; t < 2; ++t) {
            const float v0 = __uint_as_float(w4[e + t] << 16) * s;
            const float v1 = __uint_as_float(w4[e + t] & 0xFFFF0000u) * s;
            rb[2 * t] = __float_as_uint(__builtin_amdgcn_fmed3f(v0, -8.0f, 7.0f) + 12582912.0f);
            rb[2 * t + 1] = __float_as_uint(__builtin_amdgcn_fmed3f(v1, -8.0f, 7.0f) + 12582912.0f);
          }
          lv[2 * i + (e >> 1)] = __builtin_amdgcn_perm(rb[1], rb[0], 0x0c0c0400u) | __builtin_amdgcn_perm(rb[3], rb[2], 0x04000c0cu);
        }
      }
      if (rowsum_out) {
#pragma unroll
        for (int c = 0; c < 4; ++c) sum = __builtin_amdgcn_sdot4((int)lv[c], 0x01010101, sum, false);
      }
      if (MX6) {
        // E3M2 codes of four levels at once from two 8-entry byte tables (v_perm as the lookup): levels
        // 0 .. 7 -> 00 0C 10 12 14 15 16 17; levels -8 .. -1, by their low three bits -> 38 37 36 35 34 32 30 2C
        u32 t24[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const u32 sel = lv[c] & 0x07070707u;
          const u32 pos = __builtin_amdgcn_perm(0x17161514u, 0x12100C00u, sel);
          const u32 neg = __builtin_amdgcn_perm(0x2C303234u, 0x35363738u, sel);
          const u32 nm = ((lv[c] >> 7) & 0x01010101u) * 255u;           // bytes of negative levels
          const u32 cd = (neg & nm) | (pos & ~nm);
          // four 6-bit codes in four bytes -> 24 bits
          const u32 pr = ((cd >> 2) & 0x0FC00FC0u) | (cd & 0x003F003Fu);
          t24[c] = (pr & 0xFFFu) | ((pr >> 4) & 0xFFF000u);
        }
        const u32 w3[3] = {t24[0] | (t24[1] << 24), (t24[1] >> 8) | (t24[2] << 16), (t24[2] >> 16) | (t24[3] << 8)};
        const int kb = h >> 3, u = (h >> 1) & 3;
        unsigned char* b = blk + (int64_t)kb * 3072;
        u32* pp = reinterpret_cast<u32*>(b + r * 64 + ((u ^ ((r >> 2) & 3)) << 4));
        if ((h & 1) == 0) {                                   // stream bytes 0..11
          pp[0] = w3[0]; pp[1] = w3[1]; pp[2] = w3[2];
        } else {                                              // stream bytes 12..15 and 16..23
          pp[3] = w3[0];
          u32* qq = reinterpret_cast<u32*>(b + 2048 + r * 32 + ((u ^ ((r >> 3) & 3)) << 3));
          qq[0] = w3[1]; qq[1] = w3[2];
        }
      } else {
        // nibble form: byte b of a word = level b | level 4 + b << 4
#pragma unroll
        for (int g = 0; g < 2; ++g)
          out[2 * h + g] = (lv[2 * g] & 0x0F0F0F0Fu) | ((lv[2 * g + 1] << 4) & 0xF0F0F0F0u);
      }
    }
  }
  if (rowsum_out) {
    sum = bl_wave_sum_i32(sum);
    if (lane == 0) redi[wave] = sum;
    __syncthreads();
    if (tid == 0) {
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

// ---------------------------------------------------------------- Top_k + INT8, keys in registers
// (helpers and the four-wave body: topk_regs.h)
// GLU: 0 = X is the token matrix (bfloat16); 1 / 2 = the tokens are bf16(X2 * max(X, 0)^2) of a gate
// matrix X and an up matrix X2, bfloat16 / float32 (eq. 5 folded into the load)
template <int CPW, int GLU>
__global__ __launch_bounds__(QA_THREADS) void quant_topk_int8_regs_kernel(
    const void* __restrict__ X, const void* __restrict__ X2, int K, int Kp, int topk, float eps,
    u32* __restrict__ q_out, float* __restrict__ scale_out, int32_t* __restrict__ rowsum_out) {
  const int64_t m = blockIdx.x;
  const size_t row = (size_t)m * K * (GLU == 2 ? 4 : 2);
  qa_topk_row_regs<CPW, GLU>(reinterpret_cast<const unsigned char*>(X) + row,
                             GLU ? reinterpret_cast<const unsigned char*>(X2) + row : nullptr, K, Kp, topk, eps,
                             q_out + m * (int64_t)(Kp / 4), scale_out + m, rowsum_out ? rowsum_out + m : nullptr);
}

// Few tokens (decode): what counts is how long one token takes, not how many run at once.  Eight
// waves per token, 11-bit keys and three bits of the threshold per pass (topk_regs.h); codes and
// scales only (the codes are those of the kernels above bit for bit).
template <int CPW>
__global__ __launch_bounds__(512) void quant_topk_int8_regs8_kernel(
    const uint16_t* __restrict__ X, int K, int Kp, int topk, float eps, u32* __restrict__ q_out,
    float* __restrict__ scale_out) {
  __shared__ __align__(16) u32 sh[80];
  const int64_t m = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n_chunks = Kp >> 8;
  const int per_wave = (n_chunks + 7) / 8;
  const int c_begin = min(wave * per_wave, n_chunks);
  const int nc = min(c_begin + per_wave, n_chunks) - c_begin;
  const uint16_t* x = X + m * (int64_t)K;
  u32 raw[CPW][2];
  const int ch0 = c_begin * 256 + lane * 4;
#pragma unroll
  for (int i = 0; i < CPW; ++i) {
    uint2 v = make_uint2(0u, 0u);
    if (i < nc && ch0 + i * 256 < K) v = *reinterpret_cast<const uint2*>(x + ch0 + i * 256);   // K % 4 == 0 by dispatch
    raw[i][0] = v.x;
    raw[i][1] = v.y;
  }
  qa_topk_row_regs8<CPW>(raw, nc, c_begin, topk, eps, q_out + m * (int64_t)(Kp / 4), scale_out + m, sh);
}

// The same selection with one wave per token, for many tokens of moderate width: the fixed cost of a
// pass (wave sum, compare, branch) is paid once per token instead of four times, and there is no LDS
// traffic and no barrier at all.  A lane holds up to 4 * NB chunks' worth of keys (NB blocks of 16
// keys); a workgroup is four tokens.  (Wider rows need too many registers for that: one wave per
// SIMD, or two waves per token, measured slower than the four-wave kernel above.)
template <int NB, int GLU>
__global__ __launch_bounds__(QA_THREADS) void quant_topk_int8_wave_kernel(
    const void* __restrict__ X, const void* __restrict__ X2, int64_t M, int K, int Kp, int topk, float eps,
    u32* __restrict__ q_out, float* __restrict__ scale_out, int32_t* __restrict__ rowsum_out) {
  constexpr int NC = 4 * NB;                              // chunks of 256 channels a lane can hold
  constexpr int NWD = (NB + 1) / 2;                       // mask words: 32 keys each
  const int lane = threadIdx.x & 63;
  const int64_t m = (int64_t)blockIdx.x * QA_WAVES + (threadIdx.x >> 6);
  if (m >= M) return;                                     // (no barriers in this kernel)
  const int nc = Kp / 256;                                // <= NC by dispatch
  constexpr int c_begin = 0;

  // one pass over the row: 4 consecutive channels (8 bytes) per lane and chunk, zero beyond K
  u32 raw[NC][2];
  const size_t row = (size_t)m * K * (GLU == 2 ? 4 : 2);
  const unsigned char* x = reinterpret_cast<const unsigned char*>(X) + row;
  const unsigned char* x2 = GLU ? reinterpret_cast<const unsigned char*>(X2) + row : nullptr;
  const int ch0 = c_begin * 256 + lane * 4;               // (one address per lane, chunks at constant distances)
  const int left = K - ch0;
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    uint2 v = make_uint2(0u, 0u);
    if (i < nc && i * 256 < left) v = qa_token4<GLU>(x, x2, ch0 + i * 256);   // K % 4 == 0 by dispatch
    raw[i][0] = v.x; raw[i][1] = v.y;
  }
  u32 kmax;
  {
    typedef unsigned short us2 __attribute__((ext_vector_type(2)));
    us2 km = __builtin_bit_cast(us2, QA_GUARD);
#pragma unroll
    for (int i = 0; i < NC; ++i)
#pragma unroll
      for (int h = 0; h < 2; ++h) km = __builtin_elementwise_max(km, __builtin_bit_cast(us2, raw[i][h] | QA_GUARD));
    const u32 km2 = __builtin_bit_cast(u32, km);
    kmax = bl_wave_max_u32(max(km2 & 0x7FFFu, (km2 >> 16) & 0x7FFFu));
    kmax = (u32)__builtin_amdgcn_readfirstlane((int)kmax);
  }
  const float gamma = __uint_as_float(kmax << 16);
  const float s = 127.0f / (gamma + eps);
  if (lane == 0) scale_out[m] = gamma / 127.0f;

  // Rows wider than 4096 channels are FFN states, mostly zeros: if no more than topk keys lie above
  // C = kmax - 8 binades, keeping exactly those gives the codes of the exact selection (a key at or
  // below C has code 0 kept or not) and the search is skipped.
  bool early = false;
  if (NB > 4 && kmax > 1024u) {                           // wave-uniform
    const u32 cc = (kmax - 1024u + 1u) * 0x10001u;
    int n_hi = 0;
#pragma unroll
    for (int i = 0; i < NC; ++i)
#pragma unroll
      for (int h = 0; h < 2; ++h) n_hi += __popc(((raw[i][h] | QA_GUARD) - cc) & QA_GUARD);
    early = qa_wave_sum_dpp(n_hi) <= topk;
  }
  u32 act[NWD];
#pragma unroll
  for (int w = 0; w < NWD; ++w) {
    const int nreal = min(max(nc - 8 * w, 0), 8);         // chunks the token does not have stay out
    act[w] = nreal >= 8 ? 0xFFFFFFFFu : ((1u << (4 * nreal)) - 1u);
  }
  u32 tau = early ? kmax - 1024u : 0u;
  int above = 0;
  if (!early) {
    // bit planes of the lane's keys; mask word w covers blocks 2w, 2w+1 = local chunks 8w .. 8w+7,
    // chunk i in bits 4 (i % 8) .. +3, element j of the chunk in bit j of those
    u32 pl[NB][8];
#pragma unroll
    for (int B = 0; B < NB; ++B) {
#pragma unroll
      for (int i = 0; i < 8; ++i) pl[B][i] = raw[4 * B + (i >> 1)][i & 1] & 0x7FFF7FFFu;
      qa_bit_transpose16(pl[B]);
    }
    const int top_bit = 31 - __clz((int)(kmax | 1u));
#pragma unroll
    for (int bit = 14; bit >= 0; --bit) {
      if (bit <= top_bit) {                                 // wave-uniform
        u32 xw[NWD];
        int cnt = 0;
#pragma unroll
        for (int w = 0; w < NWD; ++w) {
          u32 p;
          if (2 * w + 1 < NB)
            p = __builtin_amdgcn_perm(pl[2 * w + 1][bit >> 1], pl[2 * w][bit >> 1], (bit & 1) ? 0x07060302u : 0x05040100u);
          else
            p = (bit & 1) ? pl[2 * w][bit >> 1] >> 16 : pl[2 * w][bit >> 1] & 0xFFFFu;
          xw[w] = act[w] & p;
          cnt += __popc(xw[w]);
        }
        const int total = qa_wave_sum_dpp(cnt);
        if (above + total >= topk) {
          tau |= 1u << bit;
#pragma unroll
          for (int w = 0; w < NWD; ++w) act[w] = xw[w];
        } else {
          above += total;
#pragma unroll
          for (int w = 0; w < NWD; ++w) act[w] ^= xw[w];
        }
      }
    }
  }
  // (nothing of the coding below may be computed ahead of the search: it would double the registers)
#pragma unroll
  for (int i = 0; i < NC; ++i) asm volatile("" : "+v"(raw[i][0]), "+v"(raw[i][1]));

  // act marks the keys equal to tau; of those the first r in channel order are kept
  int eq_total = 0, eq_base = 0;                          // eq_base: keys equal to tau in earlier chunks
#pragma unroll
  for (int w = 0; w < NWD; ++w) eq_total += __popc(act[w]);
  eq_total = qa_wave_sum_dpp(eq_total);
  const int r = topk - above;
  // (keys equal to a tau 8 binades below the row maximum have code 0 kept or not: no prefix search then)
  const bool eq_all = eq_total <= r || tau + 1024u <= kmax;   // wave-uniform
  const u32 t1 = (tau + 1u) * 0x10001u, t0 = tau * 0x10001u;
  const u32 tk = eq_all ? t0 : t1;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  int sum = 0;
  u32* out0 = q_out + m * (int64_t)(Kp / 4) + c_begin * 64 + lane;
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    if (i < nc) {                                         // wave-uniform
      const u32 pg0 = raw[i][0] | QA_GUARD, pg1 = raw[i][1] | QA_GUARD;
      u32 k0 = (pg0 - tk) & QA_GUARD, k1 = (pg1 - tk) & QA_GUARD;   // kept: key >= tau or key > tau
      if (!eq_all && eq_base < r) {                       // wave-uniform
        const u32 eq4 = (act[i >> 3] >> (4 * (i & 7))) & 0xFu;
        if (__ballot(eq4 != 0)) {
          const bool eqf[4] = {(eq4 & 1u) != 0, (eq4 & 2u) != 0, (eq4 & 4u) != 0, (eq4 & 8u) != 0};
          int rank = eq_base, in_chunk = 0;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint64_t b = __ballot(eqf[j]);
            rank += __popcll(b & lt_mask);
            in_chunk += __popcll(b);
          }
          if (eqf[0]) { if (rank < r) k0 |= 0x8000u; ++rank; }
          if (eqf[1]) { if (rank < r) k0 |= 0x80000000u; ++rank; }
          if (eqf[2]) { if (rank < r) k1 |= 0x8000u; ++rank; }
          if (eqf[3]) { if (rank < r) k1 |= 0x80000000u; ++rank; }
          eq_base += in_chunk;
        }
      }
      const float xs[4] = {__uint_as_float(raw[i][0] << 16), __uint_as_float(raw[i][0] & 0xFFFF0000u),
                           __uint_as_float(raw[i][1] << 16), __uint_as_float(raw[i][1] & 0xFFFF0000u)};
      u32 rb[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) rb[j] = __float_as_uint(xs[j] * s + 12582912.0f);
      const u32 w01 = __builtin_amdgcn_perm(rb[1], rb[0], 0x0c0c0400u);   // bytes: rb0.b0, rb1.b0, 0, 0
      const u32 w23 = __builtin_amdgcn_perm(rb[3], rb[2], 0x04000c0cu);   // bytes: 0, 0, rb2.b0, rb3.b0
      const u32 keep4 = (__builtin_amdgcn_perm(k1, k0, 0x07050301u) >> 7) * 255u;
      const u32 word = (w01 | w23) & keep4;
      sum = __builtin_amdgcn_sdot4((int)word, 0x01010101, sum, false);
      out0[i * 64] = word;
    }
  }
  if (rowsum_out) {
    sum = qa_wave_sum_dpp(sum);
    if (lane == 0) rowsum_out[m] = sum;
  }
}

// ---------------------------------------------------------------- FP4 E2M1, block of 32 (eq. 8-9)
// One thread per block of 32 channels.
// MX: codes and scales in the block order of the block-float GEMM (32 tokens x 128 channels per
// block, channels of a unit in natural nibble order) instead of token-major.
// E1M2 = false: E2M1 (top value 6); true: E1M2 (the uniform grid j / 4, top value 1.75; row-major
// nibbles only)
template <typename RawT, bool MX, bool E1M2 = false>
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
  if (sizeof(RawT) == 2 && (K & 31) == 0 && blk * 32 < K) {
    // whole block of a bfloat16 row that is 64-byte aligned: four 16-byte loads
    uint4 w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) w[i] = reinterpret_cast<const uint4*>(x)[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const u32 ww[4] = {w[i].x, w[i].y, w[i].z, w[i].w};
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {
        v[8 * i + 2 * e2] = __uint_as_float(ww[e2] << 16);
        v[8 * i + 2 * e2 + 1] = __uint_as_float(ww[e2] & 0xFFFF0000u);
      }
    }
#pragma unroll
    for (int j = 0; j < 32; ++j) a = fmaxf(a, fabsf(v[j]));
  } else {
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      v[j] = (blk * 32 + j < K) ? qa_to_f32<RawT>(x[j]) : 0.0f;
      a = fmaxf(a, fabsf(v[j]));
    }
  }
  // smallest e with a / 2^e <= 6 = 1.5 * 2^2 (E1M2: <= 1.75 = 1.75 * 2^0)
  int e = 0;
  if (a != 0.0f) {
    const u32 ab = __float_as_uint(a);
    const int be = (int)(ab >> 23);                       // biased exponent (0 for subnormals)
    const u32 mant = ab & 0x7FFFFFu;
    if (E1M2) e = (be - 127) + ((mant <= 0x600000u) ? 0 : 1);
    else e = (be - 127) - ((mant <= 0x400000u) ? 2 : 1);
    if (be == 0) e = -127;                                // subnormal maximum: below the clamp
    e = max(-127, min(127, e));
  }
  // block (m / 32, blk / 4): token row r = m % 32, unit u = blk % 4
  const int64_t mxb = (m >> 5) * (int64_t)(Kp / 128) + (blk >> 2);
  const int r = (int)(m & 31), u = blk & 3;
  if (MX) scale_out[mxb * 128 + r * 4 + u] = (uint8_t)(e + 127);
  else scale_out[m * bpr + blk] = (uint8_t)(e + 127);
  u32 nib[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const float sv = ldexpf(v[j], -e);                    // exact
    const float av = fabsf(sv);
    if (E1M2) {                                           // one step of 1/4 everywhere, av <= 1.75
      const int code = min((int)rintf(av * 4.0f), 7);
      nib[j] = (u32)code | ((sv < 0.0f && code != 0) ? 8u : 0u);
      continue;
    }
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
  if (MX) {
    u32 w4[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 32; ++j) w4[j >> 3] |= nib[j] << (4 * (j & 7));
    unsigned char* dst = reinterpret_cast<unsigned char*>(q_out) + mxb * 2048 + r * 64 + ((u ^ ((r >> 2) & 3)) << 4);
    *reinterpret_cast<uint4*>(dst) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
    return;
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
  } else if (mode == BL_ACT_INT4_ABSMEAN_MX6) {
    // value i of unit u: bits 6 i .. 6 i + 5 of the unit's stream, bytes 0..15 in the P piece and
    // bytes 16..23 in the Q piece of the token's row inside its 32-token block
    const unsigned char* blk = reinterpret_cast<const unsigned char*>(q) +
                               ((m >> 5) * (int64_t)(Kp / 128) + (k >> 7)) * 3072;
    const int r = (int)(m & 31), u = (k >> 5) & 3, bit = 6 * (k & 31);
    const unsigned char* pp = blk + r * 64 + ((u ^ ((r >> 2) & 3)) << 4);
    const unsigned char* qq = blk + 2048 + r * 32 + ((u ^ ((r >> 3) & 3)) << 3);
    u32 two = 0;                                            // the two stream bytes that hold the code
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int byte = (bit >> 3) + j;
      if (byte < 24) two |= (u32)(byte < 16 ? pp[byte] : qq[byte - 16]) << (8 * j);
    }
    const u32 c = (two >> (bit & 7)) & 63u;
    const int e = (int)((c >> 2) & 7u), mant = (int)(c & 3u);
    // levels are integers: 2^(e-3) * (1 + mant/4) for e >= 1, zero otherwise
    const int mag = e == 0 ? 0 : (((4 + mant) << e) >> 5);
    v = (c & 32u) ? -mag : mag;
  } else if (mode == BL_ACT_FP4_E2M1_B32_MX) {
    const unsigned char* blk = reinterpret_cast<const unsigned char*>(q) +
                               ((m >> 5) * (int64_t)(Kp / 128) + (k >> 7)) * 2048;
    const int r = (int)(m & 31), u = (k >> 5) & 3, i = k & 31;
    const unsigned char b = blk[r * 64 + ((u ^ ((r >> 2) & 3)) << 4) + (i >> 1)];
    v = (int)((b >> (4 * (i & 1))) & 15u);
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
  if (mode == BL_ACT_INT4_ABSMEAN || mode == BL_ACT_INT4_ABSMEAN_MX6 || mode == BL_ACT_INT4_ABSMEAN2 ||
      mode == BL_ACT_INT4_ABSMAX) {
    const int stat = mode == BL_ACT_INT4_ABSMEAN2 ? 1 : mode == BL_ACT_INT4_ABSMAX ? 2 : 0;
    // (the limit is raised once, to the widest row the library accepts)
    constexpr int max_smem = BL_MAX_K * (int)sizeof(RawT);
    if (mode == BL_ACT_INT4_ABSMEAN_MX6) {
      BL_SET_MAX_LDS_ONCE((quant_int4_kernel<RawT, VEC, true>), max_smem);
      quant_int4_kernel<RawT, VEC, true><<<(unsigned)M, QA_THREADS, smem, s>>>(X, K, Kp, eps, (u32*)q, (float*)scale, rowsum, stat);
    } else {
      BL_SET_MAX_LDS_ONCE((quant_int4_kernel<RawT, VEC, false>), max_smem);
      quant_int4_kernel<RawT, VEC, false><<<(unsigned)M, QA_THREADS, smem, s>>>(X, K, Kp, eps, (u32*)q, (float*)scale, rowsum, stat);
    }
  } else if (M <= 64) {
    constexpr int max_smem = BL_MAX_K * (int)sizeof(RawT);
    BL_SET_MAX_LDS_ONCE((quant_topk_int8_kernel<RawT, VEC, 1024>), max_smem);
    quant_topk_int8_kernel<RawT, VEC, 1024><<<(unsigned)M, 1024, smem, s>>>(X, K, Kp, topk, eps, (u32*)q, (float*)scale, rowsum, sel);
  } else {
    constexpr int max_smem = BL_MAX_K * (int)sizeof(RawT);
    BL_SET_MAX_LDS_ONCE((quant_topk_int8_kernel<RawT, VEC, QA_THREADS>), max_smem);
    quant_topk_int8_kernel<RawT, VEC, QA_THREADS><<<(unsigned)M, QA_THREADS, smem, s>>>(X, K, Kp, topk, eps, (u32*)q, (float*)scale, rowsum, sel);
  }
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

// Top_k + INT8 with the keys in registers, one memory pass (K % 4 == 0, Kp <= 12288).
template <int GLU>
static int qa_run_topk_regs(const void* x, const void* x2, int64_t M, int K, int Kp, int topk, float eps,
                            void* q, void* scale, int32_t* rowsum, hipStream_t s) {
  const int cpw = (Kp / 256 + QA_WAVES - 1) / QA_WAVES;
  // many tokens of up to 6144 channels: one wave per token (measured at 16384 tokens: 0.051 against
  // 0.075 ms at 4096 channels, 0.077 against 0.110 ms at 5460; from 8 register blocks on it loses)
  const int nb = (Kp / 256 + 3) / 4;
  if (GLU == 0 && rowsum == nullptr && M <= 256) {
    // (K % 4 == 0 and Kp <= 12288 by dispatch: at most 6 chunks of 256 channels per wave)
    if (Kp <= 8192)
      quant_topk_int8_regs8_kernel<4><<<(unsigned)M, 512, 0, s>>>((const uint16_t*)x, K, Kp, topk, eps, (u32*)q, (float*)scale);
    else
      quant_topk_int8_regs8_kernel<8><<<(unsigned)M, 512, 0, s>>>((const uint16_t*)x, K, Kp, topk, eps, (u32*)q, (float*)scale);
  } else if (M >= 2048 && nb <= 6) {
    const unsigned grid = (unsigned)((M + QA_WAVES - 1) / QA_WAVES);
    if (nb <= 4)
      quant_topk_int8_wave_kernel<4, GLU><<<grid, QA_THREADS, 0, s>>>(x, x2, M, K, Kp, topk, eps, (u32*)q, (float*)scale, rowsum);
    else
      quant_topk_int8_wave_kernel<6, GLU><<<grid, QA_THREADS, 0, s>>>(x, x2, M, K, Kp, topk, eps, (u32*)q, (float*)scale, rowsum);
  } else if (cpw <= 4) {
    quant_topk_int8_regs_kernel<4, GLU><<<(unsigned)M, QA_THREADS, 0, s>>>(x, x2, K, Kp, topk, eps, (u32*)q, (float*)scale, rowsum);
  } else if (cpw <= 8) {
    quant_topk_int8_regs_kernel<8, GLU><<<(unsigned)M, QA_THREADS, 0, s>>>(x, x2, K, Kp, topk, eps, (u32*)q, (float*)scale, rowsum);
  } else {
    quant_topk_int8_regs_kernel<12, GLU><<<(unsigned)M, QA_THREADS, 0, s>>>(x, x2, K, Kp, topk, eps, (u32*)q, (float*)scale, rowsum);
  }
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

// eq. 5 + eq. 1 + eq. 3 in one pass: the tokens are bf16(U * max(G, 0)^2)
int bl_launch_quantize_glu(const void* G, const void* U, bl_dtype dt, int64_t M, int64_t K64, int64_t topk,
                           float eps, void* q, void* scale, int32_t* rowsum, hipStream_t s) {
  const int K = (int)K64, Kp = (int)bl_round_up(K64, BL_KPAD);
  if (K % 4 != 0 || Kp > 12288) return BL_EUNSUPPORTED;
  return dt == BL_BF16 ? qa_run_topk_regs<1>(G, U, M, K, Kp, (int)topk, eps, q, scale, rowsum, s)
                       : qa_run_topk_regs<2>(G, U, M, K, Kp, (int)topk, eps, q, scale, rowsum, s);
}

int bl_launch_quantize(const void* X, bl_dtype dt, int64_t M, int64_t K64, bl_act_mode mode,
                       int64_t topk, float eps, void* q, void* scale, int32_t* rowsum,
                       int32_t* sel_idx, hipStream_t s) {
  const int K = (int)K64, Kp = (int)bl_round_up(K64, BL_KPAD);
  if (mode == BL_ACT_FP4_E2M1_B32 || mode == BL_ACT_FP4_E2M1_B32_MX || mode == BL_ACT_FP4_E1M2_B32) {
    const int64_t n = M * (Kp / 32);
    const unsigned blocks = (unsigned)((n + QA_THREADS - 1) / QA_THREADS);
    const bool mx = mode == BL_ACT_FP4_E2M1_B32_MX;
    if (mode == BL_ACT_FP4_E1M2_B32) {
      if (dt == BL_BF16) quant_fp4_kernel<uint16_t, false, true><<<blocks, QA_THREADS, 0, s>>>((const uint16_t*)X, M, K, Kp, (u32*)q, (uint8_t*)scale);
      else quant_fp4_kernel<u32, false, true><<<blocks, QA_THREADS, 0, s>>>((const u32*)X, M, K, Kp, (u32*)q, (uint8_t*)scale);
    } else if (dt == BL_BF16) {
      if (mx) quant_fp4_kernel<uint16_t, true><<<blocks, QA_THREADS, 0, s>>>((const uint16_t*)X, M, K, Kp, (u32*)q, (uint8_t*)scale);
      else quant_fp4_kernel<uint16_t, false><<<blocks, QA_THREADS, 0, s>>>((const uint16_t*)X, M, K, Kp, (u32*)q, (uint8_t*)scale);
    } else {
      if (mx) quant_fp4_kernel<u32, true><<<blocks, QA_THREADS, 0, s>>>((const u32*)X, M, K, Kp, (u32*)q, (uint8_t*)scale);
      else quant_fp4_kernel<u32, false><<<blocks, QA_THREADS, 0, s>>>((const u32*)X, M, K, Kp, (u32*)q, (uint8_t*)scale);
    }
    BL_HIP_CHECK_LAUNCH();
    return BL_OK;
  }
  if (dt == BL_BF16 && mode == BL_ACT_TOPK_INT8_ABSMAX && K % 4 == 0 && Kp <= 12288 &&
      sel_idx == nullptr)
    return qa_run_topk_regs<0>(X, nullptr, M, K, Kp, (int)topk, eps, q, scale, rowsum, s);
  const bool int4_any = mode == BL_ACT_INT4_ABSMEAN || mode == BL_ACT_INT4_ABSMEAN_MX6 ||
                        mode == BL_ACT_INT4_ABSMEAN2 || mode == BL_ACT_INT4_ABSMAX;
  if (dt == BL_BF16 && int4_any && K % 8 == 0 && Kp <= 16384) {
    // rows in registers, no LDS staging
    const int stat = mode == BL_ACT_INT4_ABSMEAN2 ? 1 : mode == BL_ACT_INT4_ABSMAX ? 2 : 0;
    const bool mx6 = mode == BL_ACT_INT4_ABSMEAN_MX6;
    const int nvv = (Kp / 16 + QA_THREADS - 1) / QA_THREADS;      // half units per thread: 1 .. 4
    const unsigned grid = mx6 ? (unsigned)((M + 7) / 8 * 8) : (unsigned)M;   // MX6: a multiple of 8
#define QA_I4(MX, NVV) quant_int4_regs_kernel<MX, NVV><<<grid, QA_THREADS, 0, s>>>((const uint16_t*)X, M, K, Kp, eps, (u32*)q, (float*)scale, rowsum, stat)
    if (mx6) { if (nvv <= 1) QA_I4(true, 1); else if (nvv <= 2) QA_I4(true, 2); else QA_I4(true, 4); }
    else { if (nvv <= 1) QA_I4(false, 1); else if (nvv <= 2) QA_I4(false, 2); else QA_I4(false, 4); }
#undef QA_I4
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
