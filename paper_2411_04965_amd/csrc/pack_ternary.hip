// Absmean ternarisation of a latent weight matrix and 2-bit packing (eq. 2 of the paper):
//   alpha = mean|W|,  T = RoundClip(W / (alpha + eps), -1, 1).
// Two kernels: a float64 partial-sum reduction of |W|, then ternarise + pack.  Every block of
// the second kernel re-adds the partial sums in one fixed order, so alpha is identical in all
// blocks and from run to run.
#include "common.h"

#define PT_THREADS 256
#define PT_MAX_PARTIALS 1024

template <typename T> __device__ __forceinline__ float pt_load(const T* p, int64_t i);
template <> __device__ __forceinline__ float pt_load<float>(const float* p, int64_t i) { return p[i]; }
template <> __device__ __forceinline__ float pt_load<uint16_t>(const uint16_t* p, int64_t i) {
  return bl_bf16_to_f32(p[i]);
}

template <typename T>
__global__ __launch_bounds__(PT_THREADS) void abs_sum_partial_kernel(const T* __restrict__ W,
                                                                     int64_t n,
                                                                     double* __restrict__ partial) {
  __shared__ double red[PT_THREADS / BL_WAVE];
  double acc = 0.0;
  for (int64_t i = (int64_t)blockIdx.x * PT_THREADS + threadIdx.x; i < n;
       i += (int64_t)gridDim.x * PT_THREADS)
    acc += (double)fabsf(pt_load<T>(W, i));
  acc = bl_wave_sum_f64(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int w = 0; w < PT_THREADS / BL_WAVE; ++w) s += red[w];
    partial[blockIdx.x] = s;
  }
}

// alpha from the partial sums, same order in every block.
__device__ __forceinline__ float pt_alpha(const double* __restrict__ partial, int n_partial,
                                          int64_t n_elem, double* red) {
  double acc = 0.0;
  for (int i = threadIdx.x; i < n_partial; i += PT_THREADS) acc += partial[i];
  acc = bl_wave_sum_f64(acc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
  __syncthreads();
  double s = 0.0;
  for (int w = 0; w < PT_THREADS / BL_WAVE; ++w) s += red[w];
  return (float)(s / (double)n_elem);
}

__device__ __forceinline__ u32 pt_code(float w, float t) {
  float r = rintf(w / t);                 // IEEE divide, round half to even
  r = fminf(fmaxf(r, -1.0f), 1.0f);
  int c = (int)r;                          // -1, 0, 1
  return (u32)c & 3u;                      // two's complement 2-bit: 00, 01, 11
}

// One thread per 32-bit word of the tiled GEMM layout: output channel n, 16 input channels.
template <typename T>
__global__ __launch_bounds__(PT_THREADS) void ternarize_pack_gemm_kernel(
    const T* __restrict__ W, int64_t N, int64_t K, int64_t Kp, float eps,
    const double* __restrict__ partial, int n_partial, u32* __restrict__ out,
    float* __restrict__ alpha_out, int64_t n_words) {
  __shared__ double red[PT_THREADS / BL_WAVE];
  const float alpha = pt_alpha(partial, n_partial, N * K, red);
  if (blockIdx.x == 0 && threadIdx.x == 0) alpha_out[0] = alpha;
  const float t = alpha + eps;
  const int64_t w = (int64_t)blockIdx.x * PT_THREADS + threadIdx.x;
  if (w >= n_words) return;
  const int64_t tile = w >> 8;              // 256 words per 1 KB tile
  const int in_tile = (int)(w & 255);
  const int word_t = in_tile & 3;
  const int i = (in_tile >> 2) & 15;
  const int g = in_tile >> 6;
  const int64_t k_tiles = Kp / 256;
  const int64_t nt = tile / k_tiles, kt = tile % k_tiles;
  const int64_t n = nt * 16 + i;
  const int64_t k0 = kt * 256 + g * 64 + word_t * 16;
  u32 word = 0;
  if (n < N) {
#pragma unroll
    for (int f = 0; f < 16; ++f) {
      const int64_t k = k0 + 4 * (f & 3) + (f >> 2);
      if (k < K) word |= pt_code(pt_load<T>(W, n * K + k), t) << (2 * f);
    }
  }
  out[w] = word;
}

// One thread per 32-bit word of the input-channel-major layout (column blocks of 512 outputs,
// 128 bytes per channel and block): channel k, 16 outputs.  Consecutive threads take
// consecutive k so that reads of W are coalesced.
template <typename T>
__global__ __launch_bounds__(PT_THREADS) void ternarize_pack_kmajor_kernel(
    const T* __restrict__ W, int64_t N, int64_t K, int64_t Np, float eps,
    const double* __restrict__ partial, int n_partial, u32* __restrict__ out,
    float* __restrict__ alpha_out, int64_t n_words) {
  __shared__ double red[PT_THREADS / BL_WAVE];
  const float alpha = pt_alpha(partial, n_partial, N * K, red);
  if (blockIdx.x == 0 && threadIdx.x == 0) alpha_out[0] = alpha;
  const float t = alpha + eps;
  const int64_t id = (int64_t)blockIdx.x * PT_THREADS + threadIdx.x;
  if (id >= n_words) return;
  const int64_t k = id % K, d = id / K;
  u32 word = 0;
#pragma unroll
  for (int f = 0; f < 16; ++f) {
    const int64_t n = d * 16 + f;
    if (n < N) word |= pt_code(pt_load<T>(W, n * K + k), t) << (2 * f);
  }
  out[((d >> 5) * K + k) * 32 + (d & 31)] = word;
}

// One thread per 32-bit word of the block-float GEMM layout: blocks of 32 outputs x 128 input
// channels (2048 bytes); inside, row r = n % 32 takes 64 bytes, its 16-byte piece p holds the
// 32 channels of unit u = p ^ ((r / 4) % 4) as E2M1 nibbles (0 -> 0000, +1 -> 0010, -1 -> 1010),
// low nibble first.  A word covers 8 consecutive channels.
template <typename T>
__global__ __launch_bounds__(PT_THREADS) void ternarize_pack_mx4_kernel(
    const T* __restrict__ W, int64_t N, int64_t K, int64_t Kp, float eps,
    const double* __restrict__ partial, int n_partial, u32* __restrict__ out,
    float* __restrict__ alpha_out, int64_t n_words) {
  __shared__ double red[PT_THREADS / BL_WAVE];
  const float alpha = pt_alpha(partial, n_partial, N * K, red);
  if (blockIdx.x == 0 && threadIdx.x == 0) alpha_out[0] = alpha;
  const float t = alpha + eps;
  const int64_t w = (int64_t)blockIdx.x * PT_THREADS + threadIdx.x;
  if (w >= n_words) return;
  const int64_t blk = w >> 9;               // 512 words per block
  const int in = (int)(w & 511);
  const int r = in >> 4, p = (in >> 2) & 3, j = in & 3;
  const int64_t KB = Kp / 128;
  const int64_t n = (blk / KB) * 32 + r;
  const int64_t k0 = (blk % KB) * 128 + 32 * (p ^ ((r >> 2) & 3)) + 8 * j;
  u32 word = 0;
  if (n < N) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int64_t k = k0 + i;
      if (k < K) {
        const u32 c = pt_code(pt_load<T>(W, n * K + k), t);        // 00, 01, 11
        word |= (((c & 2u) << 2) | ((c & 1u) << 1)) << (4 * i);    // sign to bit 3, magnitude 1.0 = 010
      }
    }
  }
  out[w] = word;
}

// One thread per 32-bit word of the 2-bit block-float GEMM layout: blocks of 32 outputs x 128 input
// channels (1024 bytes); inside, row r = n % 32 takes 32 bytes, its 8-byte piece p holds the 32
// channels of unit u = p ^ ((r / 8) % 4) as two words of 16 channels: nibble j of a word keeps
// channels j and 8 + j as (sign j, sign 8+j, magnitude j, magnitude 8+j) from bit 3 down, so that
// one mask, and one shift and mask, give their E2M1 nibbles (sign 0 magnitude 0).
template <typename T>
__global__ __launch_bounds__(PT_THREADS) void ternarize_pack_mx2_kernel(
    const T* __restrict__ W, int64_t N, int64_t K, int64_t Kp, float eps,
    const double* __restrict__ partial, int n_partial, u32* __restrict__ out,
    float* __restrict__ alpha_out, int64_t n_words) {
  __shared__ double red[PT_THREADS / BL_WAVE];
  const float alpha = pt_alpha(partial, n_partial, N * K, red);
  if (blockIdx.x == 0 && threadIdx.x == 0) alpha_out[0] = alpha;
  const float t = alpha + eps;
  const int64_t w = (int64_t)blockIdx.x * PT_THREADS + threadIdx.x;
  if (w >= n_words) return;
  const int64_t blk = w >> 8;               // 256 words per block
  const int in = (int)(w & 255);
  const int r = in >> 3, p = (in >> 1) & 3, h = in & 1;
  const int64_t KB = Kp / 128;
  const int64_t n = (blk / KB) * 32 + r;
  const int64_t k0 = (blk % KB) * 128 + 32 * (p ^ ((r >> 3) & 3)) + 16 * h;
  u32 word = 0;
  if (n < N) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      if (k0 + j < K) {
        const u32 c = pt_code(pt_load<T>(W, n * K + k0 + j), t);            // 00, 01, 11
        word |= (((c & 2u) << 2) | ((c & 1u) << 1)) << (4 * j);
      }
      if (k0 + 8 + j < K) {
        const u32 c = pt_code(pt_load<T>(W, n * K + k0 + 8 + j), t);
        word |= (((c & 2u) << 1) | (c & 1u)) << (4 * j);
      }
    }
  }
  out[w] = word;
}

// One thread per 32-bit word of the output-channel-major layout: row n, channels 16 w .. 16 w + 15,
// channel 16 w + f in bits 2 f, 2 f + 1.
template <typename T>
__global__ __launch_bounds__(PT_THREADS) void ternarize_pack_rows_kernel(
    const T* __restrict__ W, int64_t N, int64_t K, int64_t Kp, float eps,
    const double* __restrict__ partial, int n_partial, u32* __restrict__ out,
    float* __restrict__ alpha_out, int64_t n_words) {
  __shared__ double red[PT_THREADS / BL_WAVE];
  const float alpha = pt_alpha(partial, n_partial, N * K, red);
  if (blockIdx.x == 0 && threadIdx.x == 0) alpha_out[0] = alpha;
  const float t = alpha + eps;
  const int64_t w = (int64_t)blockIdx.x * PT_THREADS + threadIdx.x;
  if (w >= n_words) return;
  const int64_t wpr = Kp / 16, n = w / wpr, k0 = (w % wpr) * 16;
  u32 word = 0;
#pragma unroll
  for (int f = 0; f < 16; ++f)
    if (k0 + f < K) word |= pt_code(pt_load<T>(W, n * K + k0 + f), t) << (2 * f);
  out[w] = word;
}

__global__ __launch_bounds__(PT_THREADS) void unpack_ternary_kernel(const u32* __restrict__ packed,
                                                                    int64_t N, int64_t K,
                                                                    int64_t Kp, int64_t Np,
                                                                    int layout,
                                                                    int8_t* __restrict__ T) {
  const int64_t id = (int64_t)blockIdx.x * PT_THREADS + threadIdx.x;
  if (id >= N * K) return;
  const int64_t n = id / K, k = id % K;
  u32 word;
  int f;
  if (layout == BL_W_MX4) {
    const int r = (int)(n & 31), u = (int)((k >> 5) & 3), i = (int)(k & 31);
    const u32 w4 = packed[((n >> 5) * (Kp / 128) + (k >> 7)) * 512 + r * 16 + ((u ^ ((r >> 2) & 3)) << 2) + (i >> 3)];
    const u32 c = (w4 >> (4 * (i & 7))) & 15u;
    T[id] = (int8_t)(c == 0 ? 0 : ((c & 8u) ? -1 : 1));
    return;
  }
  if (layout == BL_W_MX2) {
    const int r = (int)(n & 31), u = (int)((k >> 5) & 3), i = (int)(k & 31);
    word = packed[((n >> 5) * (Kp / 128) + (k >> 7)) * 256 + r * 8 + ((u ^ ((r >> 3) & 3)) << 1) + (i >> 4)];
    const u32 nib = (word >> (4 * (i & 7))) << ((i >> 3) & 1);       // channel's sign in bit 3, magnitude in bit 1
    T[id] = (int8_t)((nib & 2u) ? ((nib & 8u) ? -1 : 1) : 0);
    return;
  } else if (layout == BL_W_ROWS) {
    word = packed[n * (Kp / 16) + (k >> 4)];
    f = (int)(k & 15);
  } else if (layout == BL_W_GEMM) {
    const int64_t nt = n >> 4, kt = k >> 8;
    const int i = (int)(n & 15), g = (int)((k >> 6) & 3), t = (int)((k >> 4) & 3);
    const int kk = (int)(k & 15);
    f = 4 * (kk & 3) + (kk >> 2);
    word = packed[(nt * (Kp / 256) + kt) * 256 + (g * 16 + i) * 4 + t];
  } else {
    word = packed[((n >> 9) * K + k) * 32 + ((n >> 4) & 31)];
    f = (int)(n & 15);
  }
  const u32 c = (word >> (2 * f)) & 3u;
  T[id] = (int8_t)((int)(c << 30) >> 30);   // sign-extend the 2-bit field
}

static int pt_num_partials(int64_t n) {
  int64_t b = (n + (int64_t)PT_THREADS * 16 - 1) / ((int64_t)PT_THREADS * 16);
  if (b < 1) b = 1;
  if (b > PT_MAX_PARTIALS) b = PT_MAX_PARTIALS;
  return (int)b;
}

extern "C" size_t pack_ternary_workspace_bytes(int64_t N, int64_t K) {
  (void)N; (void)K;
  return PT_MAX_PARTIALS * sizeof(double);
}

template <typename T>
static int pt_run(const T* W, int64_t N, int64_t K, float eps, bl_w_layout layout, void* out,
                  float* alpha, void* ws, hipStream_t s) {
  const int64_t n = N * K;
  const int np = pt_num_partials(n);
  double* partial = (double*)ws;
  abs_sum_partial_kernel<T><<<np, PT_THREADS, 0, s>>>(W, n, partial);
  BL_HIP_CHECK_LAUNCH();
  if (layout == BL_W_MX4) {
    const int64_t Kp = bl_round_up(K, BL_KPAD), Np = bl_round_up(N, 32);
    const int64_t n_words = Np * Kp / 8;
    const int64_t blocks = (n_words + PT_THREADS - 1) / PT_THREADS;
    ternarize_pack_mx4_kernel<T><<<(unsigned)blocks, PT_THREADS, 0, s>>>(
        W, N, K, Kp, eps, partial, np, (u32*)out, alpha, n_words);
  } else if (layout == BL_W_MX2) {
    const int64_t Kp = bl_round_up(K, BL_KPAD), Np = bl_round_up(N, 32);
    const int64_t n_words = Np * Kp / 16;
    const int64_t blocks = (n_words + PT_THREADS - 1) / PT_THREADS;
    ternarize_pack_mx2_kernel<T><<<(unsigned)blocks, PT_THREADS, 0, s>>>(
        W, N, K, Kp, eps, partial, np, (u32*)out, alpha, n_words);
  } else if (layout == BL_W_ROWS) {
    const int64_t Kp = bl_round_up(K, BL_KPAD);
    const int64_t n_words = N * Kp / 16;
    const int64_t blocks = (n_words + PT_THREADS - 1) / PT_THREADS;
    ternarize_pack_rows_kernel<T><<<(unsigned)blocks, PT_THREADS, 0, s>>>(
        W, N, K, Kp, eps, partial, np, (u32*)out, alpha, n_words);
  } else if (layout == BL_W_GEMM) {
    const int64_t Kp = bl_round_up(K, BL_KPAD), Np = bl_round_up(N, 16);
    const int64_t n_words = Np * Kp / 16;
    const int64_t blocks = (n_words + PT_THREADS - 1) / PT_THREADS;
    ternarize_pack_gemm_kernel<T><<<(unsigned)blocks, PT_THREADS, 0, s>>>(
        W, N, K, Kp, eps, partial, np, (u32*)out, alpha, n_words);
  } else {
    const int64_t Np = bl_round_up(N, 512);
    const int64_t n_words = K * (Np / 16);
    const int64_t blocks = (n_words + PT_THREADS - 1) / PT_THREADS;
    ternarize_pack_kmajor_kernel<T><<<(unsigned)blocks, PT_THREADS, 0, s>>>(
        W, N, K, Np, eps, partial, np, (u32*)out, alpha, n_words);
  }
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

int bl_launch_pack_ternary(const void* W, bl_dtype dt, int64_t N, int64_t K, float eps,
                           bl_w_layout layout, void* out, float* alpha, void* ws, hipStream_t s) {
  if (dt == BL_F32) return pt_run<float>((const float*)W, N, K, eps, layout, out, alpha, ws, s);
  return pt_run<uint16_t>((const uint16_t*)W, N, K, eps, layout, out, alpha, ws, s);
}

int bl_launch_unpack_ternary(const void* packed, int64_t N, int64_t K, bl_w_layout layout,
                             int8_t* T, hipStream_t s) {
  const int64_t blocks = (N * K + PT_THREADS - 1) / PT_THREADS;
  unpack_ternary_kernel<<<(unsigned)blocks, PT_THREADS, 0, s>>>(
      (const u32*)packed, N, K, bl_round_up(K, BL_KPAD), bl_round_up(N, 512), (int)layout, T);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}
