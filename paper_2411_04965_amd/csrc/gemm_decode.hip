// Decode-shaped (1..64 tokens) linears: the packed ternary weights are streamed from HBM once.
//   Dense path  (BL_W_GEMM tiles):   skinny int8-MFMA GEMM; three kernels by token count.
//   Sparse path (BL_W_KMAJOR rows):  eq. 1's sparsity used for I/O — only the weight rows of
//                                    channels whose INT8 code is non-zero in some token are read.
// Integer partial sums are exact, so any split of K gives the same accumulators.
#include "common.h"
#include "topk_regs.h"

#define GD_THREADS 256
#define GD_BN 64           // outputs per block (4 MFMA tiles of 16)

// ---------------------------------------------------------------- shared epilogue
__device__ __forceinline__ void gd_store4(void* Y, int y_bf16, int32_t* acc_out, size_t o, int n,
                                          int N, const int (&iv)[4], float d, float alpha) {
  float fv[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) fv[r] = ((float)iv[r] * d) * alpha;
  if ((N & 3) == 0) {
    if (y_bf16) {
      uint2 p;
      p.x = (u32)bl_f32_to_bf16_rne(fv[0]) | ((u32)bl_f32_to_bf16_rne(fv[1]) << 16);
      p.y = (u32)bl_f32_to_bf16_rne(fv[2]) | ((u32)bl_f32_to_bf16_rne(fv[3]) << 16);
      *reinterpret_cast<uint2*>((uint16_t*)Y + o) = p;
    } else {
      *reinterpret_cast<float4*>((float*)Y + o) = make_float4(fv[0], fv[1], fv[2], fv[3]);
    }
    if (acc_out) *reinterpret_cast<int4*>(acc_out + o) = make_int4(iv[0], iv[1], iv[2], iv[3]);
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (n + r < N) {
        if (y_bf16) ((uint16_t*)Y)[o + r] = bl_f32_to_bf16_rne(fv[r]);
        else ((float*)Y)[o + r] = fv[r];
        if (acc_out) acc_out[o + r] = iv[r];
      }
    }
  }
}

// ---------------------------------------------------------------- dense skinny GEMM
// Up to 16 tokens.  Block = 4 waves, one tile of 16 outputs.  The K tiles (256 channels) are dealt
// to the waves; every wave keeps MT accumulator tiles, added through LDS at the end: every block
// streams its own slice of W over all of K, no split across blocks, one launch.
template <int MT, bool A4>
__global__ __launch_bounds__(GD_THREADS) void gemm_decode_kernel(
    const unsigned char* __restrict__ A, const float* __restrict__ scale, int M, int Kp,
    const unsigned char* __restrict__ Wp, const float* __restrict__ alpha_p, int N,
    void* __restrict__ Y, int y_bf16, int32_t* __restrict__ acc_out, int32_t* __restrict__ partial,
    int NB, int S) {
  constexpr int NTB = 1;
  extern __shared__ __align__(16) unsigned char gd_smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int nb = blockIdx.x % NB, split = blockIdx.x / NB;
  const int KT = Kp >> 8;
  const int t_begin = (int)((int64_t)split * KT / S), t_end = (int)((int64_t)(split + 1) * KT / S);
  const int NT16 = (N + 15) >> 4;
  constexpr int XV = A4 ? 2 : 4;                 // 16-byte loads per token row per tile
  const int a_row_bytes = A4 ? (Kp >> 1) : Kp;

  const unsigned char* w_src[NTB];
#pragma unroll
  for (int a = 0; a < NTB; ++a) {
    const int nt = min(nb * NTB + a, NT16 - 1);
    w_src[a] = Wp + (size_t)nt * KT * 1024 + lane * 16;
  }
  const unsigned char* x_src[MT];
#pragma unroll
  for (int b = 0; b < MT; ++b) {
    const int row = min(b * 16 + li, M - 1);
    x_src[b] = A + (size_t)row * a_row_bytes + lg * (A4 ? 32 : 64);
  }

  v4i acc[NTB][MT];
#pragma unroll
  for (int a = 0; a < NTB; ++a)
#pragma unroll
    for (int b = 0; b < MT; ++b) acc[a][b] = (v4i){0, 0, 0, 0};

  // UNR tiles (256 channels each) are loaded together before they are multiplied, so that a
  // wave keeps several KB of weights in flight; the next group is prefetched meanwhile.
  constexpr int UNR = NTB == 1 ? 4 : 1;
  uint4 wr[UNR][NTB], xr[UNR][MT][XV];
  auto load_group = [&](int t) {
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int tt = min(t + 4 * u, t_end - 1);     // tiles past the end re-read the last one (unused)
#pragma unroll
      for (int a = 0; a < NTB; ++a) wr[u][a] = *reinterpret_cast<const uint4*>(w_src[a] + (size_t)tt * 1024);
#pragma unroll
      for (int b = 0; b < MT; ++b)
#pragma unroll
        for (int c = 0; c < XV; ++c)
          xr[u][b][c] = *reinterpret_cast<const uint4*>(x_src[b] + (size_t)tt * (A4 ? 128 : 256) + c * 16);
    }
  };

  int t = t_begin + wave;
  if (t < t_end) load_group(t);
  while (t < t_end) {
    uint4 wc[UNR][NTB], xc[UNR][MT][XV];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
#pragma unroll
      for (int a = 0; a < NTB; ++a) wc[u][a] = wr[u][a];
#pragma unroll
      for (int b = 0; b < MT; ++b)
#pragma unroll
        for (int c = 0; c < XV; ++c) xc[u][b][c] = xr[u][b][c];
    }
    const int tn = t + 4 * UNR;
    if (tn < t_end) load_group(tn);                // prefetch while computing
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      if (t + 4 * u >= t_end) break;
#pragma unroll
      for (int t4 = 0; t4 < 4; ++t4) {
        v4i xo[MT];
#pragma unroll
        for (int b = 0; b < MT; ++b) {
          if (A4) {
            // 64 channels = 8 words; MFMA step t4 takes words 2*t4 and 2*t4+1
            const uint4 v = xc[u][b][t4 >> 1];
            const u32 x0 = (t4 & 1) ? v.z : v.x, x1 = (t4 & 1) ? v.w : v.y;
            xo[b] = (v4i){(int)((x0 << 4) & 0xF0F0F0F0u), (int)(x0 & 0xF0F0F0F0u),
                          (int)((x1 << 4) & 0xF0F0F0F0u), (int)(x1 & 0xF0F0F0F0u)};
          } else {
            const uint4 v = xc[u][b][t4];
            xo[b] = (v4i){(int)v.x, (int)v.y, (int)v.z, (int)v.w};
          }
        }
#pragma unroll
        for (int a = 0; a < NTB; ++a) {
          const u32 w = t4 == 0 ? wc[u][a].x : t4 == 1 ? wc[u][a].y : t4 == 2 ? wc[u][a].z : wc[u][a].w;
          const v4i wo = (v4i){(int)((w << 6) & 0xC0C0C0C0u), (int)((w << 4) & 0xC0C0C0C0u),
                               (int)((w << 2) & 0xC0C0C0C0u), (int)(w & 0xC0C0C0C0u)};
#pragma unroll
          for (int b = 0; b < MT; ++b)
            acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wo, xo[b], acc[a][b], 0, 0, 0);
        }
      }
    }
    t = tn;
  }

  // cross-wave reduction: the NTB x MT accumulator tiles are dealt round-robin to the waves
  v4i* red = reinterpret_cast<v4i*>(gd_smem);     // [wave][a][b][lane]
#pragma unroll
  for (int a = 0; a < NTB; ++a)
#pragma unroll
    for (int b = 0; b < MT; ++b) red[((wave * NTB + a) * MT + b) * 64 + lane] = acc[a][b];
  __syncthreads();
  const float alpha = alpha_p[0];
  constexpr int SHIFT = A4 ? 10 : 6;
#pragma unroll
  for (int a = 0; a < NTB; ++a) {
#pragma unroll
    for (int b = 0; b < MT; ++b) {
      if (((a * MT + b) & 3) != wave) continue;
      v4i sum = (v4i){0, 0, 0, 0};
#pragma unroll
      for (int w = 0; w < 4; ++w) sum += red[((w * NTB + a) * MT + b) * 64 + lane];
      const int m = b * 16 + li;
      const int n = (nb * NTB + a) * 16 + 4 * lg;
      if (m >= M || n >= N) continue;
      const size_t o = (size_t)m * N + n;
      if (S == 1) {
        const int iv[4] = {sum[0] >> SHIFT, sum[1] >> SHIFT, sum[2] >> SHIFT, sum[3] >> SHIFT};
        gd_store4(Y, y_bf16, acc_out, o, n, N, iv, scale[m], alpha);
      } else {
        int32_t* p = partial + (size_t)split * M * N + o;
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (n + r < N) p[r] = sum[r];
      }
    }
  }
}

// One token (the kernel takes up to 4), INT4 activations: eq. 7 inside the same launch.  Every block quantizes the
// tokens itself (their rows are a few KB and come out of the cache; the statistics and the codes
// take a few hundred instructions per thread), which saves the quantizer's launch: at these sizes a
// launch costs as much as streaming the weights.  The arithmetic is that of the stand-alone
// quantizer (float64 sum of |x|, one rounding to float32, one float32 multiply per element), so
// the codes are the same bit for bit.  Codes are kept as int8 in LDS, one row per token.
#define GF_NV 4                                  // 16-byte pieces of a row per thread: K <= 8192

// eq. 7 for up to 4 bfloat16 token rows by one workgroup of 256 threads: int8 codes to `codes`
// ([M][Kp], LDS), the dequantization scales beta / sqrt(7) to dq (the same in every thread).  The
// rows are read 8 channels per piece, pieces tid, tid + 256, ... of every token (zero beyond K;
// K % 8 == 0, K <= 8192), all loads in flight together; beta = mean |x| comes from the registers
// (float64 sums, exact, so their order does not matter).  Ends with a barrier.
__device__ __forceinline__ void gf_quantize_rows(const uint16_t* __restrict__ X, int M, int K, int Kp,
                                                 float eps, unsigned char* codes, float (&dq)[4]) {
  __shared__ double red[4][GD_THREADS / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  uint4 xr[4][GF_NV];
  const int nv = K >> 3;
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int j = 0; j < GF_NV; ++j) {
      xr[m][j] = make_uint4(0u, 0u, 0u, 0u);
      const int pc = tid + GD_THREADS * j;
      if (m < M && pc < nv) xr[m][j] = reinterpret_cast<const uint4*>(X + (size_t)m * K)[pc];
    }
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    if (m < M) {                                 // block-uniform
      double a = 0.0;
#pragma unroll
      for (int j = 0; j < GF_NV; ++j) {
        const u32 w4[4] = {xr[m][j].x, xr[m][j].y, xr[m][j].z, xr[m][j].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a += (double)fabsf(__uint_as_float(w4[e] << 16));
          a += (double)fabsf(__uint_as_float(w4[e] & 0xFFFF0000u));
        }
      }
      a = bl_wave_sum_f64_dpp(a);
      if (lane == 0) red[m][wave] = a;
    }
  }
  __syncthreads();
  const float sqrt7 = 2.6457512f;                // float32(sqrt(7))
  // codes: RoundClip(x * s, -8, 7), eight to a piece
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    double tot = 0.0;
#pragma unroll
    for (int w = 0; w < GD_THREADS / 64; ++w) tot += red[m < M ? m : 0][w];
    const float beta = (float)(tot / (double)K);
    const float s = sqrt7 / (beta + eps);
    dq[m] = beta / sqrt7;
    if (m < M) {
#pragma unroll
      for (int j = 0; j < GF_NV; ++j) {
        const int pc = tid + GD_THREADS * j;
        if (pc < (Kp >> 3)) {
          const u32 w4[4] = {xr[m][j].x, xr[m][j].y, xr[m][j].z, xr[m][j].w};
          u32 cw[2] = {0u, 0u};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p0 = fminf(fmaxf(rintf(__uint_as_float(w4[e] << 16) * s), -8.0f), 7.0f);
            const float p1 = fminf(fmaxf(rintf(__uint_as_float(w4[e] & 0xFFFF0000u) * s), -8.0f), 7.0f);
            cw[e >> 1] |= (((u32)(int)p0 & 0xFFu) | (((u32)(int)p1 & 0xFFu) << 8)) << (16 * (e & 1));
          }
          *reinterpret_cast<uint2*>(codes + (size_t)m * Kp + pc * 8) = make_uint2(cw[0], cw[1]);
        }
      }
    }
  }
  __syncthreads();

}

__global__ __launch_bounds__(GD_THREADS) void gemv_a4_fused_kernel(
    const uint16_t* __restrict__ X, int M, int K, int Kp, float eps,
    const unsigned char* __restrict__ Wp, const float* __restrict__ alpha_p, int N,
    void* __restrict__ Y, int y_bf16, int32_t* __restrict__ acc_out) {
  extern __shared__ __align__(16) unsigned char gf_smem[];
  unsigned char* codes = gf_smem;                                  // [M][Kp] int8
  __shared__ __align__(16) v4i wsum[GD_THREADS / 64][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int KT = Kp >> 8;
  const int nt = blockIdx.x;                     // grid = tiles of 16 outputs
  const unsigned char* w_src = Wp + (size_t)nt * KT * 1024 + lane * 16;

  // weights first: tiles wave, wave + 4, ... in groups of 4 (the next group is fetched while one
  // is multiplied)
  constexpr int UNR = 4;
  uint4 wr[UNR];
  auto load_group = [&](int t) {
#pragma unroll
    for (int u = 0; u < UNR; ++u)
      wr[u] = *reinterpret_cast<const uint4*>(w_src + (size_t)min(t + 4 * u, KT - 1) * 1024);
  };
  int t = wave;
  if (t < KT) load_group(t);

  float dq[4];
  gf_quantize_rows(X, M, K, Kp, eps, codes, dq);

  // lane (li, lg) holds, for token li, the 64 channels lg * 64 .. of a tile, 16 per MFMA step
  v4i acc = (v4i){0, 0, 0, 0};
  const unsigned char* xrow = codes + (size_t)min(li, M - 1) * Kp + lg * 64;
  while (t < KT) {
    uint4 wc[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) wc[u] = wr[u];
    const int tn = t + 4 * UNR;
    if (tn < KT) load_group(tn);
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int tt = t + 4 * u;
      if (tt < KT) {                             // wave-uniform
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
          v4i xo = (v4i){0, 0, 0, 0};
          if (li < M) xo = *reinterpret_cast<const v4i*>(xrow + (size_t)tt * 256 + t4 * 16);
          const u32 w = t4 == 0 ? wc[u].x : t4 == 1 ? wc[u].y : t4 == 2 ? wc[u].z : wc[u].w;
          const v4i wo = (v4i){(int)((w << 6) & 0xC0C0C0C0u), (int)((w << 4) & 0xC0C0C0C0u),
                               (int)((w << 2) & 0xC0C0C0C0u), (int)(w & 0xC0C0C0C0u)};
          acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wo, xo, acc, 0, 0, 0);
        }
      }
    }
    t = tn;
  }

  // add the four waves' sums; wave 0 rescales and stores
  wsum[wave][lane] = acc;
  __syncthreads();
  if (wave != 0) return;
  v4i sum = wsum[0][lane] + wsum[1][lane] + wsum[2][lane] + wsum[3][lane];
  const int m = li, n = nt * 16 + 4 * lg;
  if (m >= M || n >= N) return;
  const int iv[4] = {sum[0] >> 6, sum[1] >> 6, sum[2] >> 6, sum[3] >> 6};
  const float d = m == 0 ? dq[0] : m == 1 ? dq[1] : m == 2 ? dq[2] : dq[3];
  gd_store4(Y, y_bf16, acc_out, (size_t)m * N + n, n, N, iv, d, alpha_p[0]);
}

// Gate-first up projection for a few tokens: U = INT4 linear of X with row-addressable weights
// (BL_W_ROWS), computed only for the outputs whose gate is open for some token, and combined with
// the gate at once: H = bf16(U * max(G, 0)^2) (eq. 5).  Every block quantizes the tokens itself
// (as above), takes NPB consecutive outputs, lists the open ones in LDS and deals them to its
// waves; a wave reads one weight row per pass (16 bytes = 64 channels per lane and 1 KB chunk),
// the lane's token codes stay in registers, byte-transposed once so that v_dot4 pairs four
// channels 4 apart (the fields of one bit position of a weight word) with their codes.
template <int MV, int NCH>
__global__ __launch_bounds__(GD_THREADS) void up_gated_kernel(
    const uint16_t* __restrict__ X, int M, int K, int Kp, float eps, const u32* __restrict__ Wr,
    const float* __restrict__ alpha_p, int N, const void* __restrict__ G, int g_f32,
    uint16_t* __restrict__ H, int NPB) {
  extern __shared__ __align__(16) unsigned char gf_smem[];
  unsigned char* codes = gf_smem;                                  // [M][Kp] int8
  __shared__ int lst[GD_THREADS];
  __shared__ int wave_cnt[GD_THREADS / 64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  float dq[4];
  gf_quantize_rows(X, M, K, Kp, eps, codes, dq);

  // this lane's codes: chunk c covers channels 4096 c + 64 lane ... + 63; word w of a chunk's
  // 16-byte weight piece covers 16 of them, xq[..][w][j] = codes of channels j, 4+j, 8+j, 12+j of those
  u32 xq[MV][NCH][4][4];
#pragma unroll
  for (int m = 0; m < MV; ++m)
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int ch = 4096 * c + 64 * lane;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (m < M && ch < Kp) v = *reinterpret_cast<const uint4*>(codes + (size_t)m * Kp + ch + 16 * w);
        const u32 t01l = __builtin_amdgcn_perm(v.y, v.x, 0x05010400u);  // x.b0 y.b0 x.b1 y.b1
        const u32 t01h = __builtin_amdgcn_perm(v.y, v.x, 0x07030602u);
        const u32 t23l = __builtin_amdgcn_perm(v.w, v.z, 0x05010400u);
        const u32 t23h = __builtin_amdgcn_perm(v.w, v.z, 0x07030602u);
        xq[m][c][w][0] = __builtin_amdgcn_perm(t23l, t01l, 0x05040100u);   // bytes 0 of x, y, z, w
        xq[m][c][w][1] = __builtin_amdgcn_perm(t23l, t01l, 0x07060302u);
        xq[m][c][w][2] = __builtin_amdgcn_perm(t23h, t01h, 0x05040100u);
        xq[m][c][w][3] = __builtin_amdgcn_perm(t23h, t01h, 0x07060302u);
      }
    }

  // the block's outputs: open gates listed, closed ones written as zero
  const int n_begin = blockIdx.x * NPB, n_end = min(n_begin + NPB, N);    // NPB <= 256
  auto gate = [&](int m, int n) -> float {
    return g_f32 ? reinterpret_cast<const float*>(G)[(size_t)m * N + n]
                 : bl_bf16_to_f32(reinterpret_cast<const uint16_t*>(G)[(size_t)m * N + n]);
  };
  {
    const int n = n_begin + tid;
    bool open = false;
    if (n < n_end)
      for (int m = 0; m < M; ++m) open |= gate(m, n) > 0.0f;
    const uint64_t bal = __ballot(open);
    if (lane == 0) wave_cnt[wave] = __popcll(bal);
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += wave_cnt[w];
    if (open) lst[before + __popcll(bal & ((1ull << lane) - 1ull))] = n;
    if (n < n_end && !open)
      for (int m = 0; m < M; ++m) H[(size_t)m * N + n] = 0;
    __syncthreads();
  }
  const int L = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
  const float alpha = alpha_p[0];
  const int wpr = Kp >> 4;                       // words per weight row
  auto load_row = [&](int idx, uint4 (&wv)[NCH]) {
    const u32* row = Wr + (size_t)lst[min(idx, L - 1)] * wpr;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      wv[c] = make_uint4(0u, 0u, 0u, 0u);
      if (1024 * c + 16 * lane < (Kp >> 2)) wv[c] = *reinterpret_cast<const uint4*>(row + 256 * c + 4 * lane);
    }
  };
  uint4 wn[NCH];
  if (wave < L) load_row(wave, wn);
  for (int idx = wave; idx < L; idx += GD_THREADS / 64) {
    uint4 wc[NCH];
#pragma unroll
    for (int c = 0; c < NCH; ++c) wc[c] = wn[c];
    if (idx + GD_THREADS / 64 < L) load_row(idx + GD_THREADS / 64, wn);
    int acc[MV];
#pragma unroll
    for (int m = 0; m < MV; ++m) acc[m] = 0;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const u32 ww[4] = {wc[c].x, wc[c].y, wc[c].z, wc[c].w};
#pragma unroll
      for (int w = 0; w < 4; ++w)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const u32 tw = (ww[w] << (6 - 2 * j)) & 0xC0C0C0C0u;     // channels j, 4+j, 8+j, 12+j, times 64
#pragma unroll
          for (int m = 0; m < MV; ++m) acc[m] = __builtin_amdgcn_sdot4((int)tw, (int)xq[m][c][w][j], acc[m], false);
        }
    }
    const int n = lst[idx];
#pragma unroll
    for (int m = 0; m < MV; ++m) {
      const int tot = qa_wave_sum_dpp(acc[m]) >> 6;
      if (m < M && lane == 0) {
        const float d = m == 0 ? dq[0] : m == 1 ? dq[1] : m == 2 ? dq[2] : dq[3];
        const float u = ((float)tot * d) * alpha;
        const float r = fmaxf(gate(m, n), 0.0f);
        const float rr = r * r;
        H[(size_t)m * N + n] = bl_f32_to_bf16_rne(u * rr);
      }
    }
  }
}

// One token, top-K + INT8 activations: eq. 1 and eq. 3 inside the same launch, for the same reason.
// Every block selects and quantizes the token itself with the four-wave register kernel's body
// (topk_regs.h) while its first weight tiles are on their way, and leaves the int8 codes in LDS.
template <int CPW>
__global__ __launch_bounds__(GD_THREADS) void gemv_a8_fused_kernel(
    const uint16_t* __restrict__ X, int K, int Kp, int topk, float eps,
    const unsigned char* __restrict__ Wp, const float* __restrict__ alpha_p, int N,
    void* __restrict__ Y, int y_bf16, int32_t* __restrict__ acc_out) {
  extern __shared__ __align__(16) unsigned char gf_smem[];         // [Kp] int8
  __shared__ float dq;
  __shared__ __align__(16) v4i wsum[GD_THREADS / 64][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int KT = Kp >> 8;
  const int nt = blockIdx.x;                     // grid = tiles of 16 outputs
  const unsigned char* w_src = Wp + (size_t)nt * KT * 1024 + lane * 16;
  constexpr int UNR = 4;
  uint4 wr[UNR];
  auto load_group = [&](int t) {
#pragma unroll
    for (int u = 0; u < UNR; ++u)
      wr[u] = *reinterpret_cast<const uint4*>(w_src + (size_t)min(t + 4 * u, KT - 1) * 1024);
  };
  int t = wave;
  if (t < KT) load_group(t);

  qa_topk_row_regs<CPW>(X, nullptr, K, Kp, topk, eps, reinterpret_cast<u32*>(gf_smem), &dq, nullptr);
  __syncthreads();

  v4i acc = (v4i){0, 0, 0, 0};
  const unsigned char* xrow = gf_smem + lg * 64;
  while (t < KT) {
    uint4 wc[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) wc[u] = wr[u];
    const int tn = t + 4 * UNR;
    if (tn < KT) load_group(tn);
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int tt = t + 4 * u;
      if (tt < KT) {                             // wave-uniform
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
          v4i xo = (v4i){0, 0, 0, 0};
          if (li == 0) xo = *reinterpret_cast<const v4i*>(xrow + (size_t)tt * 256 + t4 * 16);
          const u32 w = t4 == 0 ? wc[u].x : t4 == 1 ? wc[u].y : t4 == 2 ? wc[u].z : wc[u].w;
          const v4i wo = (v4i){(int)((w << 6) & 0xC0C0C0C0u), (int)((w << 4) & 0xC0C0C0C0u),
                               (int)((w << 2) & 0xC0C0C0C0u), (int)(w & 0xC0C0C0C0u)};
          acc = __builtin_amdgcn_mfma_i32_16x16x64_i8(wo, xo, acc, 0, 0, 0);
        }
      }
    }
    t = tn;
  }
  wsum[wave][lane] = acc;
  __syncthreads();
  if (wave != 0) return;
  v4i sum = wsum[0][lane] + wsum[1][lane] + wsum[2][lane] + wsum[3][lane];
  const int n = nt * 16 + 4 * lg;
  if (li != 0 || n >= N) return;
  const int iv[4] = {sum[0] >> 6, sum[1] >> 6, sum[2] >> 6, sum[3] >> 6};
  gd_store4(Y, y_bf16, acc_out, (size_t)n, n, N, iv, dq, alpha_p[0]);
}

// Up to 16 tokens with too few output tiles for the kernel above (written for any number of token
// tiles): block = 4 waves = 64 outputs, every wave owns one tile of 16 outputs and walks the block's whole K range (a
// slice of K when the grid would otherwise be small), so there is no reduction inside the block.
// The tokens' codes of one K tile (M rows of 128 or 256 bytes, far apart in memory) are fetched
// once per block with whole-line loads and passed through LDS (rows padded by 16 bytes, so the
// 16-byte fragment reads of 16 token rows fall into 16 different slots of a 256-byte window); a
// wave reading them straight from memory asks for 16 to 32 lines per load and uses a quarter of
// each.  Weights are fetched four K tiles ahead (HBM latency), tokens one tile ahead.
template <int MT, bool A4>
__global__ __launch_bounds__(GD_THREADS) void gemm_decode_rows_kernel(
    const unsigned char* __restrict__ A, const float* __restrict__ scale, int M, int Kp,
    const unsigned char* __restrict__ Wp, const float* __restrict__ alpha_p, int N,
    void* __restrict__ Y, int y_bf16, int32_t* __restrict__ acc_out, int32_t* __restrict__ partial,
    int NB, int S) {
  constexpr int TB = A4 ? 128 : 256;             // bytes of one token row per K tile
  constexpr int ROW = TB + 16;                   // LDS row pitch
  constexpr int PER_ROW = TB / 16;               // 16-byte pieces per row
  constexpr int XL = MT * 16 * PER_ROW / GD_THREADS;   // pieces per thread: 1 .. 4
  static_assert(MT * 16 * PER_ROW % GD_THREADS == 0 || MT == 1, "whole pieces per thread");
  constexpr int XLN = XL > 0 ? XL : 1;
  __shared__ __align__(16) unsigned char xs[2][MT * 16 * ROW];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int nb = blockIdx.x % NB, split = blockIdx.x / NB;
  const int KT = Kp >> 8;
  const int t_begin = (int)((int64_t)split * KT / S), t_end = (int)((int64_t)(split + 1) * KT / S);
  const int NT16 = (N + 15) >> 4;
  const int nt = nb * 4 + wave;
  const int a_row_bytes = A4 ? (Kp >> 1) : Kp;
  const unsigned char* w_src = Wp + (size_t)min(nt, NT16 - 1) * KT * 1024 + lane * 16;
  // piece j of this thread: row (tid + 256 j) / PER_ROW, piece (tid + 256 j) % PER_ROW
  const unsigned char* x_src[XLN];
  int x_dst[XLN];
  bool x_on[XLN];
#pragma unroll
  for (int j = 0; j < XLN; ++j) {
    const int idx = tid + GD_THREADS * j;
    const int row = idx / PER_ROW, pc = idx % PER_ROW;
    x_on[j] = row < MT * 16;                     // (MT == 1 with 128-byte rows: half the threads)
    x_src[j] = A + (size_t)min(row, M - 1) * a_row_bytes + pc * 16;
    x_dst[j] = min(row, MT * 16 - 1) * ROW + pc * 16;
  }
  v4i acc[MT];
#pragma unroll
  for (int b = 0; b < MT; ++b) acc[b] = (v4i){0, 0, 0, 0};

  constexpr int WD = 4;
  uint4 wq[WD], xn[XLN];
  auto load_x = [&](int t) {
#pragma unroll
    for (int j = 0; j < XLN; ++j)
      if (x_on[j]) xn[j] = *reinterpret_cast<const uint4*>(x_src[j] + (size_t)t * TB);
  };
  auto store_x = [&](int buf) {
#pragma unroll
    for (int j = 0; j < XLN; ++j)
      if (x_on[j]) *reinterpret_cast<uint4*>(&xs[buf][x_dst[j]]) = xn[j];
  };
  if (t_begin < t_end) {                         // block-uniform
#pragma unroll
    for (int j = 0; j < WD; ++j)
      wq[j] = *reinterpret_cast<const uint4*>(w_src + (size_t)min(t_begin + j, t_end - 1) * 1024);
    load_x(t_begin);
    store_x(0);
    __syncthreads();
  }
  const int frag = li * ROW + lg * (A4 ? 32 : 64);
  int buf = 0;
  for (int t0 = t_begin; t0 < t_end; t0 += WD) {
#pragma unroll
    for (int j = 0; j < WD; ++j) {
      const int t = t0 + j;
      if (t < t_end) {                           // block-uniform
        const uint4 wc = wq[j];
        if (t + 1 < t_end) load_x(t + 1);
        if (t + WD < t_end) wq[j] = *reinterpret_cast<const uint4*>(w_src + (size_t)(t + WD) * 1024);
        const unsigned char* xb = &xs[buf][frag];
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
          const u32 w = t4 == 0 ? wc.x : t4 == 1 ? wc.y : t4 == 2 ? wc.z : wc.w;
          const v4i wo = (v4i){(int)((w << 6) & 0xC0C0C0C0u), (int)((w << 4) & 0xC0C0C0C0u),
                               (int)((w << 2) & 0xC0C0C0C0u), (int)(w & 0xC0C0C0C0u)};
#pragma unroll
          for (int b = 0; b < MT; ++b) {
            v4i xo;
            if (A4) {
              // a lane's 64 channels = 8 words; MFMA step t4 takes words 2*t4 and 2*t4+1
              const uint2 v = *reinterpret_cast<const uint2*>(xb + b * 16 * ROW + t4 * 8);
              xo = (v4i){(int)((v.x << 4) & 0xF0F0F0F0u), (int)(v.x & 0xF0F0F0F0u),
                         (int)((v.y << 4) & 0xF0F0F0F0u), (int)(v.y & 0xF0F0F0F0u)};
            } else {
              xo = *reinterpret_cast<const v4i*>(xb + b * 16 * ROW + t4 * 16);
            }
            acc[b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wo, xo, acc[b], 0, 0, 0);
          }
        }
        // the other buffer was last read one tile ago, before the barrier every wave has passed
        if (t + 1 < t_end) store_x(buf ^ 1);
        __syncthreads();
        buf ^= 1;
      }
    }
  }

  if (nt >= NT16) return;
  const float alpha = alpha_p[0];
  constexpr int SHIFT = A4 ? 10 : 6;
#pragma unroll
  for (int b = 0; b < MT; ++b) {
    const int m = b * 16 + li;
    const int n = nt * 16 + 4 * lg;
    if (m >= M || n >= N) continue;
    const size_t o = (size_t)m * N + n;
    if (S == 1) {
      const int iv[4] = {acc[b][0] >> SHIFT, acc[b][1] >> SHIFT, acc[b][2] >> SHIFT, acc[b][3] >> SHIFT};
      gd_store4(Y, y_bf16, acc_out, o, n, N, iv, scale[m], alpha);
    } else {
      int32_t* p = partial + (size_t)split * M * N + o;
      if ((N & 3) == 0) {
        *reinterpret_cast<int4*>(p) = make_int4(acc[b][0], acc[b][1], acc[b][2], acc[b][3]);
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (n + r < N) p[r] = acc[b][r];
      }
    }
  }
}

// 17 to 64 tokens.  The tokens' codes are the larger stream here (a block of 16 outputs reads 4 KB
// of weights per 1024 channels but 32 to 64 KB of codes), and split-K partial sums cost as much
// again.  So the codes stay put: one block of 16 waves per CU keeps the codes of all tokens for its
// slice of K in LDS (up to 128 KB: all of K for INT4 codes at 4096 channels) and streams the weight
// tiles of its NWT output tiles past them.  The output tiles go in groups of up to GR_G to the
// waves, so that one expansion of a token fragment (nibbles to bytes) serves GR_G matrix
// instructions; wave u works on group u / KS and on part u % KS of the slice.  The parts are added
// in LDS (integer adds, in the space of the codes), from where whole row segments are stored.
#define GR_THREADS 1024
#define GR_WAVES 16
#define GR_G 3
#define GR_X_BYTES 131072                        // LDS for the codes (pitch = row bytes + 16)
#define GR_LDS_MAX (160 * 1024)                  // the LDS of a compute unit
// GLU: two weight matrices of one shape (gate, up).  The block's NWT tiles are then tile PAIRS in the order
// gate tile j, up tile j, a wave's group is one pair (G = 2), and the epilogue writes
// H = bf16(u * max(g, 0)^2) of the two rescaled float32 values (eq. 5; `Y` is H, bfloat16) instead of
// the products themselves.  No split of K across blocks in that form (S = 1).
template <int MT, bool A4, bool GLU = false>
__global__ __launch_bounds__(GR_THREADS) void gemm_decode_resident_kernel(
    const unsigned char* __restrict__ A, const float* __restrict__ scale, int M, int Kp,
    const unsigned char* __restrict__ Wp, const float* __restrict__ alpha_p, int N,
    void* __restrict__ Y, int y_bf16, int32_t* __restrict__ acc_out, int32_t* __restrict__ partial,
    int NBn, int S, int NWT, int KS, const unsigned char* __restrict__ Wp2 = nullptr,
    const float* __restrict__ alpha2_p = nullptr) {
  constexpr int G = GLU ? 2 : GR_G;              // output tiles per working wave
  extern __shared__ __align__(16) unsigned char gr_smem[];
  constexpr int TB = A4 ? 128 : 256;             // bytes of one token row per K tile
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int li = lane & 15, lg = lane >> 4;
  const int nbk = blockIdx.x % NBn, split = blockIdx.x / NBn;
  const int KT = Kp >> 8;
  const int t_begin = (int)((int64_t)split * KT / S), t_end = (int)((int64_t)(split + 1) * KT / S);
  const int L = t_end - t_begin;                 // tiles of this slice: L * TB * MT * 16 <= GR_X_BYTES
  const int NT16 = GLU ? 2 * ((N + 15) >> 4) : (N + 15) >> 4;   // tiles (GLU: gate and up tiles interleaved)
  const int a_row_bytes = A4 ? (Kp >> 1) : Kp;
  const int RB = L * TB, pitch = RB + 16, ppr = RB >> 4;

  // this wave's part of the work, and its first weight tiles (issued before the codes are staged)
  const int NG = (NWT + G - 1) / G;
  const int grp = wave / KS, ks = wave % KS;
  const int g0 = grp * G;                        // first output tile of the group, within the block
  const int nt0 = nbk * NWT + g0;
  const int ng = grp < NG ? max(0, min(min(G, NWT - g0), NT16 - nt0)) : 0;
  const int my_begin = t_begin + (int)((int64_t)ks * L / KS), my_end = t_begin + (int)((int64_t)(ks + 1) * L / KS);
  const unsigned char* w_src[G];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const int v = min(nt0 + g, NT16 - 1);
    if (GLU) w_src[g] = ((v & 1) ? Wp2 : Wp) + (size_t)(v >> 1) * KT * 1024 + lane * 16;
    else w_src[g] = Wp + (size_t)v * KT * 1024 + lane * 16;
  }
  uint4 wq[2][G];
  if (ng > 0 && my_begin < my_end) {
#pragma unroll
    for (int d = 0; d < 2; ++d)
#pragma unroll
      for (int g = 0; g < G; ++g)
        wq[d][g] = *reinterpret_cast<const uint4*>(w_src[g] + (size_t)min(my_begin + d, my_end - 1) * 1024);
  }

  // codes of all tokens for tiles t_begin .. t_end: wave w stages rows w, w + 16, ...
  {
    uint4 v[MT][4];
#pragma unroll
    for (int r = 0; r < MT; ++r) {
      const unsigned char* src = A + (size_t)min(wave + GR_WAVES * r, M - 1) * a_row_bytes + (size_t)t_begin * TB;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int pc = lane + 64 * j;
        v[r][j] = make_uint4(0u, 0u, 0u, 0u);
        if (pc < ppr) v[r][j] = *reinterpret_cast<const uint4*>(src + pc * 16);
      }
    }
#pragma unroll
    for (int r = 0; r < MT; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int pc = lane + 64 * j;
        if (pc < ppr) *reinterpret_cast<uint4*>(gr_smem + (wave + GR_WAVES * r) * pitch + pc * 16) = v[r][j];
      }
  }
  __syncthreads();

  v4i acc[G][MT];
#pragma unroll
  for (int g = 0; g < G; ++g)
#pragma unroll
    for (int b = 0; b < MT; ++b) acc[g][b] = (v4i){0, 0, 0, 0};
  if (ng > 0) {
    const unsigned char* xrow = gr_smem + li * pitch + lg * (A4 ? 32 : 64);
    for (int t0 = my_begin; t0 < my_end; t0 += 2) {
#pragma unroll
      for (int d = 0; d < 2; ++d) {
        const int t = t0 + d;
        if (t < my_end) {                        // wave-uniform
          uint4 wc[G];
#pragma unroll
          for (int g = 0; g < G; ++g) wc[g] = wq[d][g];
          if (t + 2 < my_end) {
#pragma unroll
            for (int g = 0; g < G; ++g)
              wq[d][g] = *reinterpret_cast<const uint4*>(w_src[g] + (size_t)(t + 2) * 1024);
          }
          const unsigned char* xb = xrow + (t - t_begin) * TB;
#pragma unroll
          for (int t4 = 0; t4 < 4; ++t4) {
            v4i xo[MT];
#pragma unroll
            for (int b = 0; b < MT; ++b) {
              if (A4) {
                // a lane's 64 channels = 8 words; MFMA step t4 takes words 2*t4 and 2*t4+1
                const uint2 v = *reinterpret_cast<const uint2*>(xb + b * 16 * pitch + t4 * 8);
                xo[b] = (v4i){(int)((v.x << 4) & 0xF0F0F0F0u), (int)(v.x & 0xF0F0F0F0u),
                              (int)((v.y << 4) & 0xF0F0F0F0u), (int)(v.y & 0xF0F0F0F0u)};
              } else {
                xo[b] = *reinterpret_cast<const v4i*>(xb + b * 16 * pitch + t4 * 16);
              }
            }
#pragma unroll
            for (int g = 0; g < G; ++g) {
              if (g < ng) {                      // wave-uniform
                const u32 w = t4 == 0 ? wc[g].x : t4 == 1 ? wc[g].y : t4 == 2 ? wc[g].z : wc[g].w;
                const v4i wo = (v4i){(int)((w << 6) & 0xC0C0C0C0u), (int)((w << 4) & 0xC0C0C0C0u),
                                     (int)((w << 2) & 0xC0C0C0C0u), (int)(w & 0xC0C0C0C0u)};
#pragma unroll
                for (int b = 0; b < MT; ++b)
                  acc[g][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wo, xo[b], acc[g][b], 0, 0, 0);
              }
            }
          }
        }
      }
    }
  }

  // Sums of the block, where the codes were.  Parts 1 .. KS-1 of every group leave their
  // accumulators in fragment order (one KB per tile, lane-contiguous); part 0 adds them to its own
  // and writes the totals as int32 [MT * 16 tokens][NWT * 16 outputs (+ 4)] behind them.
  const int OP = NWT * 16 + 4;                   // row pitch in words
  v4i* parts = reinterpret_cast<v4i*>(gr_smem);  // [working wave][g][b][lane]
  int32_t* sums = reinterpret_cast<int32_t*>(gr_smem) + (size_t)NG * KS * G * MT * 256;
  __syncthreads();
  if (ks != 0 && ng > 0) {
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
      for (int b = 0; b < MT; ++b) parts[((wave * G + g) * MT + b) * 64 + lane] = acc[g][b];
  }
  __syncthreads();
  if (ks == 0 && ng > 0) {
    for (int k = 1; k < KS; ++k)
#pragma unroll
      for (int g = 0; g < G; ++g)
#pragma unroll
        for (int b = 0; b < MT; ++b) acc[g][b] += parts[(((wave + k) * G + g) * MT + b) * 64 + lane];
#pragma unroll
    for (int g = 0; g < G; ++g)
      if (g < ng)
#pragma unroll
        for (int b = 0; b < MT; ++b)
          *reinterpret_cast<v4i*>(sums + (b * 16 + li) * OP + (g0 + g) * 16 + 4 * lg) = acc[g][b];
  }
  __syncthreads();

  const float alpha = alpha_p[0];
  constexpr int SHIFT = A4 ? 10 : 6;
  if constexpr (GLU) {
    // one thread per token and 4 consecutive outputs of one of the block's NWT / 2 tile pairs
    const float alpha2 = alpha2_p[0];
    uint16_t* H = reinterpret_cast<uint16_t*>(Y);
    const int qpr = (NWT >> 1) * 4;
    for (int i = tid; i < M * qpr; i += GR_THREADS) {
      const int m = i / qpr, c = (i % qpr) * 4;
      const int n = nbk * (NWT >> 1) * 16 + c;
      if (n >= N) continue;
      const int col = ((c >> 4) << 5) + (c & 15);          // the gate tile's columns; the up tile's are 16 further
      const v4i vg = *reinterpret_cast<const v4i*>(sums + m * OP + col);
      const v4i vu = *reinterpret_cast<const v4i*>(sums + m * OP + col + 16);
      const float d = scale[m];
      uint16_t hv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float g = ((float)(vg[r] >> SHIFT) * d) * alpha;
        const float u = ((float)(vu[r] >> SHIFT) * d) * alpha2;
        const float rl = fmaxf(g, 0.0f);
        const float rr = rl * rl;
        hv[r] = bl_f32_to_bf16_rne(u * rr);
      }
      const size_t o = (size_t)m * N + n;
      if ((N & 3) == 0) {
        *reinterpret_cast<uint2*>(H + o) = make_uint2((u32)hv[0] | ((u32)hv[1] << 16), (u32)hv[2] | ((u32)hv[3] << 16));
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (n + r < N) H[o + r] = hv[r];
      }
    }
    return;
  }
  // one thread per token and 4 consecutive outputs of the block's NWT * 16
  const int qpr = NWT * 4;                       // groups of 4 outputs per row
  for (int i = tid; i < M * qpr; i += GR_THREADS) {
    const int m = i / qpr, c = (i % qpr) * 4;
    const int n = nbk * NWT * 16 + c;
    if (n >= N) continue;
    const v4i v = *reinterpret_cast<const v4i*>(sums + m * OP + c);
    const size_t o = (size_t)m * N + n;
    if (S == 1) {
      const int iv[4] = {v[0] >> SHIFT, v[1] >> SHIFT, v[2] >> SHIFT, v[3] >> SHIFT};
      gd_store4(Y, y_bf16, acc_out, o, n, N, iv, scale[m], alpha);
    } else {
      int32_t* p = partial + (size_t)split * M * N + o;
      if ((N & 3) == 0) {
        *reinterpret_cast<v4i*>(p) = v;
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (n + r < N) p[r] = v[r];
      }
    }
  }
}

// Sum S integer partials, shift back, rescale.  One thread per 4 consecutive outputs.
__global__ __launch_bounds__(GD_THREADS) void decode_reduce_kernel(
    const int32_t* __restrict__ partial, int S, int M, int N, int shift,
    const float* __restrict__ scale, const float* __restrict__ alpha_p, void* __restrict__ Y,
    int y_bf16, int32_t* __restrict__ acc_out) {
  const int nq = (N + 3) >> 2;
  const int64_t id = (int64_t)blockIdx.x * GD_THREADS + threadIdx.x;
  if (id >= (int64_t)M * nq) return;
  const int m = (int)(id / nq), n = (int)(id % nq) * 4;
  int iv[4] = {0, 0, 0, 0};
  const bool vec = (N & 3) == 0;
  for (int s0 = 0; s0 < S; s0 += 8) {               // 8 independent loads in flight
    int4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int32_t* p = partial + ((size_t)min(s0 + j, S - 1) * M + m) * N + n;
      if (vec) v[j] = *reinterpret_cast<const int4*>(p);
      else v[j] = make_int4(p[0], n + 1 < N ? p[1] : 0, n + 2 < N ? p[2] : 0, n + 3 < N ? p[3] : 0);
    }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s0 + j < S) { iv[0] += v[j].x; iv[1] += v[j].y; iv[2] += v[j].z; iv[3] += v[j].w; }
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) iv[r] >>= shift;
  gd_store4(Y, y_bf16, acc_out, (size_t)m * N + n, n, N, iv, scale[m], alpha_p[0]);
}

// Kernel choice.  Up to 16 tokens (one MFMA tile of tokens) with enough output tiles to fill the
// chip: one 16-output tile per block, no split of K, one launch.  Up to 16 tokens and few outputs:
// 64 outputs per block and K split until the grid is large.  More tokens: codes resident in LDS.
static bool gd_single_tile(int M, int N) { return M <= 16 && (N + 15) / 16 >= 128; }
// resident kernel: tiles of K per slice so that 16 * MT rows of codes fit
static int gr_slice_tiles(int MT, bool a4) { return GR_X_BYTES / (MT * 16) / (a4 ? 128 : 256); }
static int gd_pick_split(int M, int N, int KT, bool a4) {
  if (gd_single_tile(M, N)) return 1;
  if (M > 16) {
    const int MT = M > 32 ? 4 : 2;
    const int tmax = gr_slice_tiles(MT, a4);
    return (KT + tmax - 1) / tmax;
  }
  const int NB = (N + GD_BN - 1) / GD_BN;
  int S = 1;
  while (NB * S < 512 && S * 2 <= KT && S < 32) S *= 2;
  return S;
}

size_t bl_gemm_decode_ws_bytes(int64_t M, int64_t N, int64_t K) {
  const int KT = (int)(bl_round_up(K, BL_KPAD) >> 8);
  // (the larger of the two code widths: the workspace is sized before the mode is known)
  const int S = max(gd_pick_split((int)M, (int)N, KT, false), gd_pick_split((int)M, (int)N, KT, true));
  return S > 1 ? (size_t)S * M * N * sizeof(int32_t) : 0;
}

static int gd_reduce(int S, int M, int N, int shift, const float* scale, const float* alpha, void* Y,
                     int ybf, int32_t* acc_out, void* ws, hipStream_t s) {
  const int64_t n_thr = (int64_t)M * ((N + 3) >> 2);
  decode_reduce_kernel<<<(unsigned)((n_thr + GD_THREADS - 1) / GD_THREADS), GD_THREADS, 0, s>>>(
      (const int32_t*)ws, S, M, N, shift, scale, alpha, Y, ybf, acc_out);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

template <int MT, bool A4, bool SINGLE>
static int gd_run(const void* q, const float* scale, int M, int Kp, const void* Wp,
                  const float* alpha, int N, void* Y, bl_dtype ydt, int32_t* acc_out, void* ws,
                  hipStream_t s) {
  const int KT = Kp >> 8;
  const int S = gd_pick_split(M, N, KT, A4);
  if (S > 1 && !ws) return BL_EWORKSPACE;
  const int ybf = ydt == BL_BF16 ? 1 : 0;
  if (SINGLE) {
    const int NB = (N + 15) / 16;
    const size_t smem = (size_t)4 * MT * 64 * sizeof(v4i);
    gemm_decode_kernel<MT, A4><<<(unsigned)(NB * S), GD_THREADS, smem, s>>>(
        (const unsigned char*)q, scale, M, Kp, (const unsigned char*)Wp, alpha, N, Y, ybf, acc_out,
        (int32_t*)ws, NB, S);
  } else {
    const int NB = (N + GD_BN - 1) / GD_BN;
    gemm_decode_rows_kernel<MT, A4><<<(unsigned)(NB * S), GD_THREADS, 0, s>>>(
        (const unsigned char*)q, scale, M, Kp, (const unsigned char*)Wp, alpha, N, Y, ybf, acc_out,
        (int32_t*)ws, NB, S);
  }
  BL_HIP_CHECK_LAUNCH();
  return S > 1 ? gd_reduce(S, M, N, A4 ? 10 : 6, scale, alpha, Y, ybf, acc_out, ws, s) : BL_OK;
}

template <int MT, bool A4>
static int gr_run(const void* q, const float* scale, int M, int Kp, const void* Wp,
                  const float* alpha, int N, void* Y, bl_dtype ydt, int32_t* acc_out, void* ws,
                  hipStream_t s) {
  const int KT = Kp >> 8, NT16 = (N + 15) / 16;
  const int S = gd_pick_split(M, N, KT, A4);
  if (S > 1 && !ws) return BL_EWORKSPACE;
  const int L = (KT + S - 1) / S;                        // tiles of the longest slice
  // output tiles per block: as few as still give at most one block per CU (one block takes most
  // of a CU's LDS), at most one per wave
  // (64 tokens: at most 12, so that the partial tiles and the sums fit the LDS together)
  const int nwt_max = MT == 4 ? 12 : GR_WAVES;
  int NWT = 1;
  while (NWT < nwt_max && ((NT16 + NWT - 1) / NWT) * S > bl_num_cus()) ++NWT;
  const int NBn = (NT16 + NWT - 1) / NWT;
  const int NG = (NWT + GR_G - 1) / GR_G;                // groups of output tiles, one per wave
  // parts of the slice per group: every part gets at least one tile; at most 8 working waves (two
  // per SIMD keep the matrix unit busy, and their sums must fit beside each other in LDS)
  const int KS = max(1, min(max(1, 8 / NG), KT / S));
  const size_t smem = max((size_t)MT * 16 * ((size_t)L * (A4 ? 128 : 256) + 16),
                          (size_t)NG * KS * GR_G * MT * 1024 + (size_t)MT * 16 * (NWT * 16 + 4) * sizeof(int32_t));
  auto kern = gemm_decode_resident_kernel<MT, A4>;
  // (the limit is raised once, to the most a launch can ask for: the codes' space plus row padding, or
  // eight waves' partial tiles plus the block's sums)
  BL_SET_MAX_LDS_ONCE((gemm_decode_resident_kernel<MT, A4>), GR_LDS_MAX);
  if (smem > GR_LDS_MAX) return BL_ESHAPE;
  const int ybf = ydt == BL_BF16 ? 1 : 0;
  kern<<<(unsigned)(NBn * S), GR_THREADS, smem, s>>>((const unsigned char*)q, scale, M, Kp,
                                                     (const unsigned char*)Wp, alpha, N, Y, ybf,
                                                     acc_out, (int32_t*)ws, NBn, S, NWT, KS, nullptr, nullptr);
  BL_HIP_CHECK_LAUNCH();
  return S > 1 ? gd_reduce(S, M, N, A4 ? 10 : 6, scale, alpha, Y, ybf, acc_out, ws, s) : BL_OK;
}

// Gate and up projection of 17 to 64 tokens with eq. 5 in the same launch (INT4 codes, both matrices in
// BL_W_GEMM): possible where all of K fits the LDS beside the tokens (no split across blocks).
static bool gr_glu_plan(int M, int N, int Kp, int& MT, int& NWT, int& KS, int& NBn, size_t& smem) {
  if (M <= 16 || M > 64) return false;
  MT = M > 32 ? 4 : 2;
  const int KT = Kp >> 8;
  if (KT > gr_slice_tiles(MT, true)) return false;
  const int NTv = 2 * ((N + 15) / 16);                   // gate and up tiles
  NWT = 2;
  while (NWT < 16 && (NTv + NWT - 1) / NWT > bl_num_cus()) NWT += 2;
  NBn = (NTv + NWT - 1) / NWT;
  const int NG = NWT / 2;                                // one tile pair per working wave
  for (KS = max(1, min(GR_WAVES / NG, KT)); KS >= 1; --KS) {
    smem = max((size_t)MT * 16 * ((size_t)KT * 128 + 16),
               (size_t)NG * KS * 2 * MT * 1024 + (size_t)MT * 16 * (NWT * 16 + 4) * sizeof(int32_t));
    if (smem <= GR_LDS_MAX) return bl_grid_ok(NBn);
  }
  return false;
}

bool bl_gemm_decode_glu_ok(int64_t M, int64_t N, int64_t K) {
  int MT, NWT, KS, NBn;
  size_t smem;
  if (M > 64 || N > ((int64_t)1 << 27)) return false;
  return gr_glu_plan((int)M, (int)N, (int)bl_round_up(K, BL_KPAD), MT, NWT, KS, NBn, smem);
}

template <int MT>
static int gr_go_glu(const void* q, const float* scale, int M, int Kp, const void* Wg, const float* ag, const void* Wu,
                     const float* au, int N, void* H, int NWT, int KS, int NBn, size_t smem, hipStream_t s) {
  BL_SET_MAX_LDS_ONCE((gemm_decode_resident_kernel<MT, true, true>), GR_LDS_MAX);
  gemm_decode_resident_kernel<MT, true, true><<<(unsigned)NBn, GR_THREADS, smem, s>>>(
      (const unsigned char*)q, scale, M, Kp, (const unsigned char*)Wg, ag, N, H, 1, nullptr, nullptr, NBn, 1, NWT, KS,
      (const unsigned char*)Wu, au);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

// q: INT4 nibble codes [M][Kp / 2] with their scales; H [M, N] bfloat16.
int bl_launch_gemm_decode_glu(const void* q, const float* scale, int64_t M, int64_t K, const void* Wg, const float* ag,
                              const void* Wu, const float* au, int64_t N, void* H, hipStream_t s) {
  int MT, NWT, KS, NBn;
  size_t smem;
  const int Kp = (int)bl_round_up(K, BL_KPAD);
  if (!gr_glu_plan((int)M, (int)N, Kp, MT, NWT, KS, NBn, smem)) return BL_EUNSUPPORTED;
  if (MT == 2) return gr_go_glu<2>(q, scale, (int)M, Kp, Wg, ag, Wu, au, (int)N, H, NWT, KS, NBn, smem, s);
  return gr_go_glu<4>(q, scale, (int)M, Kp, Wg, ag, Wu, au, (int)N, H, NWT, KS, NBn, smem, s);
}

// The fused INT4 linear is used for one bfloat16 token when the one-tile-per-block kernel would be
// (enough output tiles) and the row is 16-byte aligned and at most 8192 channels long.  (The kernel
// takes up to 4 tokens, but every block quantizes every token: measured per projection at 7B width,
// HIP-graph replays, fused against two launches: 7.6 / 8.9 us at one token, 9.2 / 9.1 at two,
// 12.0 / 9.1 at four.)
bool bl_gemv_a4_fused_ok(int64_t M, int64_t N, int64_t K) {
  const int64_t Kp = bl_round_up(K, BL_KPAD);
  return M == 1 && gd_single_tile((int)M, (int)N) && K % 8 == 0 && Kp <= 8 * GD_THREADS * GF_NV;
}

int bl_launch_gemv_a4_fused(const void* X, int64_t M, int64_t K, float eps, const void* Wp,
                            const float* alpha, int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out,
                            hipStream_t s) {
  if (!bl_gemv_a4_fused_ok(M, N, K)) return BL_EUNSUPPORTED;
  const int Kp = (int)bl_round_up(K, BL_KPAD);
  const size_t smem = (size_t)M * Kp;            // <= 32 KB
  gemv_a4_fused_kernel<<<(unsigned)((N + 15) / 16), GD_THREADS, smem, s>>>(
      (const uint16_t*)X, (int)M, (int)K, Kp, eps, (const unsigned char*)Wp, alpha, (int)N, Y,
      ydt == BL_BF16 ? 1 : 0, acc_out);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

int bl_launch_up_gated(const void* X, int64_t M, int64_t K, float eps, const void* Wr, const float* alpha,
                       int64_t N, const void* G, bl_dtype gdt, void* H, hipStream_t s) {
  const int Kp = (int)bl_round_up(K, BL_KPAD);
  if (M > 4 || K % 8 != 0 || Kp > 8 * GD_THREADS * GF_NV || M * Kp > 16384) return BL_EUNSUPPORTED;
  const int nch = (Kp + 4095) / 4096;            // 1 KB chunks of a weight row: 1 or 2
  const int mv = M <= 1 ? 1 : M <= 2 ? 2 : 4;
  // outputs per block: about two blocks per CU, at most one output per thread
  int npb = (int)((N + 2 * bl_num_cus() - 1) / (2 * bl_num_cus()));
  npb = max(16, min(GD_THREADS, npb));
  const unsigned grid = (unsigned)((N + npb - 1) / npb);
  const size_t smem = (size_t)M * Kp;
#define GU_CALL(MVV, NCHH)                                                                             \
  up_gated_kernel<MVV, NCHH><<<grid, GD_THREADS, smem, s>>>((const uint16_t*)X, (int)M, (int)K, Kp, eps, \
                                                          (const u32*)Wr, alpha, (int)N, G,            \
                                                          gdt == BL_F32 ? 1 : 0, (uint16_t*)H, npb)
  if (nch == 1) {
    if (mv == 1) GU_CALL(1, 1);
    else if (mv == 2) GU_CALL(2, 1);
    else GU_CALL(4, 1);
  } else {
    if (mv == 1) GU_CALL(1, 2);
    else GU_CALL(2, 2);                          // (M * Kp <= 16384: at most 2 tokens here)
  }
#undef GU_CALL
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

// The fused top-K + INT8 linear: one bfloat16 token whose keys fit the register kernel, enough
// output tiles for the one-tile-per-block kernel.
bool bl_gemv_a8_fused_ok(int64_t M, int64_t N, int64_t K) {
  return M == 1 && gd_single_tile(1, (int)N) && K % 4 == 0 && bl_round_up(K, BL_KPAD) <= 12288;
}

int bl_launch_gemv_a8_fused(const void* X, int64_t K, int64_t topk, float eps, const void* Wp,
                            const float* alpha, int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out,
                            hipStream_t s) {
  if (!bl_gemv_a8_fused_ok(1, N, K)) return BL_EUNSUPPORTED;
  const int Kp = (int)bl_round_up(K, BL_KPAD);
  const int cpw = (Kp / 256 + 3) / 4;
  const unsigned grid = (unsigned)((N + 15) / 16);
  const int ybf = ydt == BL_BF16 ? 1 : 0;
#define GF_A8(CPW)                                                                                     \
  gemv_a8_fused_kernel<CPW><<<grid, GD_THREADS, (size_t)Kp, s>>>(                                      \
      (const uint16_t*)X, (int)K, Kp, (int)topk, eps, (const unsigned char*)Wp, alpha, (int)N, Y, ybf, acc_out)
  if (cpw <= 4) GF_A8(4);
  else if (cpw <= 8) GF_A8(8);
  else GF_A8(12);
#undef GF_A8
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

int bl_launch_gemm_decode(const void* q, const float* scale, bl_act_mode mode, int64_t M,
                          int64_t K, const void* Wp, const float* alpha, int64_t N, void* Y,
                          bl_dtype ydt, int32_t* acc_out, void* ws, hipStream_t s) {
  const int Kp = (int)bl_round_up(K, BL_KPAD);
  const bool a4 = mode == BL_ACT_INT4_ABSMEAN;
  // up to 16 tokens whose codes fit the LDS: the persistent one-launch kernel
  if (bl_gemv_stream_ok(M, N, K, false))
    return bl_launch_gemv_stream(q, scale, a4, M, K, Wp, alpha, N, Y, ydt, acc_out, s);
#define GD_ARGS q, scale, (int)M, Kp, Wp, alpha, (int)N, Y, ydt, acc_out, ws, s
  if (gd_single_tile((int)M, (int)N)) return a4 ? gd_run<1, true, true>(GD_ARGS) : gd_run<1, false, true>(GD_ARGS);
  if (M <= 16) return a4 ? gd_run<1, true, false>(GD_ARGS) : gd_run<1, false, false>(GD_ARGS);
  if (M <= 32) return a4 ? gr_run<2, true>(GD_ARGS) : gr_run<2, false>(GD_ARGS);
  return a4 ? gr_run<4, true>(GD_ARGS) : gr_run<4, false>(GD_ARGS);
#undef GD_ARGS
}

// ---------------------------------------------------------------- sparse row-skipping GEMV
// Block = 4 waves, one 512-output column block and one slice of K.  The block first lists, in LDS,
// the channels of its slice with a non-zero code in at least one token (ballot compaction; padded
// to a multiple of 4 entries with a valid channel and code 0), and per token the codes of the
// listed channels packed 4 to a word.  Then a half wave reads one 128-byte weight row segment per
// load (32 lanes x 4 bytes); each lane gathers 4 listed rows, byte-transposes the four raw words so
// that a byte lane holds the four rows of one group of outputs, expands the 2-bit fields, and
// feeds v_dot4 with the four matching codes.  Rows of channels that are not listed are never read.
template <int MV>
__global__ __launch_bounds__(GD_THREADS) void gemv_sparse_kernel(
    const u32* __restrict__ Wk, int Np, int K, int Kp, const int8_t* __restrict__ q, int M, int S,
    int per, int32_t* __restrict__ partial) {
  extern __shared__ __align__(16) unsigned char gs_smem[];
  int* lst = reinterpret_cast<int*>(gs_smem);                    // [per + 4]
  u32* qp = reinterpret_cast<u32*>(gs_smem) + (per + 4);         // [MV][per / 4 + 1]
  const int qstride = (per >> 2) + 1;
  __shared__ int red[MV][16][32];
  __shared__ int wave_cnt[GD_THREADS / 64];
  __shared__ int base_sh;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int half = lane >> 5, hl = lane & 31;
  const int CB = Np >> 9;
  const int cb = blockIdx.x % CB, split = blockIdx.x / CB;
  const int k_begin = min(split * per, K), k_end = min(k_begin + per, K);   // per % 4 == 0
  const u32* wbase = Wk + (size_t)cb * K * 32 + hl;     // 128-byte row segments of this column block

  // ---- the slice's list
  if (tid == 0) base_sh = 0;
  __syncthreads();
  for (int k0 = k_begin; k0 < k_end; k0 += GD_THREADS) {
    const int k = k0 + tid;
    bool nz = false;
    if (k < k_end)
      for (int m = 0; m < M; ++m) nz |= q[(size_t)m * Kp + k] != 0;
    const uint64_t bal = __ballot(nz);
    if (lane == 0) wave_cnt[wave] = __popcll(bal);
    __syncthreads();
    int before = base_sh;
    for (int w = 0; w < wave; ++w) before += wave_cnt[w];
    if (nz) lst[before + __popcll(bal & ((1ull << lane) - 1ull))] = k;
    __syncthreads();
    if (tid == 0) base_sh += wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
    __syncthreads();
  }
  const int L = base_sh;
  const int groups = (L + 3) >> 2;                        // groups of 4 listed channels
  if (tid < 4 * groups - L) lst[L + tid] = -1;            // padding: marked, so that its code reads 0
  __syncthreads();
  for (int i = tid; i < M * groups; i += GD_THREADS) {
    const int m = i / groups, g = i % groups;
    u32 word = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int k = lst[4 * g + j];
      const u32 c = k >= 0 ? (u32)(uint8_t)q[(size_t)m * Kp + k] : 0u;
      word |= c << (8 * j);
    }
    qp[m * qstride + g] = word;
  }
  __syncthreads();
  if (tid < 4 * groups - L) lst[L + tid] = k_begin;       // (any valid channel: its code is 0)
  __syncthreads();

  int acc[MV][16];
#pragma unroll
  for (int m = 0; m < MV; ++m)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[m][j] = 0;

  for (int g = wave * 2 + half; g < groups; g += 8) {
    u32 w[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) w[r] = wbase[(size_t)lst[4 * g + r] * 32];
    // 4x4 byte transpose: x[b] = byte b of (w0, w1, w2, w3)
    const u32 t01l = __builtin_amdgcn_perm(w[1], w[0], 0x05010400u);  // w0.b0 w1.b0 w0.b1 w1.b1
    const u32 t01h = __builtin_amdgcn_perm(w[1], w[0], 0x07030602u);  // w0.b2 w1.b2 w0.b3 w1.b3
    const u32 t23l = __builtin_amdgcn_perm(w[3], w[2], 0x05010400u);
    const u32 t23h = __builtin_amdgcn_perm(w[3], w[2], 0x07030602u);
    u32 x[4];
    x[0] = __builtin_amdgcn_perm(t23l, t01l, 0x05040100u);
    x[1] = __builtin_amdgcn_perm(t23l, t01l, 0x07060302u);
    x[2] = __builtin_amdgcn_perm(t23h, t01h, 0x05040100u);
    x[3] = __builtin_amdgcn_perm(t23h, t01h, 0x07060302u);
    u32 qv[MV];
#pragma unroll
    for (int m = 0; m < MV; ++m) qv[m] = m < M ? qp[m * qstride + g] : 0u;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const u32 tw = (x[b] << (6 - 2 * j)) & 0xC0C0C0C0u;   // rows 0..3 of output 4b+j, times 64
#pragma unroll
        for (int m = 0; m < MV; ++m)
          acc[m][4 * b + j] = __builtin_amdgcn_sdot4((int)tw, (int)qv[m], acc[m][4 * b + j], false);
      }
    }
  }
  // the two half waves hold different channels of the same outputs
#pragma unroll
  for (int m = 0; m < MV; ++m)
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[m][j] += __shfl_xor(acc[m][j], 32, 64);
  // waves 1..3 add into LDS (integer adds: any order gives the same sum), wave 0 finishes
  for (int i = tid; i < MV * 16 * 32; i += GD_THREADS) (&red[0][0][0])[i] = 0;
  __syncthreads();
  if (wave > 0 && half == 0) {
#pragma unroll
    for (int m = 0; m < MV; ++m)
#pragma unroll
      for (int j = 0; j < 16; ++j) atomicAdd(&red[m][j][hl], acc[m][j]);
  }
  __syncthreads();
  if (wave == 0 && half == 0) {
#pragma unroll
    for (int m = 0; m < MV; ++m) {
      if (m >= M) break;
      int32_t* p = partial + ((size_t)split * M + m) * Np + cb * 512 + hl * 16;
#pragma unroll
      for (int j = 0; j < 16; ++j) p[j] = acc[m][j] + red[m][j][hl];
    }
  }
}

// Partials of the sparse path are [S][M][Np]; reduce + rescale into Y[M][N].
__global__ __launch_bounds__(GD_THREADS) void sparse_reduce_kernel(
    const int32_t* __restrict__ partial, int S, int M, int N, int Np,
    const float* __restrict__ scale, const float* __restrict__ alpha_p, void* __restrict__ Y,
    int y_bf16, int32_t* __restrict__ acc_out) {
  const int nq = (N + 3) >> 2;
  const int64_t id = (int64_t)blockIdx.x * GD_THREADS + threadIdx.x;
  if (id >= (int64_t)M * nq) return;
  const int m = (int)(id / nq), n = (int)(id % nq) * 4;
  int iv[4] = {0, 0, 0, 0};
  for (int s0 = 0; s0 < S; s0 += 8) {               // 8 independent loads in flight
    int4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)                     // Np is a multiple of 512: always aligned
      v[j] = *reinterpret_cast<const int4*>(partial + ((size_t)min(s0 + j, S - 1) * M + m) * Np + n);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (s0 + j < S) { iv[0] += v[j].x; iv[1] += v[j].y; iv[2] += v[j].z; iv[3] += v[j].w; }
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) iv[r] >>= 6;
  gd_store4(Y, y_bf16, acc_out, (size_t)m * N + n, n, N, iv, scale[m], alpha_p[0]);
}

#define GS_SPLIT 32
// channels per block: K dealt to GS_SPLIT slices, a multiple of 4
static int gs_per(int64_t K) { return (int)(((K + GS_SPLIT - 1) / GS_SPLIT + 3) & ~(int64_t)3); }

size_t bl_gemv_sparse_ws_bytes(int64_t M, int64_t N, int64_t K) {
  (void)K;
  return (size_t)GS_SPLIT * M * bl_round_up(N, 512) * 4;          // integer partials
}

int bl_launch_gemv_sparse(const void* q, const float* scale, int64_t M, int64_t K,
                          const void* Wk, const float* alpha, int64_t N, void* Y, bl_dtype ydt,
                          int32_t* acc_out, void* ws, hipStream_t s) {
  if (!ws) return BL_EWORKSPACE;
  if (M > 8) return BL_EUNSUPPORTED;
  const int Kp = (int)bl_round_up(K, BL_KPAD), Np = (int)bl_round_up(N, 512);
  const int per = gs_per(K);
  int32_t* partial = (int32_t*)ws;
  const int CB = Np >> 9;
  const unsigned grid = (unsigned)(CB * GS_SPLIT);
  const int MV = M <= 1 ? 1 : M <= 4 ? 4 : 8;
  const size_t smem = (size_t)(per + 4) * 4 + (size_t)MV * (per / 4 + 1) * 4;
  if (smem > 48 * 1024) return BL_EUNSUPPORTED;           // K above 300000 channels
#define GS_CALL(MVV)                                                                               \
  gemv_sparse_kernel<MVV><<<grid, GD_THREADS, smem, s>>>((const u32*)Wk, Np, (int)K, Kp, (const int8_t*)q, \
                                                        (int)M, GS_SPLIT, per, partial)
  if (MV == 1) GS_CALL(1);
  else if (MV == 4) GS_CALL(4);
  else GS_CALL(8);
#undef GS_CALL
  BL_HIP_CHECK_LAUNCH();
  const int64_t n_thr = M * ((N + 3) >> 2);
  sparse_reduce_kernel<<<(unsigned)((n_thr + GD_THREADS - 1) / GD_THREADS), GD_THREADS, 0, s>>>(
      partial, GS_SPLIT, (int)M, (int)N, Np, scale, alpha, Y, ydt == BL_BF16 ? 1 : 0, acc_out);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}
