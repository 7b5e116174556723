// FP4 (E2M1) activation variant of the W1.58A4 linear on the CDNA4 scaled FP4 matrix
// instruction (eq. 8-9 of the paper, one power-of-two scale per 32 channels):
//   Y[m, n] = alpha * sum over blocks b of 2^e[m, b] * sum_{k in b} v[m, k] * T[n, k]
// v_mfma_scale_f32_16x16x128_f8f6f4 multiplies 32 FP4 values per lane and applies one E8M0
// scale per lane and operand, which is exactly one 32-channel block: the block scales ride on
// the instruction, the weights use the neutral scale 2^0.  Ternary weights are exact in E2M1
// ({0, +1, -1} = nibbles 0000, 0010, 1010); a 2-bit field (b1 b0) becomes the nibble
// (b1 0 b0 0), two shifts and two masked merges per 8 weights, while the tile is copied to LDS.
// Accumulation is float32 inside the instruction (not bit-exact against a float64 reference).
//
// Block = 4 waves, 128 x 128 outputs, each wave 64 x 64 as 16x16 MFMA tiles (row operand =
// weights, column operand = tokens).  One K step is 256 channels: 128 bytes of FP4 per row.
#include "common.h"

#define GF_THREADS 256
#define GF_BM 128
#define GF_BN 128
#define GF_ROW 128           // bytes per LDS row (256 FP4 channels)

__device__ __forceinline__ int gf_lds_off(int row, int chunk) {
  return row * GF_ROW + ((chunk ^ (row & 7)) << 4);
}

// 16 ternary 2-bit fields -> two words of 8 E2M1 nibbles (even fields, odd fields)
__device__ __forceinline__ void gf_expand(u32 w, u32& even, u32& odd) {
  even = ((w << 2) & 0x88888888u) | ((w << 1) & 0x22222222u);
  odd = (w & 0x88888888u) | ((w >> 1) & 0x22222222u);
}

__global__ __launch_bounds__(GF_THREADS) void gemm_fp4_kernel(
    const unsigned char* __restrict__ A, const uint8_t* __restrict__ sc, int M, int Kp,
    const unsigned char* __restrict__ Wp, const float* __restrict__ alpha_p, int N,
    void* __restrict__ Y, int y_bf16, int NTB) {
  __shared__ __align__(16) unsigned char smem[(GF_BM + GF_BN) * GF_ROW];
  unsigned char* as = smem;
  unsigned char* bs = smem + GF_BM * GF_ROW;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int li = lane & 15, lg = lane >> 4;
  const int m0 = (blockIdx.x / NTB) * GF_BM, n0 = (blockIdx.x % NTB) * GF_BN;
  const int n_tiles16 = (N + 15) >> 4, k_tiles = Kp >> 8;
  const int a_row_bytes = Kp >> 1, sc_row = Kp >> 5;

  v4f acc[4][4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = (v4f){0.f, 0.f, 0.f, 0.f};

  for (int ks = 0; ks < k_tiles; ++ks) {
    // activations: 128 rows x 8 chunks of 16 bytes, straight copy
    uint4 av[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int idx = tid + GF_THREADS * j, row = idx >> 3, ch = idx & 7;
      const int gr = min(m0 + row, M - 1);
      av[j] = *reinterpret_cast<const uint4*>(A + (size_t)gr * a_row_bytes + ks * GF_ROW + ch * 16);
    }
    // weights: 8 tiles of 16 rows; one 16-byte piece = one row, 64 channels
    uint4 wv[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int idx = tid + GF_THREADS * j, ntl = idx >> 6, within = idx & 63;
      const int nt = min((n0 >> 4) + ntl, n_tiles16 - 1);
      wv[j] = *reinterpret_cast<const uint4*>(Wp + ((size_t)nt * k_tiles + ks) * 1024 + within * 16);
    }
    __syncthreads();                       // previous step's fragments have been read
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int idx = tid + GF_THREADS * j, row = idx >> 3, ch = idx & 7;
      *reinterpret_cast<uint4*>(as + gf_lds_off(row, ch)) = av[j];
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int idx = tid + GF_THREADS * j, ntl = idx >> 6, within = idx & 63;
      const int g = within >> 4, row = ntl * 16 + (within & 15);
      uint4 c0, c1;
      gf_expand(wv[j].x, c0.x, c0.y);
      gf_expand(wv[j].y, c0.z, c0.w);
      gf_expand(wv[j].z, c1.x, c1.y);
      gf_expand(wv[j].w, c1.z, c1.w);
      *reinterpret_cast<uint4*>(bs + gf_lds_off(row, 2 * g)) = c0;
      *reinterpret_cast<uint4*>(bs + gf_lds_off(row, 2 * g + 1)) = c1;
    }
    __syncthreads();
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      v8i wf[4], xf[4];
      int xs[4];
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const v4i t = *reinterpret_cast<const v4i*>(bs + gf_lds_off(wn * 64 + a * 16 + li, 4 * sub + lg));
        wf[a] = (v8i){t[0], t[1], t[2], t[3], 0, 0, 0, 0};
      }
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const int row = wm * 64 + b * 16 + li;
        const v4i t = *reinterpret_cast<const v4i*>(as + gf_lds_off(row, 4 * sub + lg));
        xf[b] = (v8i){t[0], t[1], t[2], t[3], 0, 0, 0, 0};
        const int gr = min(m0 + row, M - 1);
        xs[b] = (int)sc[(size_t)gr * sc_row + ks * 8 + 4 * sub + lg];   // this lane's 32-channel block
      }
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
              wf[a], xf[b], acc[a][b], 4 /* A: FP4 */, 4 /* B: FP4 */, 0, 127 /* 2^0 */, 0, xs[b]);
    }
  }

  const float alpha = alpha_p[0];
  const bool vec_ok = (N & 3) == 0;
#pragma unroll
  for (int b = 0; b < 4; ++b) {
    const int m = m0 + wm * 64 + b * 16 + li;
    if (m >= M) continue;
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      const int n = n0 + wn * 64 + a * 16 + 4 * lg;
      if (n >= N) continue;
      float fv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) fv[r] = acc[a][b][r] * alpha;
      const size_t o = (size_t)m * N + n;
      if (vec_ok) {
        if (y_bf16) {
          uint2 p;
          p.x = (u32)bl_f32_to_bf16_rne(fv[0]) | ((u32)bl_f32_to_bf16_rne(fv[1]) << 16);
          p.y = (u32)bl_f32_to_bf16_rne(fv[2]) | ((u32)bl_f32_to_bf16_rne(fv[3]) << 16);
          *reinterpret_cast<uint2*>((uint16_t*)Y + o) = p;
        } else {
          *reinterpret_cast<float4*>((float*)Y + o) = make_float4(fv[0], fv[1], fv[2], fv[3]);
        }
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (n + r < N) {
            if (y_bf16) ((uint16_t*)Y)[o + r] = bl_f32_to_bf16_rne(fv[r]);
            else ((float*)Y)[o + r] = fv[r];
          }
        }
      }
    }
  }
}

int bl_launch_gemm_fp4(const void* q, const uint8_t* scale, int64_t M, int64_t K, const void* Wp,
                       const float* alpha, int64_t N, void* Y, bl_dtype ydt, hipStream_t s) {
  const int Kp = (int)bl_round_up(K, BL_KPAD);
  const int MT = (int)((M + GF_BM - 1) / GF_BM), NTB = (int)((N + GF_BN - 1) / GF_BN);
  gemm_fp4_kernel<<<(unsigned)(MT * NTB), GF_THREADS, 0, s>>>(
      (const unsigned char*)q, scale, (int)M, Kp, (const unsigned char*)Wp, alpha, (int)N, Y,
      ydt == BL_BF16 ? 1 : 0, NTB);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}
