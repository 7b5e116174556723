// Prefill GEMM of the W1.58A4 and sparse W1.58A8 linears (eq. 6 and eq. 1 of the paper):
//   acc[m, n] = sum_k q[m, k] * T[n, k]   (exact int32 on v_mfma_i32_16x16x64_i8)
//   Y[m, n]   = (float(acc) * d[m]) * alpha
// Activations arrive packed (INT4 nibbles or INT8), weights 2-bit packed in 16 x 256 tiles.
// Both are expanded to int8 while they are copied into LDS, without sign extension:
//   an INT4 nibble is moved to the top of its byte  -> 16 * q,
//   a 2-bit ternary field is moved to the top of its byte -> 64 * T,
// so the MFMA accumulates 1024 * acc (64 * acc for INT8 activations), which is shifted back
// exactly in the epilogue.  |1024 * acc| <= 8 * 11008 * 1024 < 2^31.
#include "common.h"

#define GP_THREADS 256
#define GP_BK 128     // bytes (= int8 channels) per LDS row per stage

template <int BM, int BN>
struct GpSmem {
  static constexpr int a_bytes = BM * GP_BK;
  static constexpr int b_bytes = BN * GP_BK;
  static constexpr int stage = a_bytes + b_bytes;
  static constexpr int total = 2 * stage;
};

__device__ __forceinline__ int gp_lds_off(int row, int chunk) {
  return row * GP_BK + ((chunk ^ (row & 7)) << 4);
}

template <int BM, int BN, bool A4>
__global__ __launch_bounds__(GP_THREADS, 1) void gemm_prefill_kernel(
    const unsigned char* __restrict__ A, const float* __restrict__ scale, int M, int Kp,
    const unsigned char* __restrict__ Wp, const float* __restrict__ alpha_p, int N, void* __restrict__ Y,
    int y_bf16, int32_t* __restrict__ acc_out, int MT, int NTB) {
  constexpr int WM = BM / 2, WN = BN / 2;        // wave tile
  constexpr int TM = WM / 16, TN = WN / 16;      // 16x16 MFMA tiles per wave
  constexpr int PA = A4 ? 4 : 8;                 // 16-byte pieces per activation row per stage
  constexpr int LA = BM * PA / GP_THREADS;       // activation loads per thread per stage
  constexpr int LB = BN * 2 / GP_THREADS;        // weight loads per thread per stage
  extern __shared__ __align__(16) unsigned char gp_smem[];

  // ---- block -> tile: spread consecutive tiles over one XCD (blocks are dealt round-robin to
  // the 8 XCDs), then walk the tile grid in groups of 4 token tiles so that an XCD's 32
  // concurrent tiles share activations and weights in its L2.
  int pid = blockIdx.x;
  {
    const int nb = gridDim.x, q = nb >> 3, rmd = nb & 7, xcd = pid & 7, loc = pid >> 3;
    pid = xcd * q + min(xcd, rmd) + loc;
  }
  constexpr int GM = 4;
  const int per_group = GM * NTB;
  const int group = pid / per_group, in_group = pid % per_group;
  const int first_m = group * GM;
  const int gsz = min(MT - first_m, GM);
  const int mt = first_m + in_group % gsz;
  const int ntb = in_group / gsz;
  const int m0 = mt * BM, n0 = ntb * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int li = lane & 15, lg = lane >> 4;
  const int n_tiles16 = (N + 15) >> 4;
  const int k_tiles = Kp >> 8;
  const int a_row_bytes = A4 ? (Kp >> 1) : Kp;
  const int nk = Kp / GP_BK;

  // ---- per-thread global source pointers and LDS destinations
  const unsigned char* a_src[LA];
  int a_dst[LA];
#pragma unroll
  for (int j = 0; j < LA; ++j) {
    const int idx = tid + GP_THREADS * j;
    const int cq = idx % PA, row = idx / PA;
    const int gr = min(m0 + row, M - 1);
    a_src[j] = A + (size_t)gr * a_row_bytes + cq * 16;
    a_dst[j] = A4 ? gp_lds_off(row, 2 * cq) : gp_lds_off(row, cq);
  }
  const unsigned char* b_src[LB];
  int b_row[LB], b_gg[LB];
#pragma unroll
  for (int j = 0; j < LB; ++j) {
    const int idx = tid + GP_THREADS * j;
    const int i = idx & 15, gg = (idx >> 4) & 1, ntl = idx >> 5;
    const int nt = min((n0 >> 4) + ntl, n_tiles16 - 1);
    b_src[j] = Wp + ((size_t)nt * k_tiles) * 1024 + (gg * 16 + i) * 16;
    b_row[j] = ntl * 16 + i;
    b_gg[j] = gg;
  }

  uint4 a_reg[LA], b_reg[LB];
  auto load_global = [&](int ks) {
#pragma unroll
    for (int j = 0; j < LA; ++j)
      a_reg[j] = *reinterpret_cast<const uint4*>(a_src[j] + (size_t)ks * (A4 ? 64 : 128));
#pragma unroll
    for (int j = 0; j < LB; ++j)
      b_reg[j] = *reinterpret_cast<const uint4*>(b_src[j] + (size_t)(ks >> 1) * 1024 + (ks & 1) * 512);
  };
  auto store_lds = [&](int stage) {
    unsigned char* as = gp_smem + stage * GpSmem<BM, BN>::stage;
    unsigned char* bs = as + GpSmem<BM, BN>::a_bytes;
#pragma unroll
    for (int j = 0; j < LA; ++j) {
      if (A4) {
        const u32 x[4] = {a_reg[j].x, a_reg[j].y, a_reg[j].z, a_reg[j].w};
        const int idx = tid + GP_THREADS * j;
        const int cq = idx % PA, row = idx / PA;
        uint4 c0, c1;
        c0.x = (x[0] << 4) & 0xF0F0F0F0u; c0.y = x[0] & 0xF0F0F0F0u;
        c0.z = (x[1] << 4) & 0xF0F0F0F0u; c0.w = x[1] & 0xF0F0F0F0u;
        c1.x = (x[2] << 4) & 0xF0F0F0F0u; c1.y = x[2] & 0xF0F0F0F0u;
        c1.z = (x[3] << 4) & 0xF0F0F0F0u; c1.w = x[3] & 0xF0F0F0F0u;
        *reinterpret_cast<uint4*>(as + a_dst[j]) = c0;
        *reinterpret_cast<uint4*>(as + gp_lds_off(row, 2 * cq + 1)) = c1;
      } else {
        *reinterpret_cast<uint4*>(as + a_dst[j]) = a_reg[j];
      }
    }
#pragma unroll
    for (int j = 0; j < LB; ++j) {
      const u32 w[4] = {b_reg[j].x, b_reg[j].y, b_reg[j].z, b_reg[j].w};
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        uint4 c;
        c.x = (w[t] << 6) & 0xC0C0C0C0u;
        c.y = (w[t] << 4) & 0xC0C0C0C0u;
        c.z = (w[t] << 2) & 0xC0C0C0C0u;
        c.w = w[t] & 0xC0C0C0C0u;
        *reinterpret_cast<uint4*>(bs + gp_lds_off(b_row[j], 4 * b_gg[j] + t)) = c;
      }
    }
  };

  v4i acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b) acc[a][b] = (v4i){0, 0, 0, 0};

  load_global(0);
  store_lds(0);
  __syncthreads();

  for (int ks = 0; ks < nk; ++ks) {
    const int stage = ks & 1;
    if (ks + 1 < nk) load_global(ks + 1);
    const unsigned char* as = gp_smem + stage * GpSmem<BM, BN>::stage;
    const unsigned char* bs = as + GpSmem<BM, BN>::a_bytes;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      v4i wf[TN], xf[TM];
#pragma unroll
      for (int a = 0; a < TN; ++a)
        wf[a] = *reinterpret_cast<const v4i*>(bs + gp_lds_off(wn * WN + a * 16 + li, 4 * sub + lg));
#pragma unroll
      for (int b = 0; b < TM; ++b)
        xf[b] = *reinterpret_cast<const v4i*>(as + gp_lds_off(wm * WM + b * 16 + li, 4 * sub + lg));
#pragma unroll
      for (int a = 0; a < TN; ++a)
#pragma unroll
        for (int b = 0; b < TM; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wf[a], xf[b], acc[a][b], 0, 0, 0);
    }
    if (ks + 1 < nk) store_lds(stage ^ 1);
    __syncthreads();
  }

  // ---- epilogue: lane holds token m = ... + li and 4 consecutive outputs n = ... + 4*lg + r
  const float alpha = alpha_p[0];
  constexpr int SHIFT = A4 ? 10 : 6;
  const bool vec_ok = (N & 3) == 0;
#pragma unroll
  for (int b = 0; b < TM; ++b) {
    const int m = m0 + wm * WM + b * 16 + li;
    if (m >= M) continue;
    const float d = scale[m];
#pragma unroll
    for (int a = 0; a < TN; ++a) {
      const int n = n0 + wn * WN + a * 16 + 4 * lg;
      if (n >= N) continue;
      int iv[4];
      float fv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        iv[r] = acc[a][b][r] >> SHIFT;                 // exact: the low bits are zero
        fv[r] = ((float)iv[r] * d) * alpha;
      }
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
  }
}

template <int BM, int BN, bool A4>
static int gp_launch(const void* q, const float* scale, int M, int Kp, const void* Wp,
                     const float* alpha, int N, void* Y, bl_dtype ydt, int32_t* acc_out,
                     hipStream_t s) {
  auto kern = gemm_prefill_kernel<BM, BN, A4>;
  constexpr int smem = GpSmem<BM, BN>::total;
  if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
    return BL_EHIP;
  const int MT = (M + BM - 1) / BM, NTB = (N + BN - 1) / BN;
  kern<<<(unsigned)(MT * NTB), GP_THREADS, smem, s>>>(
      (const unsigned char*)q, scale, M, Kp, (const unsigned char*)Wp, alpha, N, Y,
      ydt == BL_BF16 ? 1 : 0, acc_out, MT, NTB);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

int bl_launch_gemm_prefill(const void* q, const float* scale, bl_act_mode mode, int64_t M,
                           int64_t K, const void* Wp, const float* alpha, int64_t N, void* Y,
                           bl_dtype ydt, int32_t* acc_out, hipStream_t s) {
  const int Kp = (int)bl_round_up(K, BL_KPAD);
  const bool a4 = mode == BL_ACT_INT4_ABSMEAN;
  // Large problems take 256 x 256 tiles; small ones 128 x 128 so that the grid still covers the chip.
  const bool big = (M >= 1024 && N >= 1024);
  if (a4) {
    if (big) return gp_launch<256, 256, true>(q, scale, (int)M, Kp, Wp, alpha, (int)N, Y, ydt, acc_out, s);
    return gp_launch<128, 128, true>(q, scale, (int)M, Kp, Wp, alpha, (int)N, Y, ydt, acc_out, s);
  }
  if (big) return gp_launch<256, 256, false>(q, scale, (int)M, Kp, Wp, alpha, (int)N, Y, ydt, acc_out, s);
  return gp_launch<128, 128, false>(q, scale, (int)M, Kp, Wp, alpha, (int)N, Y, ydt, acc_out, s);
}
