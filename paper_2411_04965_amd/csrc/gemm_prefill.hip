// Prefill GEMM of the W1.58A4 and sparse W1.58A8 linears (eq. 6 and eq. 1 of the paper):
//   acc[m, n] = sum_k q[m, k] * T[n, k]   (exact int32 on v_mfma_i32_16x16x64_i8)
//   Y[m, n]   = (float(acc) * d[m]) * alpha
// Activations arrive packed (INT4 nibbles or INT8), weights 2-bit packed in 16 x 256 tiles.
// Both are expanded to int8 while they are copied into LDS, without sign extension:
//   an INT4 nibble is moved to the top of its byte  -> 16 * q,
//   a 2-bit ternary field is moved to the top of its byte -> 64 * T,
// so the MFMA accumulates 1024 * acc (64 * acc for INT8 activations); the factor is a power of
// two and is folded exactly into the per-token scale in the epilogue.
// |1024 * acc| <= 8 * K * 1024 < 2^31 for K <= 32768.
//
// Block = 4 waves, tile BM x BN, each wave (BM/2) x (BN/2) as 16x16 MFMA tiles; the MFMA's
// row operand is the weight fragment and its column operand the token fragment, so a lane
// ends up with 4 consecutive outputs n of one token.  K advances 128 channels per step through
// two LDS stages.  One step is one straight-line block: the first half multiplies k 0..63
// while it expands the prefetched global data into the other stage and reads the fragments
// of the second half; after the barrier the second half multiplies k 64..127 while it issues
// the global loads two steps ahead and reads the first fragments of the next step.
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

__device__ __forceinline__ u32 gp_pack_bf16(float lo, float hi) {
  u32 r;
  asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
  return r;
}

template <int BM, int BN, bool A4, bool VEC>
__global__ __launch_bounds__(GP_THREADS, 1) void gemm_prefill_kernel(
    const unsigned char* __restrict__ A, const float* __restrict__ scale, int M, int Kp,
    const unsigned char* __restrict__ Wp, const float* __restrict__ alpha_p, int N, void* __restrict__ Y,
    int y_bf16, int32_t* __restrict__ acc_out, int MT, int NTB) {
  constexpr int WM = BM / 2, WN = BN / 2;        // wave tile
  constexpr int TM = WM / 16, TN = WN / 16;      // 16x16 MFMA tiles per wave
  constexpr int PA = A4 ? 4 : 8;                 // 16-byte pieces per activation row per stage
  constexpr int LA = BM * PA / GP_THREADS;       // activation loads per thread per stage
  constexpr int LB = BN * 2 / GP_THREADS;        // weight loads per thread per stage
  constexpr int STAGE = GpSmem<BM, BN>::stage;
  constexpr int A_BYTES = GpSmem<BM, BN>::a_bytes;
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

  // ---- global sources: one uniform base per operand plus a small per-lane offset that is
  // rebuilt for every load (two VALU operations) instead of being kept in registers.
  //   activations: load j of a thread covers row (tid / PA) + RPJ * j, 16-byte piece tid % PA
  //   weights:     load j covers 16-row tile (tid / 32) + 8 * j, row tid % 16, k-group (tid / 16) % 2
  constexpr int RPJ = GP_THREADS / PA;
  constexpr int KSB = A4 ? 64 : 128;             // activation bytes per row per step
  const unsigned char* a_base = A + (size_t)m0 * a_row_bytes;
  const u32 a_row0 = tid / PA, a_piece = (tid % PA) * 16;
  const u32 a_row_max = (u32)(M - 1 - m0);       // rows past the end of X re-read the last row
  const unsigned char* b_base = Wp + (size_t)(n0 >> 4) * k_tiles * 1024;
  const u32 b_tile0 = tid >> 5, b_piece = (((tid >> 4) & 1) * 16 + (tid & 15)) * 16;
  const u32 b_tile_max = (u32)(n_tiles16 - 1 - (n0 >> 4));
  const u32 b_tile_bytes = (u32)k_tiles * 1024;
  const int a_dst0 = A4 ? gp_lds_off(a_row0, 2 * (tid % PA)) : gp_lds_off(a_row0, tid % PA);
  const int b_dst0 = A_BYTES + gp_lds_off(b_tile0 * 16 + (tid & 15), 4 * ((tid >> 4) & 1));

  uint4 a_reg[LA], b_reg[LB];
  auto load_a = [&](int j, int ks) {
    const u32 off = min(a_row0 + RPJ * j, a_row_max) * (u32)a_row_bytes + a_piece;
    a_reg[j] = *reinterpret_cast<const uint4*>(a_base + (size_t)ks * KSB + off);
  };
  auto load_b = [&](int j, int ks) {
    const u32 off = min(b_tile0 + 8 * j, b_tile_max) * b_tile_bytes + b_piece;
    b_reg[j] = *reinterpret_cast<const uint4*>(b_base + (size_t)ks * 512 + off);
  };
  // The expansion of one stage is cut into NWR_A + NWR_B single 16-byte LDS writes so that it
  // can be spread over the MFMA stream.  Rows of load j sit RPJ (resp. 128) rows below those of
  // load 0, a multiple of 8, so the swizzle is the same and the offset is an immediate.
  constexpr int NWR_A = A4 ? 2 * LA : LA;
  constexpr int NWR_B = 4 * LB;
  auto write_a = [&](unsigned char* st, int i) {
    if (A4) {
      const int j = i >> 1;
      const u32 x0 = (i & 1) ? a_reg[j].z : a_reg[j].x, x1 = (i & 1) ? a_reg[j].w : a_reg[j].y;
      uint4 c;
      c.x = (x0 << 4) & 0xF0F0F0F0u; c.y = x0 & 0xF0F0F0F0u;
      c.z = (x1 << 4) & 0xF0F0F0F0u; c.w = x1 & 0xF0F0F0F0u;
      *reinterpret_cast<uint4*>(st + j * (RPJ * GP_BK) + (a_dst0 ^ ((i & 1) << 4))) = c;
    } else {
      *reinterpret_cast<uint4*>(st + i * (RPJ * GP_BK) + a_dst0) =
          make_uint4(a_reg[i].x, a_reg[i].y, a_reg[i].z, a_reg[i].w);
    }
  };
  auto write_b = [&](unsigned char* st, int i) {
    const int j = i >> 2, t = i & 3;
    const u32 w = t == 0 ? b_reg[j].x : t == 1 ? b_reg[j].y : t == 2 ? b_reg[j].z : b_reg[j].w;
    uint4 c;
    c.x = (w << 6) & 0xC0C0C0C0u;
    c.y = (w << 4) & 0xC0C0C0C0u;
    c.z = (w << 2) & 0xC0C0C0C0u;
    c.w = w & 0xC0C0C0C0u;
    *reinterpret_cast<uint4*>(st + j * (128 * GP_BK) + (b_dst0 ^ (t << 4))) = c;
  };

  // fragment addresses: row = wave base + tile * 16 + li, chunk = 4 * sub + lg
  const int swz0 = ((lg) ^ (li & 7)) << 4, swz1 = ((4 + lg) ^ (li & 7)) << 4;
  const int xf_base = (wm * WM + li) * GP_BK;
  const int wf_base = A_BYTES + (wn * WN + li) * GP_BK;
  auto read_x = [&](int stage, int sub, int b) -> v4i {
    return *reinterpret_cast<const v4i*>(gp_smem + stage * STAGE + xf_base + b * (16 * GP_BK) + (sub ? swz1 : swz0));
  };
  auto read_w = [&](int stage, int sub, int a) -> v4i {
    return *reinterpret_cast<const v4i*>(gp_smem + stage * STAGE + wf_base + a * (16 * GP_BK) + (sub ? swz1 : swz0));
  };

  // Accumulators are pinned to AGPRs and updated in place: the tied "+a" operand keeps the
  // register allocator from rotating 256 accumulator registers through copies.
  v4i acc[TN][TM];
#pragma unroll
  for (int a = 0; a < TN; ++a)
#pragma unroll
    for (int b = 0; b < TM; ++b) acc[a][b] = (v4i){0, 0, 0, 0};
#define GP_MFMA(C, WF, XF) \
  asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+a"(C) : "v"(WF), "v"(XF))

  // ---- prologue: stage 0 <- step 0, registers <- step 1, fragments <- (step 0, first half)
#pragma unroll
  for (int j = 0; j < LA; ++j) load_a(j, 0);
#pragma unroll
  for (int j = 0; j < LB; ++j) load_b(j, 0);
#pragma unroll
  for (int i = 0; i < NWR_A; ++i) write_a(gp_smem, i);
#pragma unroll
  for (int i = 0; i < NWR_B; ++i) write_b(gp_smem, i);
  {
    const int k1 = min(1, nk - 1);
#pragma unroll
    for (int j = 0; j < LA; ++j) load_a(j, k1);
#pragma unroll
    for (int j = 0; j < LB; ++j) load_b(j, k1);
  }
  __syncthreads();
  // Token fragments are needed by every MFMA row of a half step: two full sets (xf, xg).
  // Weight fragments are needed by one row only: a ring of 4, read two rows ahead.
  v4i xf[TM], xg[TM], wr[4];
#pragma unroll
  for (int b = 0; b < TM; ++b) xf[b] = read_x(0, 0, b);
  wr[0] = read_w(0, 0, 0);
  wr[1] = read_w(0, 0, 1);

  static_assert(TM == TN && (TN == 4 || TN == 8), "the interleaving below assumes a square wave tile");
  static_assert(NWR_A == TN && NWR_B == TN, "one A write and one B write per MFMA row");
  constexpr int A_EVERY = TN / LA, B_EVERY = TN / LB;
  for (int ks = 0; ks < nk; ++ks) {
    const int stage = ks & 1;
    unsigned char* st_other = gp_smem + (stage ^ 1) * STAGE;
    const int ks2 = min(ks + 2, nk - 1);
    // first half: k 0..63 of this step.  Per MFMA row: one token fragment of the second half,
    // the weight fragment two rows ahead, and one activation piece and one weight piece
    // expanded into the other stage (written in the order in which they were loaded).
#pragma unroll
    for (int a = 0; a < TN; ++a) {
      xg[a] = read_x(stage, 1, a);
      wr[(a + 2) & 3] = (a + 2 < TN) ? read_w(stage, 0, a + 2) : read_w(stage, 1, a + 2 - TN);
      write_a(st_other, a);
      write_b(st_other, a);
#pragma unroll
      for (int b = 0; b < TM; ++b) GP_MFMA(acc[a][b], wr[a & 3], xf[b]);
    }
    __syncthreads();
    // second half: k 64..127.  Per MFMA row: the global loads whose data the same row of the
    // next first half will write, one token fragment of the next step, and the weight
    // fragment two rows ahead (the last two belong to the next step, whose stage is complete
    // now that the barrier has passed).
#pragma unroll
    for (int a = 0; a < TN; ++a) {
      if (a % A_EVERY == 0) load_a(a / A_EVERY, ks2);
      if (a % B_EVERY == 0) load_b(a / B_EVERY, ks2);
      xf[a] = read_x(stage ^ 1, 0, a);
      wr[(a + 2) & 3] = (a + 2 < TN) ? read_w(stage, 1, a + 2) : read_w(stage ^ 1, 0, a + 2 - TN);
#pragma unroll
      for (int b = 0; b < TM; ++b) GP_MFMA(acc[a][b], wr[a & 3], xg[b]);
    }
    // The MFMAs are issued from inline assembly, so the compiler does not know that their
    // results need wait states before a VALU may read them; the register allocator reads
    // accumulators right at the loop exit.  16 wait states here cover the last MFMA.
    asm volatile("s_nop 15" ::: "memory");
  }
#undef GP_MFMA

  // ---- epilogue: lane holds token m = ... + li and 4 consecutive outputs n = ... + 4*lg + r.
  // float(1024 acc) * (d / 1024) rounds exactly like float(acc) * d.
  const float alpha = alpha_p[0];
  const float unscale = A4 ? (1.0f / 1024.0f) : (1.0f / 64.0f);
  constexpr int SHIFT = A4 ? 10 : 6;
#pragma unroll
  for (int b = 0; b < TM; ++b) {
    const int m = m0 + wm * WM + b * 16 + li;
    const float d = (m < M ? scale[m] : 0.0f) * unscale;
#pragma unroll
    for (int a = 0; a < TN; ++a) {
      const int n = n0 + wn * WN + a * 16 + 4 * lg;
      float fv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) fv[r] = ((float)acc[a][b][r] * d) * alpha;
      const size_t o = (size_t)m * N + n;
      if (VEC) {
        if (m < M && n < N) {
          if (y_bf16) {
            uint2 p;
            p.x = gp_pack_bf16(fv[0], fv[1]);
            p.y = gp_pack_bf16(fv[2], fv[3]);
            *reinterpret_cast<uint2*>((uint16_t*)Y + o) = p;
          } else {
            *reinterpret_cast<float4*>((float*)Y + o) = make_float4(fv[0], fv[1], fv[2], fv[3]);
          }
          if (acc_out)
            *reinterpret_cast<int4*>(acc_out + o) =
                make_int4(acc[a][b][0] >> SHIFT, acc[a][b][1] >> SHIFT, acc[a][b][2] >> SHIFT, acc[a][b][3] >> SHIFT);
        }
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (m < M && n + r < N) {
            if (y_bf16) ((uint16_t*)Y)[o + r] = bl_f32_to_bf16_rne(fv[r]);
            else ((float*)Y)[o + r] = fv[r];
            if (acc_out) acc_out[o + r] = acc[a][b][r] >> SHIFT;
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
  constexpr int smem = GpSmem<BM, BN>::total;
  const int MT = (M + BM - 1) / BM, NTB = (N + BN - 1) / BN;
  const bool vec = (N & 3) == 0;
  auto kern = vec ? gemm_prefill_kernel<BM, BN, A4, true> : gemm_prefill_kernel<BM, BN, A4, false>;
  if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
    return BL_EHIP;
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
