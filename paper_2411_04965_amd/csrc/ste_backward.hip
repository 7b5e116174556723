// Straight-through backward of a quantized linear layer (Section 2.2, "Gradient approximation"):
// the quantizers and the Top_k mask are passed over, so with the dequantized operands
// Xq = d_m q[m, k] and Wq = alpha T[n, k] of the forward pass
//     dX[m, k] = sum_n dY[m, n] Wq[n, k]          dW[n, k] = sum_m dY[m, n] Xq[m, k].
// Both are dense real-valued contractions: bfloat16 operands on `v_mfma_f32_32x32x16_bf16`, float32
// accumulators (the paper trains in mixed precision and fixes nothing further).  Ternary weights and
// the integer codes are exact in bfloat16; the one rounding of an operand is bf16(dY d_m) for dW.
//
// Every contraction is brought to the form C[r, c] = sum_j A[r, j] B[c, j] with j contiguous in
// both operands (what an MFMA lane wants: 8 consecutive j of one row), by three small streaming kernels
// that write into the workspace:
//     Tb  [K][Nc]  bfloat16 = T^T expanded from the input-channel-major 2-bit layout
//     dYt [N][Mc]  bfloat16 = (dY d_m)^T
//     qt  [K][Mc]  bfloat16 = q^T
// (Nc, Mc: rounded up to 64, the padding zero).  Then dX = alpha (dY . Tb^T) and dW = dYt . qt^T.
#include "common.h"

typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

#define SB_BK 64
#define SB_THREADS 256

// ---------------------------------------------------------------- operand preparation
// Tb[k][n] = T[n][k] as bfloat16 (0, 0x3F80, 0xBF80) from BL_W_KMAJOR: one thread per word of 16 outputs.
__global__ __launch_bounds__(256) void ste_expand_weights_kernel(const u32* __restrict__ Wk, int64_t N, int64_t K,
                                                                 int64_t Nc, uint16_t* __restrict__ Tb) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t words_per_row = Nc >> 4;
  if (id >= K * words_per_row) return;
  const int64_t k = id / words_per_row, d = id - k * words_per_row;   // outputs 16 d ... 16 d + 15
  // (Nc <= N rounded up to 512: word d lies inside the layout, whose padding codes are zero)
  const u32 w = Wk[((d >> 5) * K + k) * 32 + (d & 31)];
  u32 o[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const u32 c0 = (w >> (4 * j)) & 3u, c1 = (w >> (4 * j + 2)) & 3u;
    const u32 v0 = (c0 & 1u) ? (0x3F80u | ((c0 & 2u) << 14)) : 0u;
    const u32 v1 = (c1 & 1u) ? (0x3F80u | ((c1 & 2u) << 14)) : 0u;
    o[j] = v0 | (v1 << 16);
  }
  uint4* dst = reinterpret_cast<uint4*>(Tb + k * Nc + 16 * d);
  dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
  dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
}

// Rows of dY whose length is no multiple of 64 are copied once to rows of Nc elements (zero padded), which the
// other kernels then read: 16-byte aligned rows, and a contraction of whole 64-element steps.  One thread per 16-byte piece.
__global__ __launch_bounds__(256) void ste_pad_rows_kernel(const uint16_t* __restrict__ in, int64_t M, int64_t N, int64_t Nc,
                                                           uint16_t* __restrict__ out) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t ppr = Nc >> 3;
  if (id >= M * ppr) return;
  const int64_t m = id / ppr, c = (id - m * ppr) * 8;
  u32 o[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const u32 lo = c + 2 * e < N ? in[m * N + c + 2 * e] : 0u;
    const u32 hi = c + 2 * e + 1 < N ? in[m * N + c + 2 * e + 1] : 0u;
    o[e] = lo | (hi << 16);
  }
  *reinterpret_cast<uint4*>(out + m * Nc + c) = make_uint4(o[0], o[1], o[2], o[3]);
}

// out[c][r] = bf16(f(in[r][c])) for a 64 x 64 tile per workgroup, through LDS.
//   MODE 0: in = dY (bfloat16 [R][C]), f = value * scale[r]            (one float32 multiply, RNE)
//   MODE 1: in = INT8 codes [R][ld_in] (one byte per channel), f = the integer
//   MODE 2: in = INT4 codes [R][ld_in] (nibble form: per 8 channels a word, byte b = q[b] | q[4 + b] << 4)
// Rows r >= R and the padding up to Rc come out as zeros; columns c >= C are not written.
template <int MODE>
__global__ __launch_bounds__(256) void ste_transpose_kernel(const void* __restrict__ in, const float* __restrict__ scale,
                                                            int64_t R, int64_t C, int64_t ld_in, int64_t Rc,
                                                            uint16_t* __restrict__ out) {
  __shared__ uint16_t tile[64][64 + 2];
  const int tid = threadIdx.x;
  const int64_t r0 = (int64_t)blockIdx.x * 64, c0 = (int64_t)blockIdx.y * 64;
  // thread -> (row, 8 columns) twice: 64 rows x 8 pieces = 512 pieces
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int p = tid + 256 * it;
    const int rr = p >> 3, pc = p & 7;
    const int64_t r = r0 + rr, c = c0 + 8 * pc;
    uint16_t v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = 0;
    if (r < R && c < C) {                                   // (a piece that straddles C reads the row's zero padding)
      if (MODE == 0) {
        const uint4 x = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(in) + r * ld_in + c);
        const float s = scale[r];
        const u32 w4[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[2 * e] = bl_f32_to_bf16_rne(__uint_as_float(w4[e] << 16) * s);
          v[2 * e + 1] = bl_f32_to_bf16_rne(__uint_as_float(w4[e] & 0xFFFF0000u) * s);
        }
      } else if (MODE == 1) {
        const uint2 x = *reinterpret_cast<const uint2*>(reinterpret_cast<const signed char*>(in) + r * ld_in + c);
        const u32 w2[2] = {x.x, x.y};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int q = (int)(signed char)((w2[j >> 2] >> (8 * (j & 3))) & 0xFFu);
          v[j] = (uint16_t)(__float_as_uint((float)q) >> 16);             // |q| <= 128: exact in bfloat16
        }
      } else {
        const u32 x = *reinterpret_cast<const u32*>(reinterpret_cast<const unsigned char*>(in) + r * ld_in + (c >> 1));
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const u32 nib = (x >> (8 * (j & 3) + 4 * (j >> 2))) & 0xFu;
          const int q = (int)(nib ^ 8u) - 8;                               // two's complement nibble
          v[j] = (uint16_t)(__float_as_uint((float)q) >> 16);
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) tile[8 * pc + j][rr] = v[j];
  }
  __syncthreads();
  // thread -> (column of the input = row of the output, 8 rows of the input) twice
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int p = tid + 256 * it;
    const int cc = p >> 3, pr = p & 7;
    const int64_t c = c0 + cc;
    if (c < C && r0 + 8 * pr < Rc) {
      u32 o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = (u32)tile[cc][8 * pr + 2 * e] | ((u32)tile[cc][8 * pr + 2 * e + 1] << 16);
      *reinterpret_cast<uint4*>(out + c * Rc + r0 + 8 * pr) = make_uint4(o[0], o[1], o[2], o[3]);
    }
  }
}

// ---------------------------------------------------------------- the contraction
// C[r][c] = mul * sum_j A[r][j] B[c][j]; A [R][lda], B [Cn][ldb] bfloat16, J % 64 == 0 (the callers pad the
// contraction with zeros), lda % 8 == 0, ldb % 8 == 0.  Rows past the end re-read the last row and their
// outputs are not stored.  A workgroup of four waves (2 x 2) owns a tile
// of 64 TM x 64 TN outputs, a wave TM x TN MFMA tiles of 32 x 32: 4 x 4 for large problems (256 x 256 per
// workgroup, 256 accumulator registers, every fragment read from LDS feeds four MFMAs), 2 x 2 for small ones.
// 64 contraction indices per step, two LDS stages, the next step's operands in registers while the current
// one is multiplied.  A row of a stage is 128 bytes whose 16-byte piece p sits at p ^ ((row / 2) % 8): the
// 16 rows that one phase of a fragment read touches then cover the 16 slots of a 256-byte bank window.
template <typename OutT, int TM, int TN>
__global__ __launch_bounds__(SB_THREADS) void ste_gemm_nt_kernel(const uint16_t* __restrict__ A, int64_t lda,
                                                                 const uint16_t* __restrict__ B, int64_t ldb, int R,
                                                                 int Cn, int J, const float* __restrict__ mul_p,
                                                                 OutT* __restrict__ Cout, int64_t ldc, int RT, int CT) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr int STAGE = (BM + BN) * 128;                                    // bytes: A rows, then B rows
  constexpr int PA = BM * 8 / SB_THREADS, PB = BN * 8 / SB_THREADS;        // 16-byte pieces per thread and step
  extern __shared__ __align__(16) unsigned char sb_lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int r0, c0;
  bl_tile_origin(blockIdx.x, RT * CT, RT, CT, BM, BN, r0, c0);
  const int wr = (wave >> 1) * (32 * TM), wc = (wave & 1) * (32 * TN);

  // copy assignment: piece id = tid + 256 i: row = id / 8, piece = id % 8 (the same piece column for every i)
  const int prow = tid >> 3, pp = tid & 7;
  // rows prow + 32 i: (row / 2) % 8 does not depend on i, so one LDS offset serves all pieces of a thread
  const int lds_off = prow * 128 + ((pp ^ ((prow >> 1) & 7)) << 4);
  // (addresses are formed per load: 16 + 16 row pointers would take the registers the fragments need)
  v4i ra[PA], rb[PB];                     // (a first-class vector type: the arrays then stay in registers)
  auto load = [&](int j0) {
    const int64_t col = j0 + 8 * pp;
#pragma unroll
    for (int i = 0; i < PA; ++i) ra[i] = *reinterpret_cast<const v4i*>(A + (int64_t)min(r0 + prow + 32 * i, R - 1) * lda + col);
#pragma unroll
    for (int i = 0; i < PB; ++i) rb[i] = *reinterpret_cast<const v4i*>(B + (int64_t)min(c0 + prow + 32 * i, Cn - 1) * ldb + col);
  };
  auto stage_store = [&](int st) {
    unsigned char* sa = sb_lds + st * STAGE + lds_off;
#pragma unroll
    for (int i = 0; i < PA; ++i) *reinterpret_cast<v4i*>(sa + i * 32 * 128) = ra[i];
#pragma unroll
    for (int i = 0; i < PB; ++i) *reinterpret_cast<v4i*>(sa + BM * 128 + i * 32 * 128) = rb[i];
  };

  v16f acc[TM][TN];
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

  const int li = lane & 31, kg = lane >> 5;
  // fragment addresses: row wr + 32 a + li (A) or wc + 32 b + li (B); (row / 2) % 8 is the same for every a, b
  const int fsw = (li >> 1) & 7;
  const int fa_off = (wr + li) * 128, fb_off = BM * 128 + (wc + li) * 128;
  const int steps = (J + SB_BK - 1) / SB_BK;
  // Pipeline: the operands of step s + 2 are requested during step s and written to LDS during step s + 1,
  // a quarter of the pieces in each of the four sub-steps (A pieces in sub-steps 0, 1, B pieces in 2, 3): every
  // load has a whole step to arrive, and neither the requests nor the LDS writes come as a burst (a wave that
  // issues many loads back to back stalls on them, and it is the only wave of its SIMD).  A piece's register
  // is written to LDS and at once refilled by the next request, so one register set serves.  No branch in the
  // loop (past the last step the requests re-read the last step's pieces and the LDS writes fill a stage that
  // nobody reads any more), so that the compiler can count the loads in flight.
  load(0);
  stage_store(0);
  load(min(1, steps - 1) * SB_BK);
  __syncthreads();
  for (int s = 0; s < steps; ++s) {
    const int cur = s & 1;
    const unsigned char* st = sb_lds + cur * STAGE;
    unsigned char* sn = sb_lds + (cur ^ 1) * STAGE + lds_off;               // stage of step s + 1
    const int64_t coln = min(s + 2, steps - 1) * SB_BK + 8 * pp;           // column of step s + 2
    v8bf fa[2][TM], fb[2][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a) fa[0][a] = *reinterpret_cast<const v8bf*>(st + fa_off + a * 32 * 128 + ((kg ^ fsw) << 4));
#pragma unroll
    for (int b = 0; b < TN; ++b) fb[0][b] = *reinterpret_cast<const v8bf*>(st + fb_off + b * 32 * 128 + ((kg ^ fsw) << 4));
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks < 2) {
#pragma unroll
        for (int i = ks * (PA / 2); i < (ks + 1) * (PA / 2); ++i) {
          *reinterpret_cast<v4i*>(sn + i * 32 * 128) = ra[i];
          ra[i] = *reinterpret_cast<const v4i*>(A + (int64_t)min(r0 + prow + 32 * i, R - 1) * lda + coln);
        }
      } else {
#pragma unroll
        for (int i = (ks - 2) * (PB / 2); i < (ks - 1) * (PB / 2); ++i) {
          *reinterpret_cast<v4i*>(sn + BM * 128 + i * 32 * 128) = rb[i];
          rb[i] = *reinterpret_cast<const v4i*>(B + (int64_t)min(c0 + prow + 32 * i, Cn - 1) * ldb + coln);
        }
      }
      if (ks + 1 < 4) {                                                     // fragments one sub-step ahead
        const int poff = ((2 * (ks + 1) + kg) ^ fsw) << 4;
#pragma unroll
        for (int a = 0; a < TM; ++a) fa[(ks + 1) & 1][a] = *reinterpret_cast<const v8bf*>(st + fa_off + a * 32 * 128 + poff);
#pragma unroll
        for (int b = 0; b < TN; ++b) fb[(ks + 1) & 1][b] = *reinterpret_cast<const v8bf*>(st + fb_off + b * 32 * 128 + poff);
      }
      __builtin_amdgcn_sched_barrier(0);                                   // (all of that stays ahead of the MFMAs)
#pragma unroll
      for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
          acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks & 1][a], fb[ks & 1][b], acc[a][b], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
  }

  // D of a 32 x 32 MFMA tile: lane (li, kg) holds column li, rows 8 (v / 4) + 4 kg + v % 4
  const float mul = mul_p ? mul_p[0] : 1.0f;
#pragma unroll
  for (int a = 0; a < TM; ++a)
#pragma unroll
    for (int b = 0; b < TN; ++b) {
      const int c = c0 + wc + 32 * b + li;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = r0 + wr + 32 * a + 8 * (v >> 2) + 4 * kg + (v & 3);
        if (r < R && c < Cn) {
          const float val = acc[a][b][v] * mul;
          if constexpr (std::is_same<OutT, float>::value) Cout[(int64_t)r * ldc + c] = val;
          else Cout[(int64_t)r * ldc + c] = bl_f32_to_bf16_rne(val);
        }
      }
    }
}

// ---------------------------------------------------------------- host
size_t bl_ste_workspace_bytes(int64_t M, int64_t N, int64_t K) {
  const int64_t Nc = bl_round_up(N, 64), Mc = bl_round_up(M, 64);
  return (size_t)(K * Nc + N * Mc + K * Mc + (N % 64 ? M * Nc : 0)) * 2;
}

template <typename OutT, int TM, int TN>
static int sb_gemm_go(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, int64_t R, int64_t Cn, int64_t J,
                      const float* mul, OutT* C, int64_t ldc, hipStream_t s) {
  constexpr int BM = 64 * TM, BN = 64 * TN;
  constexpr size_t smem = 2 * (size_t)(BM + BN) * 128;
  const int64_t RT = (R + BM - 1) / BM, CT = (Cn + BN - 1) / BN;
  if (!bl_grid_ok(RT * CT)) return BL_ESHAPE;
  BL_SET_MAX_LDS_ONCE((ste_gemm_nt_kernel<OutT, TM, TN>), smem);
  ste_gemm_nt_kernel<OutT, TM, TN><<<(unsigned)(RT * CT), SB_THREADS, smem, s>>>(A, lda, B, ldb, (int)R, (int)Cn, (int)J,
                                                                                mul, C, ldc, (int)RT, (int)CT);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

// 256 x 256 tiles where they fill the chip at least twice, else 128 x 128.
template <typename OutT>
static int sb_gemm(const uint16_t* A, int64_t lda, const uint16_t* B, int64_t ldb, int64_t R, int64_t Cn, int64_t J,
                   const float* mul, OutT* C, int64_t ldc, hipStream_t s) {
  if (((R + 255) / 256) * ((Cn + 255) / 256) >= 2 * (int64_t)bl_num_cus())
    return sb_gemm_go<OutT, 4, 4>(A, lda, B, ldb, R, Cn, J, mul, C, ldc, s);
  return sb_gemm_go<OutT, 2, 2>(A, lda, B, ldb, R, Cn, J, mul, C, ldc, s);
}

// q: INT4 nibble codes [M][Kp / 2] (a4 = true) or INT8 codes [M][Kp]; Wk: BL_W_KMAJOR.
int bl_launch_ste_backward(const void* dY, int64_t M, int64_t N, int64_t K, const void* q, const float* scale, bool a4,
                           const void* Wk, const float* alpha, void* dX, bl_dtype dx_dtype, float* dW, void* ws,
                           hipStream_t s) {
  const int64_t Nc = bl_round_up(N, 64), Mc = bl_round_up(M, 64), Kp = bl_round_up(K, BL_KPAD);
  uint16_t* Tb = reinterpret_cast<uint16_t*>(ws);
  uint16_t* dYt = Tb + K * Nc;
  uint16_t* qt = dYt + N * Mc;
  const uint16_t* dYa = reinterpret_cast<const uint16_t*>(dY);           // dY with 16-byte aligned rows
  int64_t ldy = N;
  if (N % 64) {                                                          // (the contraction of dX runs to Nc)
    uint16_t* dYp = qt + K * Mc;
    const int64_t pieces = M * (Nc >> 3);
    if (!bl_grid_ok((pieces + 255) / 256)) return BL_ESHAPE;
    ste_pad_rows_kernel<<<(unsigned)((pieces + 255) / 256), 256, 0, s>>>(dYa, M, N, Nc, dYp);
    BL_HIP_CHECK_LAUNCH();
    dYa = dYp;
    ldy = Nc;
  }
  if (dX) {
    const int64_t words = K * (Nc >> 4);
    if (!bl_grid_ok((words + 255) / 256)) return BL_ESHAPE;
    ste_expand_weights_kernel<<<(unsigned)((words + 255) / 256), 256, 0, s>>>(reinterpret_cast<const u32*>(Wk), N, K, Nc, Tb);
    BL_HIP_CHECK_LAUNCH();
    int rc;
    if (dx_dtype == BL_F32)
      rc = sb_gemm<float>(dYa, ldy, Tb, Nc, M, K, Nc, alpha, reinterpret_cast<float*>(dX), K, s);
    else
      rc = sb_gemm<uint16_t>(dYa, ldy, Tb, Nc, M, K, Nc, alpha, reinterpret_cast<uint16_t*>(dX), K, s);
    if (rc != BL_OK) return rc;
  }
  if (dW) {
    const dim3 g1((unsigned)(Mc / 64), (unsigned)((N + 63) / 64)), g2((unsigned)(Mc / 64), (unsigned)((K + 63) / 64));
    if (g1.y > 65535u || g2.y > 65535u) return BL_ESHAPE;
    ste_transpose_kernel<0><<<g1, 256, 0, s>>>(dYa, scale, M, N, ldy, Mc, dYt);
    BL_HIP_CHECK_LAUNCH();
    if (a4) ste_transpose_kernel<2><<<g2, 256, 0, s>>>(q, nullptr, M, K, Kp / 2, Mc, qt);
    else ste_transpose_kernel<1><<<g2, 256, 0, s>>>(q, nullptr, M, K, Kp, Mc, qt);
    BL_HIP_CHECK_LAUNCH();
    const int rc = sb_gemm<float>(dYt, Mc, qt, Mc, N, K, Mc, nullptr, dW, K, s);
    if (rc != BL_OK) return rc;
  }
  return BL_OK;
}
