// Prefill GEMM of the W1.58A4 linear (eq. 6 of the paper) on the CDNA4 block-float matrix
// instruction:
//   acc[m, n] = sum_k q[m, k] * T[n, k],   Y[m, n] = (acc * d[m]) * alpha.
// v_mfma_f32_32x32x64_f8f6f4 multiplies 6-bit and 4-bit floating-point operands at twice the
// INT8 rate.  Every INT4 level -8..7 is exact in E3M2 and every ternary weight in E2M1, the
// products are integers of magnitude <= 8 and the float32 accumulator holds integers below
// 2^24 exactly, so for K <= 32768 (|acc| <= 2^18) the result equals the int32 accumulator bit
// for bit, whatever the order of the additions.
//
// Both operands arrive in HBM in the order in which LDS wants them (see the format notes in the
// public header): blocks of 32 rows x 256 channels, rows XOR-swizzled by 16-byte (8-byte) piece so
// that the fragment reads are free of bank conflicts.  The copy from global memory to LDS is
// therefore linear and is done by global_load_lds_dwordx4: no staging registers, no LDS write
// instructions and no vector work in the main loop, which consists of MFMAs, fragment reads and
// the asynchronous loads.
//
// Structure.  Persistent blocks (one per CU) walk the tile list; block = 4 waves, tile
// 256 x 256, each wave 128 x 128 as 4 x 4 MFMA tiles; the MFMA's row operand is the weight
// fragment and its column operand the token fragment, so a lane ends up with groups of 4
// consecutive outputs n of one token.  K advances 256 channels per step through two LDS stages
// of 80 KB (the whole LDS), four MFMA sub-steps of 64 channels each, with two register sets of
// fragments: sub-step s computes on one set while the other is filled for sub-step s + 1.
// One barrier per step, at the end of sub-step 2: by then every wave has read its last
// fragments of the step's stage, and (after waiting for its own loads) the next step's stage is
// complete.  Behind the barrier the loads of the step after next go into the stage just freed.
// Each wave copies the row blocks 2w and 2w + 1 of both operands.
#include "common.h"

#define GX_THREADS 256
#define GX_BM 256
#define GX_BN 256
#define GX_XQ 32768                  // stage layout: [XP 8 x 4096 | XQ 8 x 2048 | W 8 x 4096]
#define GX_W 49152
#define GX_STAGE 81920
#define GX_LDS (2 * GX_STAGE)
#define GX_A_BLOCK 6144              // bytes of 32 tokens x 256 channels of 6-bit codes
#define GX_W_BLOCK 4096              // bytes of 32 outputs x 256 channels of 4-bit codes

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v6i __attribute__((ext_vector_type(6)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) unsigned char lds_uchar;

__device__ __forceinline__ u32 gx_pack_bf16(float lo, float hi) {
  u32 r;
  asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
  return r;
}

// Four (two) asynchronous 1 KB copies global -> LDS: lane l moves 16 bytes from base + voff + o to
// LDS byte address lds + 16 l + o for o = 0, 1024, ...  (M0 holds the LDS address; the immediate
// offset applies to both sides.)  The copies are counted by vmcnt like any other load.
// (The host pass of the compiler parses kernel bodies too and knows no scalar-register
// constraint, so it sees empty statements here.)
#if defined(__HIP_DEVICE_COMPILE__)
#define GX_DMA4(lds, base, voff)                                                        \
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"                                        \
               "global_load_lds_dwordx4 %1, %2\n\t"                                     \
               "global_load_lds_dwordx4 %1, %2 offset:1024\n\t"                         \
               "global_load_lds_dwordx4 %1, %2 offset:2048\n\t"                         \
               "global_load_lds_dwordx4 %1, %2 offset:3072"                             \
               ::"s"(lds), "v"(voff), "s"(base) : "memory")
#define GX_DMA2(lds, base, voff)                                                        \
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\t"                                        \
               "global_load_lds_dwordx4 %1, %2\n\t"                                     \
               "global_load_lds_dwordx4 %1, %2 offset:1024"                             \
               ::"s"(lds), "v"(voff), "s"(base) : "memory")
#else
#define GX_DMA4(lds, base, voff) ((void)0)
#define GX_DMA2(lds, base, voff) ((void)0)
#endif

// OUT: 0 = bf16 rows through the LDS transpose (N % 8 == 0), 1 = 4 outputs per store (N % 4 == 0),
// 2 = one output per store (any N).  ACC: also write the integer accumulators (tests).
template <int OUT, bool ACC>
__global__ __launch_bounds__(GX_THREADS, 1) void gemm_a4_mx_kernel(
    const unsigned char* __restrict__ A, const float* __restrict__ scale, int M, int KB,
    const unsigned char* __restrict__ Wp, const float* __restrict__ alpha_p, int N, void* __restrict__ Y,
    int y_bf16, int32_t* __restrict__ acc_out, int MT, int NTB) {
  extern __shared__ __align__(16) unsigned char gx_smem[];
  const u32 lds0 = (u32)(uintptr_t)(lds_uchar*)gx_smem;      // LDS byte address of the first stage
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;     // MFMA operand row / k-half of this lane
  const int n_tiles = MT * NTB;
  const int MB = (M + 31) >> 5, NB = (N + 31) >> 5;           // 32-row blocks of the operands
  constexpr int WM = 128, WN = 128, TM = 4, TN = 4;

  // ---- asynchronous copies.  The cursor names the (tile, K block) that is copied next and
  // moves on along the block's stream of tiles by itself.
  struct Cursor {
    const unsigned char* a[2];
    const unsigned char* w[2];
    int kb, tile;
    bool live;                                   // false once the stream has run out
  };
  auto point = [&](Cursor& c, int tile) {
    int m0, n0;
    bl_tile_origin(tile, n_tiles, MT, NTB, GX_BM, GX_BN, m0, n0);
    c.tile = tile;
    c.kb = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      // row blocks past the end of an operand re-read its last block (their results are never stored)
      const int ab = min((m0 >> 5) + 2 * wave + i, MB - 1), wb = min((n0 >> 5) + 2 * wave + i, NB - 1);
      c.a[i] = A + (size_t)ab * KB * GX_A_BLOCK;
      c.w[i] = Wp + (size_t)wb * KB * GX_W_BLOCK;
    }
  };
  auto advance = [&](Cursor& c) {
    if (++c.kb == KB) {
      const int nt = c.tile + (int)gridDim.x;
      if (nt < n_tiles) point(c, nt);
      else c.live = false;
    } else {
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        c.a[i] += GX_A_BLOCK;
        c.w[i] += GX_W_BLOCK;
      }
    }
  };
  const u32 dma_voff = lane * 16;
  // copy part p (0..5) of the cursor's K block into the stage at LDS address st
  auto dma_part = [&](const Cursor& c, u32 st, int p) {
    const int i = p / 3, rb = 2 * wave + i;
    if (p % 3 == 0) GX_DMA4(st + rb * 4096, c.a[i], dma_voff);
    else if (p % 3 == 1) GX_DMA2(st + GX_XQ + rb * 2048, c.a[i] + 4096, dma_voff);
    else GX_DMA4(st + GX_W + rb * 4096, c.w[i], dma_voff);
  };

  // ---- fragment addresses (within a stage): lane (l32, lh) reads unit u = 2 s + lh of its row
  int xp_off[4], xq_off[4], w_off[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const int u = 2 * s + lh;
    xp_off[s] = (wm * WM + l32) * 128 + ((u ^ (l32 & 7)) << 4);
    xq_off[s] = GX_XQ + (wm * WM + l32) * 64 + ((u ^ ((l32 >> 2) & 7)) << 3);
    w_off[s] = GX_W + (wn * WN + l32) * 128 + ((u ^ (l32 & 7)) << 4);
  }
  struct Frags {
    v6i x[TM];
    v4i w[TN];
  };
  auto read_x = [&](const unsigned char* st, int s, int b) -> v6i {
    const v4i p = *reinterpret_cast<const v4i*>(st + xp_off[s] + b * 4096);
    const v2i q = *reinterpret_cast<const v2i*>(st + xq_off[s] + b * 2048);
    return (v6i){p[0], p[1], p[2], p[3], q[0], q[1]};
  };
  auto read_w = [&](const unsigned char* st, int s, int a) -> v4i {
    return *reinterpret_cast<const v4i*>(st + w_off[s] + a * 4096);
  };

#if defined(__HIP_DEVICE_COMPILE__)
#define GX_MFMA(C, WF, XF) \
  asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0 cbsz:4 blgp:3" : "+a"(C) : "v"(WF), "v"(XF))
#else
#define GX_MFMA(C, WF, XF) ((void)0)
#endif

  const float alpha = alpha_p[0];

  // ---- first tile of this block: stage 0 <- step 0, stage 1 <- step 1 (in flight), fragments
  int tile = blockIdx.x;
  int m0, n0;
  bl_tile_origin(tile, n_tiles, MT, NTB, GX_BM, GX_BN, m0, n0);
  Cursor cur;
  cur.live = true;
  point(cur, tile);
#pragma unroll
  for (int p = 0; p < 6; ++p) dma_part(cur, lds0, p);
  advance(cur);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (cur.live) {
#pragma unroll
    for (int p = 0; p < 6; ++p) dma_part(cur, lds0 + GX_STAGE, p);
    advance(cur);
  }
  Frags F[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    F[0].x[i] = read_x(gx_smem, 0, i);
    F[0].w[i] = read_w(gx_smem, 0, i);
  }

  int g = 0;                                     // steps done by this block (stage = g & 1)
  while (true) {
    const int next = tile + (int)gridDim.x;
    const bool has_next = next < n_tiles;
    v16f acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
      for (int b = 0; b < TM; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.0f;
    float dsc[TM];                               // per-token scales of this tile
#pragma unroll
    for (int b = 0; b < TM; ++b) {
      const int m = m0 + wm * WM + b * 32 + l32;
      dsc[b] = m < M ? scale[m] : 0.0f;
    }

    for (int kb = 0; kb < KB; ++kb, ++g) {
      const unsigned char* st_own = gx_smem + (g & 1) * GX_STAGE;
      const unsigned char* st_other = gx_smem + ((g & 1) ^ 1) * GX_STAGE;
      const u32 lds_own = lds0 + (g & 1) * GX_STAGE;
      const bool last = kb == KB - 1;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        Frags& use = F[s & 1];
        Frags& fill = F[(s & 1) ^ 1];
        const unsigned char* src = s < 3 ? st_own : st_other;
        const int ns = (s + 1) & 3;
        // Behind the barrier (sub-step 3) the own stage is free: the step after next goes
        // there.  At the end of a tile the stage first serves the epilogue as transpose space.
        const bool dma_now = s == 3 && !last && cur.live;
#pragma unroll
        for (int a = 0; a < TN; ++a) {
#pragma unroll
          for (int b = 0; b < TM; ++b) {
            GX_MFMA(acc[a][b], use.w[a], use.x[b]);
            const int i = a * TM + b;              // one slot behind each MFMA
            if (i < 4) fill.x[i] = read_x(src, ns, i);
            else if (i < 8) fill.w[i - 4] = read_w(src, ns, i - 4);
            else if (i < 14 && dma_now) dma_part(cur, lds_own, i - 8);
          }
        }
        if (s == 3 && dma_now) advance(cur);
        if (s == 2) {
          // own loads of the next step have landed; every wave is done reading this stage
          asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
          __syncthreads();
        }
      }
    }
    // The MFMAs are issued from inline assembly: the compiler does not know that their results
    // need wait states before a vector instruction may read them.
    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");

    // ---- epilogue.  acc[a][b][r] is output n = 32 a + 8 (r / 4) + 4 lh + r % 4 of token
    // m = 32 b + l32 (relative to the wave tile).  The stage of the tile's last step is free
    // (its refill was held back) and serves as transpose space.
    const int free_stage = (g - 1) & 1;
    if (OUT == 0) {
      constexpr int TB_ROW = WN * 2 + 32;
      unsigned char* tbuf = gx_smem + free_stage * GX_STAGE + wave * (32 * TB_ROW);
      constexpr int LANES_PER_ROW = WN * 2 / 16;           // 16 lanes cover one token's 256 bytes
      constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
      constexpr int NPASS = 32 / ROWS_PER_PASS;
      const int rr = lane / LANES_PER_ROW, cc = lane % LANES_PER_ROW;
      uint16_t* ywave = (uint16_t*)Y + (size_t)(m0 + wm * WM) * N + (n0 + wn * WN);
      const u32 lane_off = (u32)rr * (u32)N + cc * 8;
      const bool interior = (m0 + GX_BM <= M) && (n0 + GX_BN <= N);
      const int m_left = M - (m0 + wm * WM) - rr, n_left = N - (n0 + wn * WN) - cc * 8;
#pragma unroll
      for (int b = 0; b < TM; ++b) {
        const float d = dsc[b];
#pragma unroll
        for (int a = 0; a < TN; ++a) {
          asm volatile("" : "+a"(acc[a][b]));
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            float fv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) fv[r] = (acc[a][b][4 * q4 + r] * d) * alpha;
            uint2 p;
            p.x = gx_pack_bf16(fv[0], fv[1]);
            p.y = gx_pack_bf16(fv[2], fv[3]);
            *reinterpret_cast<uint2*>(tbuf + l32 * TB_ROW + (a * 32 + 8 * q4 + 4 * lh) * 2) = p;
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        if (interior) {                                    // uniform: all reads in flight, then all stores
          v4i v[NPASS];
#pragma unroll
          for (int i = 0; i < NPASS; ++i)
            v[i] = *reinterpret_cast<const v4i*>(tbuf + (rr + i * ROWS_PER_PASS) * TB_ROW + cc * 16);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < NPASS; ++i)
            *reinterpret_cast<v4i*>(ywave + (size_t)(b * 32 + i * ROWS_PER_PASS) * N + lane_off) = v[i];
        } else {
#pragma unroll
          for (int i = 0; i < NPASS; ++i) {
            const int row = b * 32 + i * ROWS_PER_PASS;
            const v4i v = *reinterpret_cast<const v4i*>(tbuf + (rr + i * ROWS_PER_PASS) * TB_ROW + cc * 16);
            if (row < m_left && 0 < n_left) *reinterpret_cast<v4i*>(ywave + (size_t)row * N + lane_off) = v;
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int b = 0; b < TM; ++b) {
        const int m = m0 + wm * WM + b * 32 + l32;
        const float d = dsc[b];
#pragma unroll
        for (int a = 0; a < TN; ++a) {
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int n = n0 + wn * WN + a * 32 + 8 * q4 + 4 * lh;
            const size_t o = (size_t)m * N + n;
            float fv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) fv[r] = (acc[a][b][4 * q4 + r] * d) * alpha;
            if (OUT == 1) {
              if (m < M && n < N) {
                if (y_bf16) {
                  uint2 p;
                  p.x = gx_pack_bf16(fv[0], fv[1]);
                  p.y = gx_pack_bf16(fv[2], fv[3]);
                  *reinterpret_cast<uint2*>((uint16_t*)Y + o) = p;
                } else {
                  *reinterpret_cast<float4*>((float*)Y + o) = make_float4(fv[0], fv[1], fv[2], fv[3]);
                }
              }
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                if (m < M && n + r < N) {
                  if (y_bf16) ((uint16_t*)Y)[o + r] = bl_f32_to_bf16_rne(fv[r]);
                  else ((float*)Y)[o + r] = fv[r];
                }
              }
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (ACC) {
#pragma unroll
      for (int b = 0; b < TM; ++b) {
        const int m = m0 + wm * WM + b * 32 + l32;
#pragma unroll
        for (int a = 0; a < TN; ++a) {
#pragma unroll
          for (int q4 = 0; q4 < 4; ++q4) {
            const int n = n0 + wn * WN + a * 32 + 8 * q4 + 4 * lh;
            const size_t o = (size_t)m * N + n;
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (m < M && n + r < N) acc_out[o + r] = (int32_t)acc[a][b][4 * q4 + r];
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (!has_next) break;
    tile = next;
    bl_tile_origin(tile, n_tiles, MT, NTB, GX_BM, GX_BN, m0, n0);
    __syncthreads();                   // transpose space has been read out by every wave
    // the refill that was held back: the step after the next tile's first
    if (cur.live) {
#pragma unroll
      for (int p = 0; p < 6; ++p) dma_part(cur, lds0 + free_stage * GX_STAGE, p);
      advance(cur);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no copy may be in flight when the LDS is released
#undef GX_MFMA
}

static int gx_num_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return 256;
    cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  }
  return cus;
}

template <int OUT, bool ACC>
static int gx_go(const void* q, const float* scale, int M, int KB, const void* Wp, const float* alpha,
                 int N, void* Y, int y_bf16, int32_t* acc_out, int MT, int NTB, hipStream_t s) {
  if (hipFuncSetAttribute((const void*)gemm_a4_mx_kernel<OUT, ACC>,
                          hipFuncAttributeMaxDynamicSharedMemorySize, GX_LDS) != hipSuccess)
    return BL_EHIP;
  const int grid = min(MT * NTB, gx_num_cus());      // persistent blocks, one per CU (all of its LDS)
  gemm_a4_mx_kernel<OUT, ACC><<<(unsigned)grid, GX_THREADS, GX_LDS, s>>>(
      (const unsigned char*)q, scale, M, KB, (const unsigned char*)Wp, alpha, N, Y, y_bf16, acc_out, MT, NTB);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

int bl_launch_gemm_a4_mx(const void* q, const float* scale, int64_t M, int64_t K, const void* Wp,
                         const float* alpha, int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out,
                         hipStream_t s) {
  const int KB = (int)(bl_round_up(K, BL_KPAD) / 256);
  const int MT = (int)((M + GX_BM - 1) / GX_BM), NTB = (int)((N + GX_BN - 1) / GX_BN);
  const int out = (ydt == BL_BF16 && (N & 7) == 0) ? 0 : ((N & 3) == 0 ? 1 : 2);
  const int yb = ydt == BL_BF16 ? 1 : 0;
#define GX_CALL(OUT, ACC) gx_go<OUT, ACC>(q, scale, (int)M, KB, Wp, alpha, (int)N, Y, yb, acc_out, MT, NTB, s)
  if (acc_out) return out == 0 ? GX_CALL(0, true) : out == 1 ? GX_CALL(1, true) : GX_CALL(2, true);
  return out == 0 ? GX_CALL(0, false) : out == 1 ? GX_CALL(1, false) : GX_CALL(2, false);
#undef GX_CALL
}
