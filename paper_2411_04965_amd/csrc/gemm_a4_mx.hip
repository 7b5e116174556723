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
// public header): blocks of 32 rows x 128 channels, rows XOR-swizzled by 16-byte (8-byte) piece so
// that the fragment reads are free of bank conflicts (the LDS serves 256 bytes per clock: 16 lanes
// of a 16-byte read, 32 lanes of an 8-byte read, which must fall into distinct slots of a 256-byte
// window).  The copy from global memory to LDS is
// therefore linear and is done by global_load_lds_dwordx4: no staging registers, no LDS write
// instructions and no vector work in the main loop, which consists of MFMAs, fragment reads and
// the asynchronous loads.
//
// Structure.  Persistent blocks (one per CU) walk the tile list; block = 4 waves, tile
// 256 x 256, each wave 128 x 128 as 4 x 4 MFMA tiles; the MFMA's row operand is the weight
// fragment and its column operand the token fragment, so a lane ends up with groups of 4
// consecutive outputs n of one token.  K advances 128 channels per step through a ring of four
// LDS stages of 40 KB (the whole LDS), two MFMA sub-steps of 64 channels each, with two register
// sets of fragments: a sub-step computes on one set while the other is filled for the next.
// One barrier per step, at the end of its first sub-step: by then every wave has read its last
// fragments of the step's stage, and (after waiting for its own loads) the next step's stage is
// complete.  Behind the barrier the loads of step g + 4 go into the stage of step g.
//
// The asynchronous loads are limited by the 64 bytes per clock between L1 and the CU: a 1 KB
// load occupies a wave's share of that path for 64 cycles, and a burst of loads stalls the MFMA
// stream of the issuing wave.  The tile needs 40 KB per 1024 MFMA cycles, 62% of the path, so
// the loads are issued evenly, five per sub-step, each behind its own MFMA, and run three steps
// ahead of the MFMAs.  Each wave copies the row blocks 2w and 2w + 1 of both operands.
#include "common.h"

#define GX_THREADS 256
#define GX_BM 256
#define GX_BN 256
#define GX_XQ 16384                  // stage layout: [XP 8 x 2048 | XQ 8 x 1024 | W 8 x 2048]
#define GX_W 24576
#define GX_STAGE 40960
#define GX_NSTAGE 4
#define GX_LDS (GX_NSTAGE * GX_STAGE)
#define GX_A_BLOCK 3072              // bytes of 32 tokens x 128 channels of 6-bit codes
#define GX_W_BLOCK 2048              // bytes of 32 outputs x 128 channels of 4-bit codes
#define GX_LOADS_PER_STEP 10         // asynchronous 1 KB loads per wave and step

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v6i __attribute__((ext_vector_type(6)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) unsigned char lds_uchar;

__device__ __forceinline__ u32 gx_pack_bf16(float lo, float hi) {
  u32 r;
  asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
  return r;
}

// One asynchronous 1 KB copy global -> LDS: lane l moves 16 bytes from base + voff to LDS byte
// address lds + 16 l (M0 holds the LDS address).  The copies are counted by vmcnt like any other
// load.  (The host pass of the compiler parses kernel bodies too and knows no scalar-register
// constraint, so it sees empty statements here.)
#if defined(__HIP_DEVICE_COMPILE__)
#define GX_DMA(lds, base, voff)                                                         \
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"          \
               ::"s"(lds), "v"(voff), "s"(base) : "memory")
#define GX_WAIT_LOADS(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")
#else
#define GX_DMA(lds, base, voff) ((void)0)
#define GX_WAIT_LOADS(n) ((void)0)
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

  // ---- asynchronous copies.  The cursor names the (tile, K step) that is copied next and
  // moves on along the block's stream of tiles by itself.
  struct Cursor {
    const unsigned char* a[2];
    const unsigned char* w[2];
    int kb, tile;
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
  // one step on; behind the block's last step the cursor stays where it is (the loads go on, so
  // that the number of loads in flight is the same at every barrier; their data is never used)
  auto advance = [&](Cursor& c) {
    if (c.kb + 1 == KB) {
      const int nt = c.tile + (int)gridDim.x;
      if (nt < n_tiles) point(c, nt);
    } else {
      ++c.kb;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        c.a[i] += GX_A_BLOCK;
        c.w[i] += GX_W_BLOCK;
      }
    }
  };
  const u32 dma_voff = lane * 16;
  // load p (0..9) of the cursor's K step into the stage at LDS address st: row block 2w + p / 5,
  // there XP (2 KB), XQ (1 KB), W (2 KB)
  auto dma_part = [&](const Cursor& c, u32 st, int p) {
    const int i = p / 5, j = p % 5, rb = 2 * wave + i;
    if (j < 2) GX_DMA(st + rb * 2048 + j * 1024, c.a[i] + j * 1024, dma_voff);
    else if (j == 2) GX_DMA(st + GX_XQ + rb * 1024, c.a[i] + 2048, dma_voff);
    else GX_DMA(st + GX_W + rb * 2048 + (j - 3) * 1024, c.w[i] + (j - 3) * 1024, dma_voff);
  };

  // ---- fragment addresses (within a stage): lane (l32, lh) reads unit u = 2 s + lh of its row
  int xp_off[2], xq_off[2], w_off[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const int u = 2 * s + lh;
    xp_off[s] = (wm * WM + l32) * 64 + ((u ^ ((l32 >> 2) & 3)) << 4);
    xq_off[s] = GX_XQ + (wm * WM + l32) * 32 + ((u ^ ((l32 >> 3) & 3)) << 3);
    w_off[s] = GX_W + (wn * WN + l32) * 64 + ((u ^ ((l32 >> 2) & 3)) << 4);
  }
  struct Frags {
    v6i x[TM];
    v4i w[TN];
  };
  auto read_x = [&](const unsigned char* st, int s, int b) -> v6i {
    const v4i p = *reinterpret_cast<const v4i*>(st + xp_off[s] + b * 2048);
    const v2i q = *reinterpret_cast<const v2i*>(st + xq_off[s] + b * 1024);
    return (v6i){p[0], p[1], p[2], p[3], q[0], q[1]};
  };
  auto read_w = [&](const unsigned char* st, int s, int a) -> v4i {
    return *reinterpret_cast<const v4i*>(st + w_off[s] + a * 2048);
  };

#if defined(__HIP_DEVICE_COMPILE__)
#define GX_MFMA(C, WF, XF) \
  asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0 cbsz:4 blgp:3" : "+a"(C) : "v"(WF), "v"(XF))
// first MFMA on an accumulator tile: C = 0 (saves clearing 256 registers per output tile)
#define GX_MFMA0(C, WF, XF) \
  asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, 0 cbsz:4 blgp:3" : "=a"(C) : "v"(WF), "v"(XF))
#else
#define GX_MFMA(C, WF, XF) ((void)0)
#define GX_MFMA0(C, WF, XF) ((void)0)
#endif

  const float alpha = alpha_p[0];

  // ---- first tile of this block.  Loads of step g are issued in two halves of five: the
  // first during sub-step 1 of step g - 4, the second during sub-step 0 of step g - 3.  So the
  // loop starts with steps 0, 1, 2 and the first half of step 3 under way.
  int tile = blockIdx.x;
  int m0, n0;
  bl_tile_origin(tile, n_tiles, MT, NTB, GX_BM, GX_BN, m0, n0);
  Cursor cur;
  point(cur, tile);
#pragma unroll
  for (int st = 0; st < 3; ++st) {
#pragma unroll
    for (int p = 0; p < GX_LOADS_PER_STEP; ++p) dma_part(cur, lds0 + st * GX_STAGE, p);
    advance(cur);
  }
#pragma unroll
  for (int p = 0; p < GX_LOADS_PER_STEP / 2; ++p) dma_part(cur, lds0 + 3 * GX_STAGE, p);
  GX_WAIT_LOADS(2 * GX_LOADS_PER_STEP + GX_LOADS_PER_STEP / 2);      // step 0 has landed
  __syncthreads();
  Frags F[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    F[0].x[i] = read_x(gx_smem, 0, i);
    F[0].w[i] = read_w(gx_smem, 0, i);
  }
  // Per-token scales of a tile.  The compiler cannot count the asynchronous loads, so wherever
  // it has to wait for a load of its own it waits for every load in flight.  The scales are
  // therefore fetched where that is cheap: here, and for every later tile inside the epilogue of
  // the tile before it (see there).
  auto load_scales = [&](int tm0, float (&d)[TM]) {
#pragma unroll
    for (int b = 0; b < TM; ++b) {
      const int m = tm0 + wm * WM + b * 32 + l32;
      d[b] = m < M ? scale[m] : 0.0f;
    }
  };
  float dsc[TM];
  load_scales(m0, dsc);
  asm volatile("" : "+v"(dsc[0]), "+v"(dsc[1]), "+v"(dsc[2]), "+v"(dsc[3]));

  int g = 0;                                     // steps done by this block (stage = g % 4)
  // When step g reaches its barrier, the loads in flight that are younger than those of step
  // g + 1 (which must have landed) are the 20 of steps g + 2 and g + 3 and, for the two steps
  // behind the epilogue of an interior bf16 tile, also that epilogue's 32 stores.  (Any other
  // epilogue waits for its stores itself.)  Vector memory operations complete in order, so
  // "at most that many in flight" is the condition to wait for; operations this count does not
  // know of (the scale loads of a tile) only make the wait longer.
  constexpr int EPI_STORES = 32;
  int steps_behind_stores = 0;
  while (true) {
    const int next = tile + (int)gridDim.x;
    const bool has_next = next < n_tiles;
    const bool interior = (m0 + GX_BM <= M) && (n0 + GX_BN <= N);
    v16f acc[TN][TM];
    int nm0 = m0, nn0 = n0;                      // origin of the block's next tile
    if (has_next) bl_tile_origin(next, n_tiles, MT, NTB, GX_BM, GX_BN, nm0, nn0);
    float dsc_next[TM];

    for (int kb = 0; kb < KB; ++kb, ++g) {
      const unsigned char* st_own = gx_smem + (g & 3) * GX_STAGE;
      const unsigned char* st_next = gx_smem + ((g + 1) & 3) * GX_STAGE;
      const u32 lds_own = lds0 + (g & 3) * GX_STAGE, lds_prev = lds0 + ((g + 3) & 3) * GX_STAGE;
      const bool last = kb == KB - 1;
      // ---- sub-step 0: computes on F[0], fills F[1] from the own stage, issues the second half
      // of the loads of step g + 3 (into the stage that step g - 1 has left)
#pragma unroll
      for (int a = 0; a < TN; ++a) {
#pragma unroll
        for (int b = 0; b < TM; ++b) {
          if (kb == 0) GX_MFMA0(acc[a][b], F[0].w[a], F[0].x[b]);
          else GX_MFMA(acc[a][b], F[0].w[a], F[0].x[b]);
          const int i = a * TM + b;              // one slot behind each MFMA
          if (i < 4) F[1].x[i] = read_x(st_own, 1, i);
          else if (i < 8) F[1].w[i - 4] = read_w(st_own, 1, i - 4);
          if (i % 3 == 2) dma_part(cur, lds_prev, 5 + i / 3);          // slots 2, 5, 8, 11, 14
        }
      }
      advance(cur);
      // own loads of the next step have landed; every wave is done reading this stage
      if (steps_behind_stores > 0) {
        GX_WAIT_LOADS(2 * GX_LOADS_PER_STEP + EPI_STORES);
        --steps_behind_stores;
      } else {
        GX_WAIT_LOADS(2 * GX_LOADS_PER_STEP);
      }
      __syncthreads();
      // ---- sub-step 1: computes on F[1], fills F[0] from the next step's stage, issues the
      // first half of the loads of step g + 4 into the own stage, which is free now.  At the end
      // of a tile the stage first serves the epilogue as transpose space: the loads follow it.
#pragma unroll
      for (int a = 0; a < TN; ++a) {
#pragma unroll
        for (int b = 0; b < TM; ++b) {
          GX_MFMA(acc[a][b], F[1].w[a], F[1].x[b]);
          const int i = a * TM + b;
          if (i < 4) F[0].x[i] = read_x(st_next, 0, i);
          else if (i < 8) F[0].w[i - 4] = read_w(st_next, 0, i - 4);
          if (i % 3 == 2 && !last) dma_part(cur, lds_own, i / 3);
        }
      }
    }
    // The MFMAs are issued from inline assembly: the compiler does not know that their results
    // need wait states before a vector instruction may read them.
    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");

    // ---- epilogue.  acc[a][b][r] is output n = 32 a + 8 (r / 4) + 4 lh + r % 4 of token
    // m = 32 b + l32 (relative to the wave tile).  The stage of the tile's last step is free
    // (its refill was held back) and serves as transpose space.
    const int free_stage = (g - 1) & 3;
    if (OUT == 0) {
      constexpr int TB_ROW = WN * 2 + 32;
      unsigned char* tbuf = gx_smem + free_stage * GX_STAGE + wave * (32 * TB_ROW);
      static_assert(4 * 32 * TB_ROW <= GX_STAGE, "transpose space must fit into one stage");
      constexpr int LANES_PER_ROW = WN * 2 / 16;           // 16 lanes cover one token's 256 bytes
      constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
      constexpr int NPASS = 32 / ROWS_PER_PASS;
      const int rr = lane / LANES_PER_ROW, cc = lane % LANES_PER_ROW;
      uint16_t* ywave = (uint16_t*)Y + (size_t)(m0 + wm * WM) * N + (n0 + wn * WN);
      const u32 lane_off = (u32)rr * (u32)N + cc * 8;
      const int m_left = M - (m0 + wm * WM) - rr, n_left = N - (n0 + wn * WN) - cc * 8;
      // scales of the next tile: requested now, waited for behind the first column's arithmetic,
      // when the last asynchronous loads are a few thousand cycles old and nothing else is in flight
      load_scales(nm0, dsc_next);
#pragma unroll
      for (int b = 0; b < TM; ++b) {
        const float d = dsc[b];
        if (b == 1) asm volatile("" : "+v"(dsc_next[0]), "+v"(dsc_next[1]), "+v"(dsc_next[2]), "+v"(dsc_next[3]));
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
      load_scales(nm0, dsc_next);
      asm volatile("" : "+v"(dsc_next[0]), "+v"(dsc_next[1]), "+v"(dsc_next[2]), "+v"(dsc_next[3]));
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
    m0 = nm0;
    n0 = nn0;
#pragma unroll
    for (int b = 0; b < TM; ++b) dsc[b] = dsc_next[b];
    if (OUT == 0 && !ACC && interior) {
      steps_behind_stores = 2;
    } else {
      GX_WAIT_LOADS(0);                // a store count that depends on the tile: wait for all of them
      steps_behind_stores = 0;
    }
    __syncthreads();                   // transpose space has been read out by every wave
    // the loads that were held back: first half of the step after the next three
#pragma unroll
    for (int p = 0; p < GX_LOADS_PER_STEP / 2; ++p) dma_part(cur, lds0 + free_stage * GX_STAGE, p);
  }
  GX_WAIT_LOADS(0);                    // no copy may be in flight when the LDS is released
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
  const int KB = (int)(bl_round_up(K, BL_KPAD) / 128);
  const int MT = (int)((M + GX_BM - 1) / GX_BM), NTB = (int)((N + GX_BN - 1) / GX_BN);
  const int out = (ydt == BL_BF16 && (N & 7) == 0) ? 0 : ((N & 3) == 0 ? 1 : 2);
  const int yb = ydt == BL_BF16 ? 1 : 0;
#define GX_CALL(OUT, ACC) gx_go<OUT, ACC>(q, scale, (int)M, KB, Wp, alpha, (int)N, Y, yb, acc_out, MT, NTB, s)
  if (acc_out) return out == 0 ? GX_CALL(0, true) : out == 1 ? GX_CALL(1, true) : GX_CALL(2, true);
  return out == 0 ? GX_CALL(0, false) : out == 1 ? GX_CALL(1, false) : GX_CALL(2, false);
#undef GX_CALL
}
