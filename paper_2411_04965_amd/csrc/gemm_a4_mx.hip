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
// window).  The copy from global memory to LDS is therefore linear: lane l of a wave moves bytes
// 16 l .. 16 l + 15 of a 1 KB piece, no address arithmetic and no vector work on the way.
// The copy goes through registers (global_load_dwordx4, one step later ds_write_b128).  The
// direct global-to-LDS load was measured at 33 bytes per clock and CU for data that hits in L2,
// plain loads at more than 50; the 256 x 256 tile needs 40 bytes per MFMA-bound clock.
//
// Structure.  Persistent blocks (one per CU) walk the tile list; block = 4 waves, tile
// 256 x 256, each wave 128 x 128 as 4 x 4 MFMA tiles; the MFMA's row operand is the weight
// fragment and its column operand the token fragment, so a lane ends up with groups of 4
// consecutive outputs n of one token.  K advances 128 channels per step through two LDS
// stages, two MFMA sub-steps of 64 channels each, with two register sets of fragments: a
// sub-step computes on one set while the other is filled for the next.  One step is one
// straight-line block with one barrier in the middle:
//   sub-step 0  computes on F[0], reads F[1] (sub-step 1 of this step) from the own stage, and
//               writes the weights of step g + 1 into the other stage;
//   barrier
//   sub-step 1  computes on F[1], reads F[0] (sub-step 0 of step g + 1) from the other stage,
//               and writes the activations of step g + 2 into the own stage, which nobody
//               reads any more once the barrier has been passed.
// So a stage is read only before the barrier of its own step (second fragments) and behind the
// barrier of the step before (first fragments), and every write is separated from the reads of
// the data it replaces and of the data it brings by a barrier.  Each staging register is
// refilled from global memory right behind the write that consumed it, a full step before it is
// written out again.  The K stream of a block runs on across its tiles.  Each wave copies the
// row blocks 2w and 2w + 1 of both operands.
#include <type_traits>

#include "common.h"

#define GX_THREADS 256
#define GX_BM 256
#define GX_BN 256
#define GX_XQ 16384                  // stage layout: [XP 8 x 2048 | XQ 8 x 1024 | W 8 x 2048]
#define GX_W 24576
#define GX_STAGE 40960
#define GX_TB (2 * GX_STAGE)         // transpose space of the epilogue, behind the two stages
#define GX_TB_BYTES 36864
#define GX_LDS (GX_TB + GX_TB_BYTES)
#define GX_A_BLOCK 3072              // bytes of 32 tokens x 128 channels of 6-bit codes
#define GX_W_BLOCK 2048              // bytes of 32 outputs x 128 channels of 4-bit codes

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v6i __attribute__((ext_vector_type(6)));
typedef float v16f __attribute__((ext_vector_type(16)));

__device__ __forceinline__ u32 gx_pack_bf16(float lo, float hi) {
  u32 r;
  asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
  return r;
}

// OUT: 0 = bf16 rows through the LDS transpose (N % 8 == 0), 1 = 4 outputs per store (N % 4 == 0),
// 2 = one output per store (any N).  ACC: also write the integer accumulators (tests).
// FP4: the activations are E2M1 codes with one E8M0 scale per token and 32 channels (eq. 8-9)
// instead of E3M2 codes of INT4 levels: 2 KB instead of 3 KB per block, the same instruction in its
// scaled form with the block scales as the column operand's scale (`xsc`, 128 bytes per block in
// block order; each lane holds exactly one 32-channel block of one token per instruction), no
// per-token scale, float32 sums that are no longer integers.
// W2: the weights arrive as 2-bit codes (1 KB per block, BL_W_MX2) and are expanded to E2M1 nibbles
// in registers behind the fragment read (3 vector instructions per 16 channels) instead of being
// stored expanded: half the weight bytes from HBM, L2 and LDS, two instead of four pieces per
// wave and step.
// GLU: gate and up projection of an FFN in one pass with eq. 5 in the epilogue.  Wp / Wp2 are the gate
// and the up weights ([N, K] each); a 256-column tile is 128 outputs of both: weight rows 64 w .. 64 w + 63
// of the tile (the rows wave w stages) are gate outputs for even w and up outputs for odd w, of the
// same 64 outputs, so the wave that owns columns 128 wn .. holds G in its column tiles 0, 1 and U of
// the same outputs in its column tiles 2, 3.  The epilogue forms H = bf16(U * max(G, 0)^2) from the
// rescaled float32 values (the order of relu2_glu) and writes H[M, N] only; G and U never leave
// the registers.
template <int OUT, bool ACC, bool FP4, bool W2, bool GLU = false>
__global__ __launch_bounds__(GX_THREADS, 1) void gemm_a4_mx_kernel(
    const unsigned char* __restrict__ A, const float* __restrict__ scale,
    const unsigned char* __restrict__ xsc, int M, int KB,
    const unsigned char* __restrict__ Wp, const float* __restrict__ alpha_p, int N, void* __restrict__ Y,
    int y_bf16, int32_t* __restrict__ acc_out, int MT, int NTB,
    const unsigned char* __restrict__ Wp2 = nullptr, const float* __restrict__ alpha2_p = nullptr) {
  extern __shared__ __align__(16) unsigned char gx_smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;     // MFMA operand row / k-half of this lane
  const int n_tiles = MT * NTB;
  const int MB = (M + 31) >> 5, NB = (N + 31) >> 5;           // 32-row blocks of the operands
  constexpr int WM = 128, WN = 128, TM = 4, TN = 4;
  constexpr int LA = FP4 ? 4 : 6, LB = W2 ? 2 : 4;   // 1 KB pieces per wave and step: activations, weights
  constexpr int A_BLOCK = FP4 ? 2048 : GX_A_BLOCK;
  constexpr int W_BLOCK = W2 ? 1024 : GX_W_BLOCK;

  // ---- global loads.  One cursor per operand names the (tile, K step) that is loaded next and
  // moves on along the block's stream of tiles by itself; weights run two steps ahead of the
  // MFMAs, activations three.
  struct Cursor {
    const unsigned char* p[2];                   // row blocks 2w and 2w + 1 of the operand
    int kb, tile;
  };
  auto point = [&](Cursor& c, int tile, bool is_a) {
    int m0, n0;
    bl_tile_origin(tile, n_tiles, MT, NTB, GX_BM, GX_BN, m0, n0);
    c.tile = tile;
    c.kb = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      // row blocks past the end of an operand re-read its last block (their results are never stored)
      if (is_a) c.p[i] = A + (size_t)min((m0 >> 5) + 2 * wave + i, MB - 1) * KB * A_BLOCK;
      else if (GLU) c.p[i] = ((wave & 1) ? Wp2 : Wp) + (size_t)min((n0 >> 6) + 2 * (wave >> 1) + i, NB - 1) * KB * W_BLOCK;
      else c.p[i] = Wp + (size_t)min((n0 >> 5) + 2 * wave + i, NB - 1) * KB * W_BLOCK;
    }
  };
  // one step on; behind the block's last step the cursor stays where it is (loads that nobody uses)
  // (the usual case without a taken branch: it sits between two MFMA sequences)
  auto advance = [&](Cursor& c, bool is_a) {
    const bool last = c.kb + 1 == KB;
    const int by = last ? 0 : (is_a ? A_BLOCK : W_BLOCK);
    c.kb += last ? 0 : 1;
#pragma unroll
    for (int i = 0; i < 2; ++i) c.p[i] += by;
    if (__builtin_expect(last, 0)) {
      const int nt = c.tile + (int)gridDim.x;
      if (nt < n_tiles) point(c, nt, is_a);
    }
  };
  // Two sets of staging registers, used by even and odd steps in turn: a register is refilled
  // right behind the LDS write that consumed it and written out again two steps later, so a
  // load has two steps (about 1.5 microseconds) to arrive.
  v4i a_reg[2][LA], b_reg[2][LB];
  const int lane16 = lane * 16;
  // piece j of the activations: row block 2w + j / 3, there XP (2 KB) then XQ (1 KB); FP4 blocks
  // are 2 KB and go where XP goes
  constexpr int PA = LA / 2;                     // pieces per row block
  auto load_a = [&](const Cursor& c, int set, int j) {
    a_reg[set][j] = *reinterpret_cast<const v4i*>(c.p[j / PA] + (j % PA) * 1024 + lane16);
  };
  constexpr int PB = LB / 2;                     // pieces per row block
  auto load_b = [&](const Cursor& c, int set, int j) {
    b_reg[set][j] = *reinterpret_cast<const v4i*>(c.p[j / PB] + (j % PB) * 1024 + lane16);
  };
  auto store_a = [&](unsigned char* st, int set, int j) {
    const int rb = 2 * wave + j / PA, i = j % PA;
    unsigned char* dst = i < 2 ? st + rb * 2048 + i * 1024 : st + GX_XQ + rb * 1024;
    *reinterpret_cast<v4i*>(dst + lane16) = a_reg[set][j];
  };
  auto store_b = [&](unsigned char* st, int set, int j) {
    *reinterpret_cast<v4i*>(st + GX_W + (2 * wave + j / PB) * W_BLOCK + (j % PB) * 1024 + lane16) = b_reg[set][j];
  };

  // ---- FP4: block scales of the wave's four token blocks, one word (4 units) per lane and step,
  // fetched two steps ahead into two register sets like the operands
  struct SCursor {
    const unsigned char* p[TM];
    int kb, tile;
  };
  auto point_s = [&](SCursor& c, int tile) {
    int m0, n0;
    bl_tile_origin(tile, n_tiles, MT, NTB, GX_BM, GX_BN, m0, n0);
    c.tile = tile;
    c.kb = 0;
#pragma unroll
    for (int b = 0; b < TM; ++b)
      c.p[b] = xsc + (size_t)min((m0 >> 5) + wm * 4 + b, MB - 1) * KB * 128 + l32 * 4;
  };
  auto advance_s = [&](SCursor& c) {
    const bool last = c.kb + 1 == KB;
    const int by = last ? 0 : 128;
    c.kb += last ? 0 : 1;
#pragma unroll
    for (int b = 0; b < TM; ++b) c.p[b] += by;
    if (__builtin_expect(last, 0)) {
      const int nt = c.tile + (int)gridDim.x;
      if (nt < n_tiles) point_s(c, nt);
    }
  };
  u32 sc_reg[2][TM];
  auto load_s = [&](const SCursor& c, int set) {
#pragma unroll
    for (int b = 0; b < TM; ++b) sc_reg[set][b] = *reinterpret_cast<const u32*>(c.p[b]);
  };

  // ---- fragment addresses (within a stage): lane (l32, lh) reads unit u = 2 s + lh of its row
  int xp_off[2], xq_off[2], w_off[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    const int u = 2 * s + lh;
    xp_off[s] = (wm * WM + l32) * 64 + ((u ^ ((l32 >> 2) & 3)) << 4);
    xq_off[s] = GX_XQ + (wm * WM + l32) * 32 + ((u ^ ((l32 >> 3) & 3)) << 3);
    w_off[s] = W2 ? GX_W + (wn * WN + l32) * 32 + ((u ^ ((l32 >> 3) & 3)) << 3)
                  : GX_W + (wn * WN + l32) * 64 + ((u ^ ((l32 >> 2) & 3)) << 4);
  }
  typedef typename std::conditional<FP4, v4i, v6i>::type XFrag;
  struct Frags {
    XFrag x[TM];
    v4i w[TN];
    v2i wr[TN];                                  // W2: the 2-bit codes as read, expanded a few slots later
  };
  auto read_x = [&](const unsigned char* st, int s, int b) -> XFrag {
    const v4i p = *reinterpret_cast<const v4i*>(st + xp_off[s] + b * 2048);
    if constexpr (FP4) {
      return p;
    } else {
      const v2i q = *reinterpret_cast<const v2i*>(st + xq_off[s] + b * 1024);
      return (v6i){p[0], p[1], p[2], p[3], q[0], q[1]};
    }
  };
  // two words of 16 two-bit codes (nibble j: sign and magnitude of channels j and 8 + j as bits
  // s_j s_8+j m_j m_8+j) -> four words of E2M1 nibbles in channel order (s 0 m 0)
  auto expand_w = [&](const v2i& w) -> v4i {
    const u32 w0 = (u32)w[0], w1 = (u32)w[1];
    return (v4i){(int)(w0 & 0xAAAAAAAAu), (int)((w0 << 1) & 0xAAAAAAAAu),
                 (int)(w1 & 0xAAAAAAAAu), (int)((w1 << 1) & 0xAAAAAAAAu)};
  };
  // ... done in the slot where it is written: the empty statements keep the compiler from moving
  // the arithmetic across the MFMAs around it in program order
  // (half h = word h of the codes -> words 2 h and 2 h + 1 of the fragment: three instructions)
  auto expand_here = [&](Frags& f, int a, int h) {
    u32 c = (u32)f.wr[a][h];
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("" : "+v"(c));                  // not earlier ...
#endif
    u32 lo = c & 0xAAAAAAAAu, hi = (c << 1) & 0xAAAAAAAAu;
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("" : "+v"(lo), "+v"(hi));       // ... and not later than here
#endif
    f.w[a][2 * h] = (int)lo;
    f.w[a][2 * h + 1] = (int)hi;
  };
  // W2: the read only (the expansion waits for the data, so it sits some MFMAs further down)
  auto read_w = [&](Frags& f, const unsigned char* st, int s, int a) {
    if constexpr (W2) f.wr[a] = *reinterpret_cast<const v2i*>(st + w_off[s] + a * 1024);
    else f.w[a] = *reinterpret_cast<const v4i*>(st + w_off[s] + a * 2048);
  };

  // The accumulators are pinned to AGPRs and updated in place.  (The host pass of the compiler
  // parses kernel bodies too and knows neither these register classes nor 192-bit operands, so it
  // sees empty statements here.)
#if defined(__HIP_DEVICE_COMPILE__)
#define GX_MFMA(C, WF, XF) \
  asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, %0 cbsz:4 blgp:3" : "+a"(C) : "v"(WF), "v"(XF))
// first MFMA on an accumulator tile: C = 0 (saves clearing 256 registers per output tile)
#define GX_MFMA0(C, WF, XF) \
  asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %1, %2, 0 cbsz:4 blgp:3" : "=a"(C) : "v"(WF), "v"(XF))
// scaled form, both operands E2M1: SA / SX = scale words of the row / column operand, of which the
// instruction takes byte 0 (HI = 0) or byte 2 (HI = 1) of SX and byte 0 of SA
#define GX_MFMA_S(C, WF, XF, SA, SX, HI)                                                              \
  asm volatile("v_mfma_scale_f32_32x32x64_f8f6f4 %0, %1, %2, %0, %3, %4 op_sel_hi:[0," #HI ",0] cbsz:4 blgp:4" \
               : "+a"(C) : "v"(WF), "v"(XF), "v"(SA), "v"(SX))
#define GX_MFMA0_S(C, WF, XF, SA, SX, HI)                                                             \
  asm volatile("v_mfma_scale_f32_32x32x64_f8f6f4 %0, %1, %2, 0, %3, %4 op_sel_hi:[0," #HI ",0] cbsz:4 blgp:4" \
               : "=a"(C) : "v"(WF), "v"(XF), "v"(SA), "v"(SX))
#else
#define GX_MFMA(C, WF, XF) ((void)0)
#define GX_MFMA0(C, WF, XF) ((void)0)
#define GX_MFMA_S(C, WF, XF, SA, SX, HI) ((void)0)
#define GX_MFMA0_S(C, WF, XF, SA, SX, HI) ((void)0)
#endif
  [[maybe_unused]] const u32 one_scale = 127u;   // E8M0 of 2^0 for the ternary weights

  const float alpha = alpha_p[0];

  // ---- first tile of this block: stage 0 <- step 0, activation areas of stage 1 <- step 1,
  // registers <- weights of steps 1, 2 and activations of steps 2, 3; fragments <- step 0
  int tile = blockIdx.x;
  int m0, n0;
  bl_tile_origin(tile, n_tiles, MT, NTB, GX_BM, GX_BN, m0, n0);
  Cursor ca, cb;
  point(ca, tile, true);
  point(cb, tile, false);
  SCursor cs;
  if constexpr (FP4) {                           // scales of steps 0 and 1
    point_s(cs, tile);
    load_s(cs, 0);
    advance_s(cs);
    load_s(cs, 1);
    advance_s(cs);
  }
#pragma unroll
  for (int j = 0; j < LA; ++j) load_a(ca, 0, j);
#pragma unroll
  for (int j = 0; j < LB; ++j) load_b(cb, 0, j);
  advance(ca, true);
  advance(cb, false);
#pragma unroll
  for (int j = 0; j < LA; ++j) load_a(ca, 1, j);
  advance(ca, true);
#pragma unroll
  for (int j = 0; j < LA; ++j) store_a(gx_smem, 0, j);
#pragma unroll
  for (int j = 0; j < LB; ++j) store_b(gx_smem, 0, j);
#pragma unroll
  for (int j = 0; j < LA; ++j) store_a(gx_smem + GX_STAGE, 1, j);
  // (in the order in which the loop refills them: weights of an even step, activations of an even
  // step, weights of an odd step, activations of an odd step.  The compiler derives the loop's
  // wait counts from the oldest-first order of the loads in flight on every path into the loop)
#pragma unroll
  for (int j = 0; j < LB; ++j) load_b(cb, 0, j);               // weights of step 1: written by step 0
  advance(cb, false);
#pragma unroll
  for (int j = 0; j < LA; ++j) load_a(ca, 0, j);               // activations of step 2: written by step 0
  advance(ca, true);
#pragma unroll
  for (int j = 0; j < LB; ++j) load_b(cb, 1, j);               // weights of step 2: written by step 1
  advance(cb, false);
#pragma unroll
  for (int j = 0; j < LA; ++j) load_a(ca, 1, j);               // activations of step 3: written by step 1
  advance(ca, true);
  __syncthreads();
  Frags F[2];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    F[0].x[i] = read_x(gx_smem, 0, i);
    read_w(F[0], gx_smem, 0, i);
  }
  if constexpr (W2) F[0].w[0] = expand_w(F[0].wr[0]);

  while (true) {
    const int next = tile + (int)gridDim.x;
    const bool has_next = next < n_tiles;
    const bool interior = (m0 + GX_BM <= M) && (GLU ? (n0 >> 1) + GX_BN / 2 <= N : n0 + GX_BN <= N);
    v16f acc[TN][TM];
    // Per-token scales of this tile, fetched now: a global load inside the epilogue would have
    // to wait for the stores issued before it (loads and stores share one counter).
    float dsc[TM];
#pragma unroll
    for (int b = 0; b < TM; ++b) {
      const int m = m0 + wm * WM + b * 32 + l32;
      if constexpr (FP4) dsc[b] = 1.0f;          // (acc * 1) * alpha: the scales are inside acc
      else dsc[b] = m < M ? scale[m] : 0.0f;
    }

    // One step; PAR = parity of the step = its stage and its set of staging registers (KB is
    // even, so the parity carries over from tile to tile).
    auto step = [&](auto par, bool first) {
      constexpr int PAR = decltype(par)::value;
      unsigned char* st_own = gx_smem + PAR * GX_STAGE;
      unsigned char* st_other = gx_smem + (PAR ^ 1) * GX_STAGE;
      // FP4: this step's scale words; a lane of the upper half (units 1 and 3) moves its bytes down,
      // so that the instruction takes byte 0 in sub-step 0 and byte 2 in sub-step 1
      u32 sx[TM];
#pragma unroll
      for (int b = 0; b < TM; ++b) sx[b] = FP4 ? sc_reg[PAR][b] >> (8 * lh) : 0u;
      // ---- sub-step 0.  Slots behind the MFMAs: fragment reads first, then one LDS write and
      // the global load that refills its register (a 16-byte LDS write costs the MFMA stream
      // least directly behind the reads, and nothing here is vector arithmetic).
#pragma unroll
      for (int a = 0; a < TN; ++a) {
#pragma unroll
        for (int b = 0; b < TM; ++b) {
          if constexpr (FP4) {
            if (first) GX_MFMA0_S(acc[a][b], F[0].w[a], F[0].x[b], one_scale, sx[b], 0);
            else GX_MFMA_S(acc[a][b], F[0].w[a], F[0].x[b], one_scale, sx[b], 0);
          } else {
            if (first) GX_MFMA0(acc[a][b], F[0].w[a], F[0].x[b]);
            else GX_MFMA(acc[a][b], F[0].w[a], F[0].x[b]);
          }
          const int i = a * TM + b;              // one slot behind each MFMA
          if (i < 4) F[1].x[i] = read_x(st_own, 1, i);
          else if (i < 8) read_w(F[1], st_own, 1, i - 4);
          else if (i % 2 == 0 && (i - 8) / 2 < LB) {   // slots 8, 10, ...: weights of the next step
            store_b(st_other, PAR, (i - 8) / 2);
            load_b(cb, PAR, (i - 8) / 2);
          }
          if constexpr (W2) {                    // codes -> E2M1, one row of MFMAs ahead of its use
            if ((b == 1 || b == 2) && a + 1 < TN) expand_here(F[0], a + 1, b - 1);
            if (i == 13 || i == 14) expand_here(F[1], 0, i - 13);
          }
        }
      }
      advance(cb, false);
      __syncthreads();
      // ---- sub-step 1
#pragma unroll
      for (int a = 0; a < TN; ++a) {
#pragma unroll
        for (int b = 0; b < TM; ++b) {
          if constexpr (FP4) GX_MFMA_S(acc[a][b], F[1].w[a], F[1].x[b], one_scale, sx[b], 1);
          else GX_MFMA(acc[a][b], F[1].w[a], F[1].x[b]);
          const int i = a * TM + b;
          if (i < 4) F[0].x[i] = read_x(st_other, 0, i);
          else if (i < 8) read_w(F[0], st_other, 0, i - 4);
          else if (i < 8 + LA) {                 // slots 8 ..: activations of the step after next
            store_a(st_own, PAR, i - 8);
            load_a(ca, PAR, i - 8);
          }
          if constexpr (W2) {
            if ((b == 1 || b == 2) && a + 1 < TN) expand_here(F[1], a + 1, b - 1);
            if (i == 13 || i == 14) expand_here(F[0], 0, i - 13);
          }
        }
      }
      advance(ca, true);
      if constexpr (FP4) {                       // scales of the step after next
        load_s(cs, PAR);
        advance_s(cs);
      }
    };
    for (int kb = 0; kb < KB; kb += 2) {
      step(std::integral_constant<int, 0>{}, kb == 0);
      step(std::integral_constant<int, 1>{}, false);
    }
    // The MFMAs are issued from inline assembly: the compiler does not know that their results
    // need wait states before a vector instruction may read them.
    asm volatile("s_nop 15\n\ts_nop 7" ::: "memory");

    // The staging registers already hold data of the next tile: make their loads complete
    // here, before the epilogue's stores join the same counter.
#pragma unroll
    for (int set = 0; set < 2; ++set) {
#pragma unroll
      for (int j = 0; j < LA; ++j) asm volatile("" ::"v"(a_reg[set][j]));
#pragma unroll
      for (int j = 0; j < LB; ++j) asm volatile("" ::"v"(b_reg[set][j]));
    }

    // ---- epilogue.  acc[a][b][r] is output n = 32 a + 8 (r / 4) + 4 lh + r % 4 of token
    // m = 32 b + l32 (relative to the wave tile).  bf16 rows leave through an LDS transpose
    // (its own space behind the stages) so that every store instruction writes whole lines.
    if constexpr (GLU) {
      // acc[a][b] (a = 0, 1) is G and acc[a + 2][b] is U of output n = n0 / 2 + 64 wn + 32 a + 8 (r / 4) +
      // 4 lh + r % 4, token m = 32 b + l32 of the wave tile
      const float alpha2 = alpha2_p[0];
      const int nw = (n0 >> 1) + wn * (WN / 2);                // first H column of this wave
      if (OUT == 0) {
        constexpr int TB_ROW = WN + 32;                      // 64 bfloat16 per token + padding
        unsigned char* tbuf = gx_smem + GX_TB + wave * (32 * (WN * 2 + 32));
        constexpr int LANES_PER_ROW = WN / 16;               // 8 lanes cover one token's 128 bytes
        constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
        constexpr int NPASS = 32 / ROWS_PER_PASS;
        const int rr = lane / LANES_PER_ROW, cc = lane % LANES_PER_ROW;
        uint16_t* ywave = (uint16_t*)Y + (size_t)(m0 + wm * WM) * N + nw;
        const u32 lane_off = (u32)rr * (u32)N + cc * 8;
        const int m_left = M - (m0 + wm * WM) - rr, n_left = N - nw - cc * 8;
#pragma unroll
        for (int b = 0; b < TM; ++b) {
          const float d = dsc[b];
#pragma unroll
          for (int a = 0; a < TN / 2; ++a) {
            asm volatile("" : "+a"(acc[a][b]));
            asm volatile("" : "+a"(acc[a + 2][b]));
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              float hv[4];
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const float g = (acc[a][b][4 * q4 + r] * d) * alpha;
                const float u = (acc[a + 2][b][4 * q4 + r] * d) * alpha2;
                const float rl = fmaxf(g, 0.0f);
                const float rr2 = rl * rl;
                hv[r] = u * rr2;
              }
              uint2 p;
              p.x = gx_pack_bf16(hv[0], hv[1]);
              p.y = gx_pack_bf16(hv[2], hv[3]);
              *reinterpret_cast<uint2*>(tbuf + l32 * TB_ROW + (a * 32 + 8 * q4 + 4 * lh) * 2) = p;
            }
            __builtin_amdgcn_sched_barrier(0);
          }
#pragma unroll
          for (int i = 0; i < NPASS; ++i) {
            const int row = b * 32 + i * ROWS_PER_PASS;
            const v4i v = *reinterpret_cast<const v4i*>(tbuf + (rr + i * ROWS_PER_PASS) * TB_ROW + cc * 16);
            if (interior || (row < m_left && 0 < n_left)) *reinterpret_cast<v4i*>(ywave + (size_t)row * N + lane_off) = v;
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      } else {
#pragma unroll
        for (int b = 0; b < TM; ++b) {
          const int m = m0 + wm * WM + b * 32 + l32;
          const float d = dsc[b];
#pragma unroll
          for (int a = 0; a < TN / 2; ++a) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
              const int n = nw + a * 32 + 8 * q4 + 4 * lh;
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const float g = (acc[a][b][4 * q4 + r] * d) * alpha;
                const float u = (acc[a + 2][b][4 * q4 + r] * d) * alpha2;
                const float rl = fmaxf(g, 0.0f);
                const float rr2 = rl * rl;
                if (m < M && n + r < N) ((uint16_t*)Y)[(size_t)m * N + n + r] = bl_f32_to_bf16_rne(u * rr2);
              }
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    } else
    if (OUT == 0) {
      constexpr int TB_ROW = WN * 2 + 32;
      unsigned char* tbuf = gx_smem + GX_TB + wave * (32 * TB_ROW);
      static_assert(4 * 32 * TB_ROW <= GX_TB_BYTES, "transpose space");
      constexpr int LANES_PER_ROW = WN * 2 / 16;           // 16 lanes cover one token's 256 bytes
      constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
      constexpr int NPASS = 32 / ROWS_PER_PASS;
      const int rr = lane / LANES_PER_ROW, cc = lane % LANES_PER_ROW;
      uint16_t* ywave = (uint16_t*)Y + (size_t)(m0 + wm * WM) * N + (n0 + wn * WN);
      const u32 lane_off = (u32)rr * (u32)N + cc * 8;
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
    // (no barrier: the epilogue touches neither stage, and each wave has its own transpose space)
  }
#undef GX_MFMA
#undef GX_MFMA0
}

template <int OUT, bool ACC, bool FP4, bool W2>
static int gx_go(const void* q, const float* scale, const uint8_t* xsc, int M, int KB, const void* Wp,
                 const float* alpha, int N, void* Y, int y_bf16, int32_t* acc_out, int MT, int NTB,
                 hipStream_t s) {
  BL_SET_MAX_LDS_ONCE((gemm_a4_mx_kernel<OUT, ACC, FP4, W2>), GX_LDS);
  const int grid = min(MT * NTB, bl_num_cus());      // persistent blocks, one per CU (all of its LDS)
  gemm_a4_mx_kernel<OUT, ACC, FP4, W2><<<(unsigned)grid, GX_THREADS, GX_LDS, s>>>(
      (const unsigned char*)q, scale, (const unsigned char*)xsc, M, KB, (const unsigned char*)Wp, alpha, N, Y,
      y_bf16, acc_out, MT, NTB);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

int bl_launch_gemm_a4_mx(const void* q, const float* scale, int64_t M, int64_t K, const void* Wp, bool w2,
                         const float* alpha, int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out,
                         hipStream_t s) {
  const int KB = (int)(bl_round_up(K, BL_KPAD) / 128);
  const int MT = (int)((M + GX_BM - 1) / GX_BM), NTB = (int)((N + GX_BN - 1) / GX_BN);
  const int out = (ydt == BL_BF16 && (N & 7) == 0) ? 0 : ((N & 3) == 0 ? 1 : 2);
  const int yb = ydt == BL_BF16 ? 1 : 0;
#define GX_CALL(OUT, ACC) \
  (w2 ? gx_go<OUT, ACC, false, true>(q, scale, nullptr, (int)M, KB, Wp, alpha, (int)N, Y, yb, acc_out, MT, NTB, s) \
      : gx_go<OUT, ACC, false, false>(q, scale, nullptr, (int)M, KB, Wp, alpha, (int)N, Y, yb, acc_out, MT, NTB, s))
  if (acc_out) return out == 0 ? GX_CALL(0, true) : out == 1 ? GX_CALL(1, true) : GX_CALL(2, true);
  return out == 0 ? GX_CALL(0, false) : out == 1 ? GX_CALL(1, false) : GX_CALL(2, false);
#undef GX_CALL
}

// Gate and up projection with the ReLU^2 GLU in the epilogue: H[M, N] bfloat16 from INT4 activations in the
// MX6 form and two weight matrices [N, K] in the same block-float layout.
template <int OUT, bool W2>
static int gx_go_glu(const void* q, const float* scale, int M, int KB, const void* Wg, const float* ag, const void* Wu,
                     const float* au, int N, void* H, int MT, int NTB, hipStream_t s) {
  BL_SET_MAX_LDS_ONCE((gemm_a4_mx_kernel<OUT, false, false, W2, true>), GX_LDS);
  const int grid = min(MT * NTB, bl_num_cus());
  gemm_a4_mx_kernel<OUT, false, false, W2, true><<<(unsigned)grid, GX_THREADS, GX_LDS, s>>>(
      (const unsigned char*)q, scale, nullptr, M, KB, (const unsigned char*)Wg, ag, N, H, 1, nullptr, MT, NTB,
      (const unsigned char*)Wu, au);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

int bl_launch_gemm_a4_mx_glu(const void* q, const float* scale, int64_t M, int64_t K, const void* Wg, const float* ag,
                             const void* Wu, const float* au, bool w2, int64_t N, void* H, hipStream_t s) {
  const int KB = (int)(bl_round_up(K, BL_KPAD) / 128);
  const int MT = (int)((M + GX_BM - 1) / GX_BM), NTB = (int)((N + GX_BN / 2 - 1) / (GX_BN / 2));
  const bool rows = (N & 7) == 0;
  if (w2) return rows ? gx_go_glu<0, true>(q, scale, (int)M, KB, Wg, ag, Wu, au, (int)N, H, MT, NTB, s)
                      : gx_go_glu<2, true>(q, scale, (int)M, KB, Wg, ag, Wu, au, (int)N, H, MT, NTB, s);
  return rows ? gx_go_glu<0, false>(q, scale, (int)M, KB, Wg, ag, Wu, au, (int)N, H, MT, NTB, s)
              : gx_go_glu<2, false>(q, scale, (int)M, KB, Wg, ag, Wu, au, (int)N, H, MT, NTB, s);
}

// FP4 activations (E2M1 codes and E8M0 block scales in the MX form) x BL_W_MX4 weights.
int bl_launch_gemm_fp4_mx(const void* q, const uint8_t* xscale, int64_t M, int64_t K, const void* Wp, bool w2,
                          const float* alpha, int64_t N, void* Y, bl_dtype ydt, hipStream_t s) {
  const int KB = (int)(bl_round_up(K, BL_KPAD) / 128);
  const int MT = (int)((M + GX_BM - 1) / GX_BM), NTB = (int)((N + GX_BN - 1) / GX_BN);
  const int out = (ydt == BL_BF16 && (N & 7) == 0) ? 0 : ((N & 3) == 0 ? 1 : 2);
  const int yb = ydt == BL_BF16 ? 1 : 0;
#define GX_CALL4(OUT) \
  (w2 ? gx_go<OUT, false, true, true>(q, nullptr, xscale, (int)M, KB, Wp, alpha, (int)N, Y, yb, nullptr, MT, NTB, s) \
      : gx_go<OUT, false, true, false>(q, nullptr, xscale, (int)M, KB, Wp, alpha, (int)N, Y, yb, nullptr, MT, NTB, s))
  return out == 0 ? GX_CALL4(0) : out == 1 ? GX_CALL4(1) : GX_CALL4(2);
#undef GX_CALL4
}
