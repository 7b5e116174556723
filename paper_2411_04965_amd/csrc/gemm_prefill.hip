// Prefill GEMM of the W1.58A4 and sparse W1.58A8 linears (eq. 6 and eq. 1 of the paper):
//   acc[m, n] = sum_k q[m, k] * T[n, k]   (exact int32 on v_mfma_i32_32x32x32_i8)
//   Y[m, n]   = (float(acc) * d[m]) * alpha
// Activations arrive packed (INT4 nibbles or INT8), weights 2-bit packed in 16 x 256 tiles.
// Both are expanded to int8 while they are copied into LDS, without sign extension:
//   an INT4 nibble is moved to the top of its byte  -> 16 * q,
//   a 2-bit ternary field is moved to the top of its byte -> 64 * T,
// so the MFMA accumulates 1024 * acc (64 * acc for INT8 activations); the factor is a power of
// two and is folded exactly into the per-token scale in the epilogue.
// |1024 * acc| <= 8 * K * 1024 < 2^31 for K <= 32768.
//
// Structure.  Persistent blocks (one per CU) walk the tile list.  Block = 4 waves, tile
// BM x BN, each wave (BM/2) x (BN/2) as 32x32 MFMA tiles; the MFMA's row operand is the weight
// fragment and its column operand the token fragment, so a lane ends up with groups of 4
// consecutive outputs n of one token.  K advances 128 channels per step through two LDS stages,
// four MFMA sub-steps of 32 channels each.  One step is one straight-line block with one
// barrier in the middle, and the copy work is split evenly over its halves: the first half
// (sub-steps 0, 1) expands the prefetched weights of the next step into the other stage, the
// second half (sub-steps 2, 3) expands the prefetched activations of the step after next into
// the activation area of the step's own stage, which nobody reads any more once the barrier
// has been passed; each half reads the MFMA fragments of the other half.  The K stream of a
// block runs on across its tiles (no per-tile prologue).  bf16 outputs leave through an LDS
// transpose so that every store instruction writes whole 128-byte lines.
//
// Issue budget.  A wave issues in order and one SIMD issues one instruction at a time; an
// MFMA costs 8 issue cycles and runs 32, a VALU operation costs 4, a 16-byte LDS access more.
// Everything that is not an MFMA must fit into the 24 free cycles behind each MFMA, so the
// per-step work is cut into small slots placed between individual MFMAs, and the 32x32x32
// MFMA is used instead of 16x16x64 (same rate, half as many instructions to issue).
#include "common.h"

#define GP_THREADS 256
#define GP_BK 128     // bytes (= int8 channels) per LDS row per stage

typedef int v16i __attribute__((ext_vector_type(16)));

template <int BM, int BN>
struct GpSmem {
  static constexpr int a_bytes = BM * GP_BK;
  static constexpr int b_bytes = BN * GP_BK;
  static constexpr int stage = a_bytes + b_bytes;
  // the bf16 transpose buffers of the epilogue (4 waves x 32 rows x (BN + 32) bytes) lie over
  // the weight area of stage 1 and run on into `extra` bytes behind it
  static constexpr int extra = 4096;
  static constexpr int total = 2 * stage + extra;
};

__device__ __forceinline__ int gp_lds_off(int row, int chunk) {
  // 16 lanes of a 16-byte access must fall into distinct 16-byte slots of a 256-byte window:
  // two rows per window, so the row's parity picks the half and (row / 2) % 8 permutes the chunks
  return row * GP_BK + ((chunk ^ ((row >> 1) & 7)) << 4);
}

__device__ __forceinline__ u32 gp_pack_bf16(float lo, float hi) {
  u32 r;
  asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
  return r;
}

// OUT: 0 = bf16 rows through the LDS transpose (N % 8 == 0), 1 = 4 outputs per store (N % 4 == 0),
// 2 = one output per store (any N).  ACC: also write the int32 accumulators (tests).
template <int BM, int BN, bool A4, int OUT, bool ACC>
__global__ __launch_bounds__(GP_THREADS, 1) void gemm_prefill_kernel(
    const unsigned char* __restrict__ A, const float* __restrict__ scale, int M, int Kp,
    const unsigned char* __restrict__ Wp, const float* __restrict__ alpha_p, int N, void* __restrict__ Y,
    int y_bf16, int32_t* __restrict__ acc_out, int MT, int NTB) {
  constexpr int WM = BM / 2, WN = BN / 2;        // wave tile
  constexpr int TM = WM / 32, TN = WN / 32;      // 32x32 MFMA tiles per wave
  constexpr int PA = A4 ? 4 : 8;                 // 16-byte pieces per activation row per stage
  constexpr int LA = BM * PA / GP_THREADS;       // activation loads per thread per stage
  constexpr int LB = BN * 2 / GP_THREADS;        // weight loads per thread per stage
  constexpr int STAGE = GpSmem<BM, BN>::stage;
  constexpr int A_BYTES = GpSmem<BM, BN>::a_bytes;
  extern __shared__ __align__(16) unsigned char gp_smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int l32 = lane & 31, lh = lane >> 5;     // MFMA operand row / k-group of this lane
  const int n_tiles16 = (N + 15) >> 4;
  const int k_tiles = Kp >> 8;
  const int a_row_bytes = A4 ? (Kp >> 1) : Kp;
  const int nk = Kp / GP_BK;
  const int n_tiles = MT * NTB;

  // ---- global sources: one uniform base per operand and tile plus a small per-lane offset.
  //   activations: load j of a thread covers row (tid / PA) + RPJ * j, 16-byte piece tid % PA
  //   weights:     load j covers 16-row tile (tid / 32) + 8 * j, row tid % 16, k-group (tid / 16) % 2
  constexpr int RPJ = GP_THREADS / PA;
  constexpr int KSB = A4 ? 64 : 128;             // activation bytes per row per step
  const u32 a_row0 = tid / PA, a_piece = (tid % PA) * 16;
  const u32 b_tile0 = tid >> 5, b_piece = (((tid >> 4) & 1) * 16 + (tid & 15)) * 16;
  const u32 b_tile_bytes = (u32)k_tiles * 1024;
  const int a_dst0 = A4 ? gp_lds_off(a_row0, 2 * (tid % PA)) : gp_lds_off(a_row0, tid % PA);
  const int b_dst0 = A_BYTES + gp_lds_off(b_tile0 * 16 + (tid & 15), 4 * ((tid >> 4) & 1));
  // The global loads run ahead of the MFMAs along the block's stream of (tile, K step) pairs,
  // weights by two steps and activations by three, and cross into the block's following tiles
  // on their own: each operand has a cursor with the uniform parameters of the tile it reads.
  struct Cursor {
    const unsigned char* base;                   // first row (activations) / weight tile of the tile
    u32 lim;                                     // rows / weight tiles past this one re-read it
    int ks, tile;
  };
  auto point_a = [&](Cursor& c, int m0) {
    c.base = A + (size_t)m0 * a_row_bytes;
    c.lim = (u32)(M - 1 - m0);
  };
  auto point_b = [&](Cursor& c, int n0) {
    c.base = Wp + (size_t)(n0 >> 4) * k_tiles * 1024;
    c.lim = (u32)(n_tiles16 - 1 - (n0 >> 4));
  };
  // one step on; behind the block's last tile the cursor stays on that tile (loads that nobody uses)
  auto advance = [&](Cursor& c, bool is_a) {
    if (++c.ks == nk) {
      c.ks = 0;
      const int nt = c.tile + (int)gridDim.x;
      if (nt < n_tiles) {
        int tm0, tn0;
        bl_tile_origin(nt, n_tiles, MT, NTB, BM, BN, tm0, tn0);
        c.tile = nt;
        if (is_a) point_a(c, tm0);
        else point_b(c, tn0);
      }
    }
  };

  uint4 a_reg[LA], b_reg[LB];
  auto load_a = [&](const Cursor& c, int j) {
    const u32 off = min(a_row0 + RPJ * j, c.lim) * (u32)a_row_bytes + a_piece;
    a_reg[j] = *reinterpret_cast<const uint4*>(c.base + (size_t)c.ks * KSB + off);
  };
  auto load_b = [&](const Cursor& c, int j) {
    const u32 off = min(b_tile0 + 8 * j, c.lim) * b_tile_bytes + b_piece;
    b_reg[j] = *reinterpret_cast<const uint4*>(c.base + (size_t)c.ks * 512 + off);
  };
  // The expansion of one stage is cut into NWR single 16-byte LDS writes per operand so that it
  // can be spread over the MFMA stream.  Rows of load j sit RPJ (resp. 128) rows below those of
  // load 0, a multiple of 16, so the swizzle is the same and the offset is an immediate.
  constexpr int NWR_A = A4 ? 2 * LA : LA;
  constexpr int NWR_B = 4 * LB;
  constexpr u32 MA = 0xF0F0F0F0u, MB = 0xC0C0C0C0u;
  auto store_a = [&](unsigned char* st, int i, const uint4& c) {
    if (A4) *reinterpret_cast<uint4*>(st + (i >> 1) * (RPJ * GP_BK) + (a_dst0 ^ ((i & 1) << 4))) = c;
    else *reinterpret_cast<uint4*>(st + i * (RPJ * GP_BK) + a_dst0) = c;
  };
  auto store_b = [&](unsigned char* st, int i, const uint4& c) {
    *reinterpret_cast<uint4*>(st + (i >> 2) * (128 * GP_BK) + (b_dst0 ^ ((i & 3) << 4))) = c;
  };
  auto a_word = [&](int i, int h) -> u32 {      // word h (0, 1) of activation piece i (INT4)
    const int j = i >> 1;
    return (i & 1) ? (h ? a_reg[j].w : a_reg[j].z) : (h ? a_reg[j].y : a_reg[j].x);
  };
  auto b_word = [&](int i) -> u32 {
    const int j = i >> 2, t = i & 3;
    return t == 0 ? b_reg[j].x : t == 1 ? b_reg[j].y : t == 2 ? b_reg[j].z : b_reg[j].w;
  };
  auto write_a = [&](unsigned char* st, int i) {
    uint4 c;
    if (A4) {
      const u32 x0 = a_word(i, 0), x1 = a_word(i, 1);
      c.x = (x0 << 4) & MA; c.y = x0 & MA; c.z = (x1 << 4) & MA; c.w = x1 & MA;
    } else {
      c = make_uint4(a_reg[i].x, a_reg[i].y, a_reg[i].z, a_reg[i].w);
    }
    store_a(st, i, c);
  };
  auto write_b = [&](unsigned char* st, int i) {
    const u32 w = b_word(i);
    uint4 c;
    c.x = (w << 6) & MB; c.y = (w << 4) & MB; c.z = (w << 2) & MB; c.w = w & MB;
    store_b(st, i, c);
  };

  // fragment addresses: row = wave base + tile * 32 + l32, 16-byte chunk = 2 * sub + lh
  const int xf_base = (wm * WM + l32) * GP_BK;
  const int wf_base = A_BYTES + (wn * WN + l32) * GP_BK;
  int swz[4];
#pragma unroll
  for (int sub = 0; sub < 4; ++sub) swz[sub] = ((2 * sub + lh) ^ ((l32 >> 1) & 7)) << 4;
  auto read_x = [&](int stage, int sub, int b) -> v4i {
    return *reinterpret_cast<const v4i*>(gp_smem + stage * STAGE + xf_base + b * (32 * GP_BK) + swz[sub]);
  };
  auto read_w = [&](int stage, int sub, int a) -> v4i {
    return *reinterpret_cast<const v4i*>(gp_smem + stage * STAGE + wf_base + a * (32 * GP_BK) + swz[sub]);
  };

  // Accumulators are pinned to AGPRs and updated in place: the tied "+a" operand keeps the
  // register allocator from rotating 256 accumulator registers through copies.
#define GP_MFMA(C, WF, XF) \
  asm volatile("v_mfma_i32_32x32x32_i8 %0, %1, %2, %0" : "+a"(C) : "v"(WF), "v"(XF))
  // The empty asm statements pin a slot's VALU work between two MFMAs: GP_PIN_IN makes an
  // input "change" at that point (nothing that depends on it can be scheduled earlier),
  // GP_PIN_OUT uses the results (they cannot be computed later).
#define GP_PIN_IN(x) asm volatile("" : "+v"(x))
#define GP_PIN_OUT(x, y) asm volatile("" ::"v"(x), "v"(y))
  static_assert(TM == TN && (TN == 2 || TN == 4), "the interleaving below assumes a square wave tile");
  constexpr int ROWS = 2 * TN;                   // MFMA rows (one weight fragment each) per half step
  static_assert(NWR_A == ROWS && NWR_B == ROWS, "one A write and one B write per MFMA row");
  constexpr int A_EVERY = ROWS / LA, B_EVERY = ROWS / LB;

  const float alpha = alpha_p[0];
  const float unscale = A4 ? (1.0f / 1024.0f) : (1.0f / 64.0f);
  constexpr int SHIFT = A4 ? 10 : 6;

  // ---- first tile of this block: stage 0 <- step 0, activation area of stage 1 <- step 1,
  // registers <- activations of step 2 and weights of step 1, fragments <- step 0
  int tile = blockIdx.x;
  int m0, n0;
  bl_tile_origin(tile, n_tiles, MT, NTB, BM, BN, m0, n0);
  Cursor ca, cb;
  ca.ks = cb.ks = 0;
  ca.tile = cb.tile = tile;
  point_a(ca, m0);
  point_b(cb, n0);
#pragma unroll
  for (int j = 0; j < LA; ++j) load_a(ca, j);
#pragma unroll
  for (int j = 0; j < LB; ++j) load_b(cb, j);
  advance(ca, true);
  advance(cb, false);
#pragma unroll
  for (int i = 0; i < NWR_A; ++i) write_a(gp_smem, i);
#pragma unroll
  for (int i = 0; i < NWR_B; ++i) write_b(gp_smem, i);
#pragma unroll
  for (int j = 0; j < LA; ++j) load_a(ca, j);
  advance(ca, true);
#pragma unroll
  for (int i = 0; i < NWR_A; ++i) write_a(gp_smem + STAGE, i);
  // (weights before activations, the order in which the loop refills them: the compiler derives
  // the loop's wait counts from the oldest-first order of the loads in flight on every path)
#pragma unroll
  for (int j = 0; j < LB; ++j) load_b(cb, j);
#pragma unroll
  for (int j = 0; j < LA; ++j) load_a(ca, j);
  advance(ca, true);
  advance(cb, false);
  __syncthreads();
  // Two full fragment sets, one per half step.  Each half reads the other half's set, so a
  // stage is read only before the barrier of its own step (second-half fragments) and after
  // the barrier of the step before (first-half fragments).  Writes: weights of step k + 1 go
  // to the other stage before the barrier of step k and are first read behind it; activations
  // of step k + 2 go to step k's own stage behind its barrier and are first read behind the
  // barrier of step k + 1.  One barrier per step orders everything.
  v4i xF[2][TM], wF[2][TN];                      // sub-steps 0, 1
  v4i xS[2][TM], wS[2][TN];                      // sub-steps 2, 3
#pragma unroll
  for (int sub = 0; sub < 2; ++sub)
#pragma unroll
    for (int a = 0; a < TN; ++a) {
      xF[sub][a] = read_x(0, sub, a);
      wF[sub][a] = read_w(0, sub, a);
    }

  while (true) {
    // The K stream runs on across tile boundaries: the last steps of a tile already fetch and
    // expand the first steps of the block's next tile, so that tile starts with its stages,
    // staging registers and fragments in place (nk is even: stage parity carries over).
    const int next = tile + (int)gridDim.x;
    const bool has_next = next < n_tiles;

    v16i acc[TN][TM];
#pragma unroll
    for (int a = 0; a < TN; ++a)
#pragma unroll
      for (int b = 0; b < TM; ++b)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[a][b][r] = 0;
    // Per-token scales of this tile, fetched now: a global load inside the epilogue would have
    // to wait for the stores issued before it (loads and stores share one counter).
    float dsc[TM];
#pragma unroll
    for (int b = 0; b < TM; ++b) {
      const int m = m0 + wm * WM + b * 32 + l32;
      dsc[b] = (m < M ? scale[m] : 0.0f) * unscale;
    }

    for (int ks = 0; ks < nk; ++ks) {
      const int stage = ks & 1;
      unsigned char* st_own = gp_smem + stage * STAGE;
      unsigned char* st_other = gp_smem + (stage ^ 1) * STAGE;

      // first half: sub-steps 0, 1 (k 0..63) on this step's stage.  Per MFMA row: one token
      // and one weight fragment of the second half, one weight piece (the next step's)
      // expanded into the other stage, and the global loads that refill the weight staging
      // registers just consumed (a full step before their data is expanded).
      // Order inside a row, from measurement: a 16-byte LDS write costs about 30 issue cycles
      // and stalls the MFMA stream least directly behind the fragment reads and not behind
      // vector instructions, which in turn are free at up to 4 per MFMA gap.  So a row writes
      // the piece expanded during the row before it and then expands its own.
      {
        uint4 cw_prev;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
          for (int a = 0; a < TN; ++a) {
            const int hrow = sub * TN + a;       // row within the half step
            uint4 cw;
            u32 w = b_word(hrow);
#pragma unroll
            for (int b = 0; b < TM; ++b) {
              GP_MFMA(acc[a][b], wF[sub][a], xF[sub][b]);
              // slots behind MFMA b of this row (4 per row; a 2-MFMA row takes two at a time)
              const int s0 = (TM == 4) ? b : 2 * b, s1 = (TM == 4) ? b : 2 * b + 1;
              if (s0 == 0) {
                xS[sub][a] = read_x(stage, 2 + sub, a);
                wS[sub][a] = read_w(stage, 2 + sub, a);
              }
              if (s0 <= 1 && 1 <= s1) {
                if (hrow > 0) store_b(st_other, hrow - 1, cw_prev);
              }
              if (s0 <= 2 && 2 <= s1) {
                GP_PIN_IN(w);
                cw.x = (w << 6) & MB; cw.y = (w << 4) & MB;
                GP_PIN_OUT(cw.x, cw.y);
              }
              if (s0 <= 3 && 3 <= s1) {
                GP_PIN_IN(w);
                cw.z = (w << 2) & MB; cw.w = w & MB;
                GP_PIN_OUT(cw.z, cw.w);
                if (hrow % B_EVERY == B_EVERY - 1) load_b(cb, hrow / B_EVERY);
              }
            }
            cw_prev = cw;
          }
        }
        store_b(st_other, ROWS - 1, cw_prev);
      }
      advance(cb, false);
      __syncthreads();
      // second half: sub-steps 2, 3 (k 64..127).  Per MFMA row: one token and one weight
      // fragment of the next step's first half from the other stage, one activation piece (of
      // the step after next) expanded into this step's own stage, and the global loads that
      // refill the activation staging registers.
      {
        uint4 cx_prev;
#pragma unroll
        for (int sub = 0; sub < 2; ++sub) {
#pragma unroll
          for (int a = 0; a < TN; ++a) {
            const int hrow = sub * TN + a;
            uint4 cx;
            u32 x0 = 0, x1 = 0;
            if (A4) {
              x0 = a_word(hrow, 0);
              x1 = a_word(hrow, 1);
            }
#pragma unroll
            for (int b = 0; b < TM; ++b) {
              GP_MFMA(acc[a][b], wS[sub][a], xS[sub][b]);
              const int s0 = (TM == 4) ? b : 2 * b, s1 = (TM == 4) ? b : 2 * b + 1;
              if (s0 == 0) {
                xF[sub][a] = read_x(stage ^ 1, sub, a);
                wF[sub][a] = read_w(stage ^ 1, sub, a);
              }
              if (s0 <= 1 && 1 <= s1) {
                if (A4) {
                  if (hrow > 0) store_a(st_own, hrow - 1, cx_prev);
                } else {                          // INT8: a plain copy, nothing to wait for
                  store_a(st_own, hrow, make_uint4(a_reg[hrow].x, a_reg[hrow].y, a_reg[hrow].z, a_reg[hrow].w));
                }
              }
              if (s0 <= 2 && 2 <= s1) {
                if (A4) {
                  GP_PIN_IN(x0);
                  cx.x = (x0 << 4) & MA; cx.y = x0 & MA;
                  GP_PIN_OUT(cx.x, cx.y);
                }
              }
              if (s0 <= 3 && 3 <= s1) {
                if (A4) {
                  GP_PIN_IN(x1);
                  cx.z = (x1 << 4) & MA; cx.w = x1 & MA;
                  GP_PIN_OUT(cx.z, cx.w);
                }
                if (hrow % A_EVERY == A_EVERY - 1) load_a(ca, hrow / A_EVERY);
              }
            }
            if (A4) cx_prev = cx;
          }
        }
        if (A4) store_a(st_own, ROWS - 1, cx_prev);
      }
      advance(ca, true);
      // The MFMAs are issued from inline assembly, so the compiler does not know that their
      // results need wait states before a VALU may read them; the register allocator reads
      // accumulators right at the loop exit.  16 wait states here cover the last MFMA.
      asm volatile("s_nop 15" ::: "memory");
    }

    // The staging registers already hold data of the next tile: make their loads complete
    // here, before the epilogue's stores join the same counter.
#pragma unroll
    for (int j = 0; j < LA; ++j) asm volatile("" ::"v"(a_reg[j].x), "v"(a_reg[j].y), "v"(a_reg[j].z), "v"(a_reg[j].w));
#pragma unroll
    for (int j = 0; j < LB; ++j) asm volatile("" ::"v"(b_reg[j].x), "v"(b_reg[j].y), "v"(b_reg[j].z), "v"(b_reg[j].w));

    // ---- epilogue.  acc[a][b][r] is output n = 32 a + 8 (r / 4) + 4 lh + r % 4 of token
    // m = 32 b + l32 (relative to the wave tile).  float(1024 acc) * (d / 1024) rounds exactly
    // like float(acc) * d.
    if (OUT == 0) {
      // bf16 through an LDS transpose, 32 tokens x WN outputs at a time.  The last step ran
      // on stage 1 (nk is even); stage 0 and the activation area of stage 1 already hold the
      // next tile's first two steps, but the weight area of stage 1 was last read before the
      // last barrier and is written again only in the next tile's first step, behind the
      // barrier at the end of the epilogue.  Rows are padded by 32 bytes against bank
      // conflicts; read back row-wise, 16 lanes cover one token's WN * 2 contiguous bytes, so
      // every store instruction writes whole 128-byte lines.
      constexpr int TB_ROW = WN * 2 + 32;
      unsigned char* tbuf = gp_smem + STAGE + A_BYTES + wave * (32 * TB_ROW);
      static_assert(4 * 32 * TB_ROW <= GpSmem<BM, BN>::b_bytes + GpSmem<BM, BN>::extra,
                    "transpose buffers must fit into the weight area of stage 1 plus the tail");
      constexpr int LANES_PER_ROW = WN * 2 / 16;           // 16 (WN = 128) or 8 (WN = 64)
      constexpr int ROWS_PER_PASS = 64 / LANES_PER_ROW;
      const int rr = lane / LANES_PER_ROW, cc = lane % LANES_PER_ROW;
      // uniform base of the wave's output block plus one per-lane offset: the stores need no
      // per-store address registers
      uint16_t* ywave = (uint16_t*)Y + (size_t)(m0 + wm * WM) * N + (n0 + wn * WN);
      const u32 lane_off = (u32)rr * (u32)N + cc * 8;
      const bool interior = (m0 + BM <= M) && (n0 + BN <= N);
      const int m_left = M - (m0 + wm * WM) - rr, n_left = N - (n0 + wn * WN) - cc * 8;
#pragma unroll
      for (int b = 0; b < TM; ++b) {
        const float d = dsc[b];
#pragma unroll
        for (int a = 0; a < TN; ++a) {
          asm volatile("" : "+a"(acc[a][b]));    // the tile stays in its AGPRs until this point
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            float fv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) fv[r] = ((float)acc[a][b][4 * g + r] * d) * alpha;
            uint2 p;
            p.x = gp_pack_bf16(fv[0], fv[1]);
            p.y = gp_pack_bf16(fv[2], fv[3]);
            *reinterpret_cast<uint2*>(tbuf + l32 * TB_ROW + (a * 32 + 8 * g + 4 * lh) * 2) = p;
          }
          // keep the scheduler from reading many accumulators ahead of their use: the next
          // tile's fragments and staging registers are live here, and a spill in this section
          // would wait on the stores in flight
          __builtin_amdgcn_sched_barrier(0);
        }
        // row b * 32 + i * ROWS_PER_PASS + rr of the wave tile per pass i
        constexpr int NPASS = 32 / ROWS_PER_PASS;
        if (interior) {                                    // uniform: all reads in flight, then all stores
          v4i v[NPASS];
#pragma unroll
          for (int i = 0; i < NPASS; ++i)
            v[i] = *reinterpret_cast<const v4i*>(tbuf + (rr + i * ROWS_PER_PASS) * TB_ROW + cc * 16);
          __builtin_amdgcn_sched_barrier(0);               // (keeps the reads from being paired off with the stores)
#pragma unroll
          for (int i = 0; i < NPASS; ++i)
            *reinterpret_cast<v4i*>(ywave + (size_t)(b * 32 + i * ROWS_PER_PASS) * N + lane_off) = v[i];
        } else {
#pragma unroll
          for (int i = 0; i < NPASS; ++i) {
            const int row = b * 32 + i * ROWS_PER_PASS;
            const uint4 v = *reinterpret_cast<const uint4*>(tbuf + (rr + i * ROWS_PER_PASS) * TB_ROW + cc * 16);
            if (row < m_left && 0 < n_left) *reinterpret_cast<uint4*>(ywave + (size_t)row * N + lane_off) = v;
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
          for (int g = 0; g < 4; ++g) {
            const int n = n0 + wn * WN + a * 32 + 8 * g + 4 * lh;
            const size_t o = (size_t)m * N + n;
            float fv[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) fv[r] = ((float)acc[a][b][4 * g + r] * d) * alpha;
            if (OUT == 1) {
              if (m < M && n < N) {
                if (y_bf16) {
                  uint2 p;
                  p.x = gp_pack_bf16(fv[0], fv[1]);
                  p.y = gp_pack_bf16(fv[2], fv[3]);
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
          for (int g = 0; g < 4; ++g) {
            const int n = n0 + wn * WN + a * 32 + 8 * g + 4 * lh;
            const size_t o = (size_t)m * N + n;
            if (OUT != 2) {
              if (m < M && n < N)
                *reinterpret_cast<int4*>(acc_out + o) =
                    make_int4(acc[a][b][4 * g] >> SHIFT, acc[a][b][4 * g + 1] >> SHIFT,
                              acc[a][b][4 * g + 2] >> SHIFT, acc[a][b][4 * g + 3] >> SHIFT);
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r)
                if (m < M && n + r < N) acc_out[o + r] = acc[a][b][4 * g + r] >> SHIFT;
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
    if (!has_next) break;
    tile = next;
    bl_tile_origin(tile, n_tiles, MT, NTB, BM, BN, m0, n0);
    if (OUT == 0) __syncthreads();     // transpose buffers are read out before stage 1 is refilled
  }
#undef GP_PIN_IN
#undef GP_PIN_OUT
#undef GP_MFMA
}

template <int BM, int BN, bool A4, int OUT, bool ACC>
static int gp_go(const void* q, const float* scale, int M, int Kp, const void* Wp, const float* alpha, int N,
                 void* Y, int y_bf16, int32_t* acc_out, int MT, int NTB, hipStream_t s) {
  constexpr int smem = GpSmem<BM, BN>::total;
  BL_SET_MAX_LDS_ONCE((gemm_prefill_kernel<BM, BN, A4, OUT, ACC>), smem);
  // persistent blocks: one per CU for the large tile (128 KB of LDS, 512 registers per lane)
  const int per_cu = (BM == 256) ? 1 : 2;
  const int grid = min(MT * NTB, bl_num_cus() * per_cu);
  gemm_prefill_kernel<BM, BN, A4, OUT, ACC><<<(unsigned)grid, GP_THREADS, smem, s>>>(
      (const unsigned char*)q, scale, M, Kp, (const unsigned char*)Wp, alpha, N, Y, y_bf16, acc_out, MT, NTB);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

template <int BM, int BN, bool A4>
static int gp_launch(const void* q, const float* scale, int M, int Kp, const void* Wp,
                     const float* alpha, int N, void* Y, bl_dtype ydt, int32_t* acc_out,
                     hipStream_t s) {
  const int MT = (M + BM - 1) / BM, NTB = (N + BN - 1) / BN;
  const int out = (ydt == BL_BF16 && (N & 7) == 0) ? 0 : ((N & 3) == 0 ? 1 : 2);
  const int yb = ydt == BL_BF16 ? 1 : 0;
#define GP_CALL(OUT, ACC) gp_go<BM, BN, A4, OUT, ACC>(q, scale, M, Kp, Wp, alpha, N, Y, yb, acc_out, MT, NTB, s)
  if (acc_out) return out == 0 ? GP_CALL(0, true) : out == 1 ? GP_CALL(1, true) : GP_CALL(2, true);
  return out == 0 ? GP_CALL(0, false) : out == 1 ? GP_CALL(1, false) : GP_CALL(2, false);
#undef GP_CALL
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
