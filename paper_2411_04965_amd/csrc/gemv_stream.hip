// Decode-shaped linears for up to 16 tokens as ONE persistent launch per call.
//
// At these sizes a launch costs as much as streaming the weights (an empty kernel takes 1.6 us
// between two others, 12 MB of weights at full HBM rate 1.6 us), so the design goal is: one launch,
// every weight byte requested in the launch's first microsecond, nothing done twice per compute unit.
//   * One workgroup of 8 waves per compute unit.  It owns a contiguous range of output tiles (16
//     outputs each, BL_W_GEMM layout: 1 KB per tile and 256 input channels) of one weight matrix or
//     of two that share the input (gate and up projection of an FFN).
//   * The tokens' int8 codes sit in LDS, one padded row per token.  They come from the stand-alone
//     quantizer (any mode; INT4 nibbles are expanded while they are copied), or the workgroup makes
//     them itself from up to 8 bfloat16 rows with eq. 7's arithmetic (float64 sum of |x|, one
//     rounding, one float32 multiply per element: bit for bit the stand-alone quantizer's codes) --
//     once per workgroup, while its weight loads are in flight.
//   * The 1 KB weight tiles of the workgroup's outputs are dealt round-robin to the waves; a wave
//     issues up to 12 tile loads at once (12 KB in flight per wave, all of its share at 7B
//     shapes), expands the 2-bit fields to int8 in registers and feeds v_mfma_i32_16x16x64_i8 with
//     the weight tile as the row operand.  Partial tiles go to LDS (one slot per output tile and
//     wave), are added after one barrier, rescaled and stored.
//   * With two matrices the outputs are stored separately, or combined as eq. 5's
//     H = bf16(U * max(G, 0)^2) in the same epilogue (the workgroup then owns the same output
//     range of both).
// Integer sums are exact, so the split of K over waves changes nothing: accumulators and outputs
// equal those of the quantizer followed by any other exact kernel.
#include "common.h"
#include "topk_regs.h"

#define GV_THREADS 512
#define GV_WAVES 8
#define GV_NE 8                // output tiles (entries) per workgroup at most
#define GV_UNR 12              // weight tiles in flight per wave and round
#define GV_LDS_MAX (158 * 1024)
#define GV_NCP 20              // 16-byte pieces of packed codes per thread at most: 160 KB / 16 / 512

struct GvMat {
  const unsigned char* W;      // BL_W_GEMM tiles
  const float* alpha;
  void* Y;                     // [M, N] outputs (nullable in the GLU form)
  int32_t* acc;                // nullable
  int N, NT;                   // outputs, tiles of 16
};

__device__ __forceinline__ void gv_store4(void* Y, int y_bf16, int32_t* acc_out, size_t o, int n, int N,
                                          const int (&iv)[4], const float (&fv)[4]) {
  if ((N & 3) == 0) {
    if (Y) {
      if (y_bf16) {
        uint2 p;
        p.x = (u32)bl_f32_to_bf16_rne(fv[0]) | ((u32)bl_f32_to_bf16_rne(fv[1]) << 16);
        p.y = (u32)bl_f32_to_bf16_rne(fv[2]) | ((u32)bl_f32_to_bf16_rne(fv[3]) << 16);
        *reinterpret_cast<uint2*>((uint16_t*)Y + o) = p;
      } else {
        *reinterpret_cast<float4*>((float*)Y + o) = make_float4(fv[0], fv[1], fv[2], fv[3]);
      }
    }
    if (acc_out) *reinterpret_cast<int4*>(acc_out + o) = make_int4(iv[0], iv[1], iv[2], iv[3]);
  } else {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      if (n + r < N) {
        if (Y) {
          if (y_bf16) ((uint16_t*)Y)[o + r] = bl_f32_to_bf16_rne(fv[r]);
          else ((float*)Y)[o + r] = fv[r];
        }
        if (acc_out) acc_out[o + r] = iv[r];
      }
    }
  }
}

// eq. 7 for up to QM bfloat16 token rows by the whole workgroup (QM <= 8 = waves): int8 codes to
// codes[m * pitch + k] (zero from K to Kp), beta / sqrt(7) to dq[m].  A thread holds pieces tid and
// tid + 512 (8 channels each) of every token (K % 8 == 0, Kp <= 8192); the kernel loads them before
// it requests any weights (memory returns loads in order, and the tokens must not wait behind the
// weight stream).  Three steps with a barrier between them: every thread sums |x| of its pieces in
// float64 (exact) into part[m][tid]; wave m adds token m's 512 partial sums and derives the scale
// once (the float64 divide and the two float32 divides are not repeated by every wave); every
// thread codes its pieces.  RoundClip as round(clamp(v)): the bounds are integers, so this equals
// clamp(round(v)); the rounding is the float32 addition of 1.5 * 2^23 (round to nearest even at
// integer spacing), the code its low byte.  The caller adds the barrier that publishes codes and dq.
#define GV_NV 2
template <int QM>
__device__ __forceinline__ void gv_quantize_rows(const uint4 (&xr)[QM][GV_NV], int M, int K, int Kp, float eps,
                                                 unsigned char* codes, int pitch, float* dq, float* sq,
                                                 double* part) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool two = K > 8 * GV_THREADS;           // (uniform) rows wider than 4096 use the second piece
  const float sqrt7 = 2.6457512f;                // float32(sqrt(7))
  if (QM == 1) {
    // one token: a barrier less.  Wave sums with DPP, and every wave adds the 8 of them and derives
    // the scale itself (the same operations on the same numbers in every wave).
    double a = 0.0;
#pragma unroll
    for (int j = 0; j < GV_NV; ++j) {
      if (j == 0 || two) {
        const u32 w4[4] = {xr[0][j].x, xr[0][j].y, xr[0][j].z, xr[0][j].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a += (double)fabsf(__uint_as_float(w4[e] << 16));
          a += (double)fabsf(__uint_as_float(w4[e] & 0xFFFF0000u));
        }
      }
    }
    a = bl_wave_sum_f64_dpp(a);
    if (lane == 0) part[wave] = a;
    __syncthreads();
    double tot = 0.0;
#pragma unroll
    for (int w = 0; w < GV_WAVES; ++w) tot += part[w];
    const float beta = (float)(tot / (double)K);
    if (tid == 0) dq[0] = beta / sqrt7;
    const float s = sqrt7 / (beta + eps);
#pragma unroll
    for (int j = 0; j < GV_NV; ++j) {
      const int pc = tid + GV_THREADS * j;
      if (pc < (Kp >> 3)) {
        const u32 w4[4] = {xr[0][j].x, xr[0][j].y, xr[0][j].z, xr[0][j].w};
        u32 rb[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float v0 = __uint_as_float(w4[e] << 16) * s;
          const float v1 = __uint_as_float(w4[e] & 0xFFFF0000u) * s;
          rb[2 * e] = __float_as_uint(__builtin_amdgcn_fmed3f(v0, -8.0f, 7.0f) + 12582912.0f);
          rb[2 * e + 1] = __float_as_uint(__builtin_amdgcn_fmed3f(v1, -8.0f, 7.0f) + 12582912.0f);
        }
        const u32 lo = __builtin_amdgcn_perm(rb[1], rb[0], 0x0c0c0400u) | __builtin_amdgcn_perm(rb[3], rb[2], 0x04000c0cu);
        const u32 hi = __builtin_amdgcn_perm(rb[5], rb[4], 0x0c0c0400u) | __builtin_amdgcn_perm(rb[7], rb[6], 0x04000c0cu);
        *reinterpret_cast<uint2*>(codes + pc * 8) = make_uint2(lo, hi);
      }
    }
    return;
  }
#pragma unroll
  for (int m = 0; m < QM; ++m) {
    if (m < M) {                                 // block-uniform
      double a = 0.0;
#pragma unroll
      for (int j = 0; j < GV_NV; ++j) {
        if (j == 0 || two) {
          const u32 w4[4] = {xr[m][j].x, xr[m][j].y, xr[m][j].z, xr[m][j].w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            a += (double)fabsf(__uint_as_float(w4[e] << 16));
            a += (double)fabsf(__uint_as_float(w4[e] & 0xFFFF0000u));
          }
        }
      }
      part[m * GV_THREADS + tid] = a;
    }
  }
  __syncthreads();
  if (wave < M) {
    double a = 0.0;
#pragma unroll
    for (int j = 0; j < GV_THREADS / 64; ++j) a += part[wave * GV_THREADS + lane + 64 * j];
    a = bl_wave_sum_f64_dpp(a);
    const float beta = (float)(a / (double)K);
    if (lane == 0) {
      sq[wave] = sqrt7 / (beta + eps);
      dq[wave] = beta / sqrt7;
    }
  }
  __syncthreads();
#pragma unroll
  for (int m = 0; m < QM; ++m) {
    if (m < M) {
      const float s = sq[m];
#pragma unroll
      for (int j = 0; j < GV_NV; ++j) {
        const int pc = tid + GV_THREADS * j;
        if (pc < (Kp >> 3)) {                    // (second piece: only rows padded beyond 4096 channels)
          const u32 w4[4] = {xr[m][j].x, xr[m][j].y, xr[m][j].z, xr[m][j].w};
          u32 rb[8];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float v0 = __uint_as_float(w4[e] << 16) * s;
            const float v1 = __uint_as_float(w4[e] & 0xFFFF0000u) * s;
            rb[2 * e] = __float_as_uint(__builtin_amdgcn_fmed3f(v0, -8.0f, 7.0f) + 12582912.0f);
            rb[2 * e + 1] = __float_as_uint(__builtin_amdgcn_fmed3f(v1, -8.0f, 7.0f) + 12582912.0f);
          }
          // low bytes of rb[0..3] and of rb[4..7] as two words
          const u32 lo = __builtin_amdgcn_perm(rb[1], rb[0], 0x0c0c0400u) | __builtin_amdgcn_perm(rb[3], rb[2], 0x04000c0cu);
          const u32 hi = __builtin_amdgcn_perm(rb[5], rb[4], 0x0c0c0400u) | __builtin_amdgcn_perm(rb[7], rb[6], 0x04000c0cu);
          *reinterpret_cast<uint2*>(codes + (size_t)m * pitch + pc * 8) = make_uint2(lo, hi);
        }
      }
    }
  }
}

// Word t4 of a lane's 16 bytes of a weight tile as the A operand of one MFMA step: the four 2-bit codes
// of each byte become four int8 values 64 T (code 00 -> 0, 01 -> 64, 11 -> -64).
__device__ __forceinline__ v4i gv_unpack(const uint4& wc, int t4) {
  const u32 w = t4 == 0 ? wc.x : t4 == 1 ? wc.y : t4 == 2 ? wc.z : wc.w;
  return (v4i){(int)((w << 6) & 0xC0C0C0C0u), (int)((w << 4) & 0xC0C0C0C0u), (int)((w << 2) & 0xC0C0C0C0u),
               (int)(w & 0xC0C0C0C0u)};
}

// A4: the activations are INT4 levels (codes from memory: nibbles, kept in LDS as 16 q; made here: q).
// QM = 0: codes and scales come from the stand-alone quantizer; QM > 0: `src` is the bfloat16 input
// and eq. 7 runs here for up to QM tokens.  GLU: the two matrices are gate and up, the workgroup owns
// the same outputs of both and stores H (eq. 5); their own outputs are stored too where Y is given.
// TK > 0: `src` is ONE bfloat16 token and eq. 1 + eq. 3 run here (Top_k of `topk` channels, INT8 absmax;
// TK = 4 or 8 chunks of 256 channels per wave; A4 = false, QM = 0).
// UNR: weight tiles a wave requests per round (all of its share at the shapes the launcher picks it for).
// Work: `upb` units (output tiles; GLU: gate/up tile pairs) per workgroup, one more for the first
// `urem` workgroups.  A workgroup's tiles form at most two contiguous runs in memory (one per
// matrix); its entries (output tiles) are numbered run 0 first.
// JT > 0: the rows have exactly 8 JT tiles of 256 channels and a wave's whole share is one round, so
// that tile u of a wave is K tile wave + 8 (u mod JT) of entry u / JT: entry changes, LDS addresses and
// the stores of the parts are fixed when the kernel is compiled.  JT = 0: any row length, any share.
template <bool A4, int QM, bool GLU, int UNR, int TK, int JT>
__global__ __launch_bounds__(GV_THREADS) void gemv_stream_kernel(
    const void* __restrict__ src, const float* __restrict__ scale, int M, int K, int Kp, float eps,
    GvMat m0, GvMat m1, uint16_t* __restrict__ H, int y_bf16, int upb, int urem, int topk) {
  extern __shared__ __align__(16) unsigned char gv_smem[];
  __shared__ float sh_dq[16], sh_sq[16];
  __shared__ __align__(16) u32 sh_tk[TK > 0 ? 80 : 4];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // every argument is fetched now, in one round trip to the argument segment (left alone the compiler
  // fetches each where it is first used, and each fetch then stalls the requests below)
  asm volatile("" ::"s"(src), "s"(scale), "s"(M), "s"(K), "s"(Kp), "s"(eps), "s"(m0.W), "s"(m0.alpha), "s"(m0.Y),
               "s"(m0.acc), "s"(m0.N), "s"(m0.NT), "s"(m1.W), "s"(m1.alpha), "s"(m1.Y), "s"(m1.acc), "s"(m1.N),
               "s"(m1.NT), "s"(H), "s"(y_bf16), "s"(upb), "s"(urem), "s"(topk));
  const int KT = Kp >> 8;

  // ---- requests first.  Tokens (or their codes), then the first batch of weight tiles: loads come back in the
  // order they were issued, so the short token rows arrive at once and the quantizer (or the copy into
  // LDS) runs while the weights stream in.  Every weight load is unconditional (indices past the
  // workgroup's last tile re-read that tile, a cache hit) so that the compiler can count the loads in
  // flight and wait for each one alone.
  constexpr int QMR = QM > 0 ? QM : 1;
  uint4 xr[QMR][GV_NV];
  constexpr int NCP = (QM > 0 || TK > 0) ? 1 : GV_NCP;                 // code pieces (16 bytes) per thread
  uint4 cr[NCP];
  const int code_ppr = A4 ? (Kp >> 5) : (Kp >> 4);                     // pieces per token row
  const int n_code_pieces = M * code_ppr;
  // (TK) this wave's chunks of 256 channels of the token: 4 consecutive channels per lane and chunk
  constexpr int TKR = TK > 0 ? TK : 4;
  u32 traw[TKR][2];
  const int tk_per_wave = ((Kp >> 8) + GV_WAVES - 1) / GV_WAVES;
  const int tk_begin = min(wave * tk_per_wave, Kp >> 8);
  const int tk_nc = min(tk_begin + tk_per_wave, Kp >> 8) - tk_begin;
  if (TK > 0) {
    const int ch0 = tk_begin * 256 + lane * 4;
#pragma unroll
    for (int i = 0; i < TKR; ++i) {
      uint2 v = make_uint2(0u, 0u);
      if (i < tk_nc && ch0 + i * 256 < K) v = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(src) + ch0 + i * 256);
      traw[i][0] = v.x;
      traw[i][1] = v.y;
    }
  } else if (QM > 0) {
    const int nv = K >> 3;
#pragma unroll
    for (int m = 0; m < QMR; ++m)
#pragma unroll
      for (int j = 0; j < GV_NV; ++j) {
        const int pc = tid + GV_THREADS * j;
        xr[m][j] = make_uint4(0u, 0u, 0u, 0u);
        if (m < M && pc < nv) xr[m][j] = reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(src) + (size_t)m * K)[pc];
      }
  } else {
#pragma unroll
    for (int j = 0; j < NCP; ++j) {
      const int pc = tid + GV_THREADS * j;
      cr[j] = make_uint4(0u, 0u, 0u, 0u);
      if (pc < n_code_pieces) cr[j] = reinterpret_cast<const uint4*>(src)[pc];
    }
  }

  const int bid = blockIdx.x;
  const int u_begin = bid * upb + min(bid, urem);
  const int n_u = upb + (bid < urem ? 1 : 0);
  // run 0: n0 entries of matrix 0 from tile nt0; run 1: n1 entries of matrix 1 from tile nt1
  const int n0 = GLU ? n_u : max(0, min(n_u, m0.NT - u_begin));
  const int n1 = GLU ? n_u : n_u - n0;
  const int nt0 = u_begin, nt1 = GLU ? u_begin : max(0, u_begin - m0.NT);
  const int NE = n0 + n1;                                              // <= GV_NE by the launch
  const int T = NE * KT, T0 = n0 * KT;                                 // 1 KB tiles: all, and of run 0
  const unsigned char* base0 = m0.W + (size_t)nt0 * KT * 1024;
  const unsigned char* base1 = m1.W + ((size_t)nt1 * KT - T0) * 1024;  // (so that flat index i sits at base1 + 1024 i)
  const u32 lane_off = lane * 16;
  uint4 wr[UNR];
  auto issue_round = [&](int i0) {
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int ic = min(i0 + GV_WAVES * u, T - 1);                    // wave-uniform
      const unsigned char* tp = (ic < T0 ? base0 : base1) + (size_t)ic * 1024;
      wr[u] = *reinterpret_cast<const uint4*>(tp + lane_off);
    }
  };
  issue_round(wave);

  const int li = lane & 15, lg = lane >> 4;
  const int pitch = Kp + 16;
  unsigned char* codes = gv_smem;                                      // [M][pitch]
  v4i* red = reinterpret_cast<v4i*>(gv_smem + (size_t)M * pitch);      // [NE][GV_WAVES][64]
  // (with fewer than 8 K tiles a wave may have no tile of some entry: its slot must read as zero)
  if (KT < GV_WAVES)
    for (int i = tid; i < NE * GV_WAVES * 64; i += GV_THREADS) red[i] = (v4i){0, 0, 0, 0};

  // ---- the tokens' codes
  if constexpr (TK > 0) {
    qa_topk_row_regs8<TKR>(traw, tk_nc, tk_begin, topk, eps, reinterpret_cast<u32*>(codes), sh_dq, sh_tk);
  } else if (QM > 0) {
    const int ne_max = (upb + (urem > 0 ? 1 : 0)) * (GLU ? 2 : 1);    // the launch's LDS holds this many entries
    double* part = reinterpret_cast<double*>(gv_smem + (size_t)M * pitch + (size_t)ne_max * GV_WAVES * 1024);
    gv_quantize_rows<QMR>(xr, M, K, Kp, eps, codes, pitch, sh_dq, sh_sq, part);
  } else if (A4) {
    // nibble rows [M][Kp / 2] -> 16 q as int8: a 16-byte piece (32 channels) becomes 32 bytes
#pragma unroll
    for (int j = 0; j < NCP; ++j) {
      const int pc = tid + GV_THREADS * j;
      if (pc < n_code_pieces) {
        const int m = pc / code_ppr, c = pc - m * code_ppr;
        const u32 w4[4] = {cr[j].x, cr[j].y, cr[j].z, cr[j].w};
        u32 o[8];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o[2 * e] = (w4[e] << 4) & 0xF0F0F0F0u;
          o[2 * e + 1] = w4[e] & 0xF0F0F0F0u;
        }
        uint4* dst = reinterpret_cast<uint4*>(codes + (size_t)m * pitch + c * 32);
        dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
        dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < NCP; ++j) {
      const int pc = tid + GV_THREADS * j;
      if (pc < n_code_pieces) {
        const int m = pc / code_ppr, c = pc - m * code_ppr;
        *reinterpret_cast<uint4*>(codes + (size_t)m * pitch + c * 16) = cr[j];
      }
    }
  }
  // (compile-time schedule) the first tiles are expanded to int8 before the barrier: a wave that waits
  // there for the other waves' codes would otherwise do this work after it, on the critical path
  constexpr int NPRE = JT > 0 ? (UNR < 6 ? UNR : 6) : 1;
  v4i wpre[NPRE][4];
  if constexpr (JT > 0) {
#pragma unroll
    for (int u = 0; u < NPRE; ++u)
      if (u / JT < NE) {                                               // wave-uniform
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
          wpre[u][t4] = gv_unpack(wr[u], t4);
          asm volatile("" : "+v"(wpre[u][t4]));
        }
      }
  }
  __syncthreads();

  // ---- the products.  Lane (li, lg) holds token li, and of a tile's 256 channels the 64 of group
  // lg, 16 per MFMA step; two accumulators take the steps in turn (no MFMA waits for the one before).
  const unsigned char* xrow = codes + (size_t)min(li, M - 1) * pitch + lg * 64;
  v4i acc0 = (v4i){0, 0, 0, 0}, acc1 = (v4i){0, 0, 0, 0};
  int cur_e = -1;
  int e_c = 0, kt_c = wave;                                            // (entry, K tile) of flat index wave + 8 j
  while (kt_c >= KT) { kt_c -= KT; ++e_c; }
  auto flush = [&]() {
    if (cur_e >= 0) red[(cur_e * GV_WAVES + wave) * 64 + lane] = acc0 + acc1;
  };
  // the token fragments of a tile are read from LDS one tile ahead, so that their latency hides
  // behind the wait for the weights
  auto read_x = [&](int kt, v4i (&x)[4]) {
#pragma unroll
    for (int t4 = 0; t4 < 4; ++t4) x[t4] = *reinterpret_cast<const v4i*>(xrow + kt * 256 + t4 * 16);
  };
  if constexpr (JT > 0) {
    // a wave meets only JT different K tiles: their token fragments stay in registers
    v4i xs[JT][4];
#pragma unroll
    for (int j = 0; j < JT; ++j) read_x(wave + GV_WAVES * j, xs[j]);
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int e = u / JT, j = u % JT;                                // (compile-time after unrolling)
      if (e < NE) {                                                    // wave-uniform
        if (j == 0) {
          acc0 = (v4i){0, 0, 0, 0};
          acc1 = (v4i){0, 0, 0, 0};
        }
#pragma unroll
        for (int t4 = 0; t4 < 4; ++t4) {
          v4i wo;
          if (u < NPRE) wo = wpre[u < NPRE ? u : 0][t4];
          else wo = gv_unpack(wr[u], t4);
          if (t4 & 1) acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(wo, xs[j][t4], acc1, 0, 0, 0);
          else acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(wo, xs[j][t4], acc0, 0, 0, 0);
        }
        if (j == JT - 1) red[(e * GV_WAVES + wave) * 64 + lane] = acc0 + acc1;
      }
    }
  } else {
    v4i xn[4];
    read_x(min(kt_c, KT - 1), xn);                                       // (lanes of token columns past M read token M - 1
                                                                         //  again: their output columns are never stored)
    for (int i0 = wave; i0 < T; i0 += GV_WAVES * UNR) {
      if (i0 != wave) issue_round(i0);                                   // (later rounds: more tiles than 8 UNR per workgroup)
  #pragma unroll
      for (int u = 0; u < UNR; ++u) {
        if (i0 + GV_WAVES * u < T) {                                     // wave-uniform
          if (e_c != cur_e) {
            flush();
            cur_e = e_c;
            acc0 = (v4i){0, 0, 0, 0};
            acc1 = (v4i){0, 0, 0, 0};
          }
          v4i xo[4];
  #pragma unroll
          for (int t4 = 0; t4 < 4; ++t4) xo[t4] = xn[t4];
          kt_c += GV_WAVES;
          while (kt_c >= KT) { kt_c -= KT; ++e_c; }
          read_x(kt_c, xn);                                              // (past the last tile: a row inside the codes' space)
          const uint4 wc = wr[u];
  #pragma unroll
          for (int t4 = 0; t4 < 4; ++t4) {
            const u32 w = t4 == 0 ? wc.x : t4 == 1 ? wc.y : t4 == 2 ? wc.z : wc.w;
            const v4i wo = (v4i){(int)((w << 6) & 0xC0C0C0C0u), (int)((w << 4) & 0xC0C0C0C0u),
                                 (int)((w << 2) & 0xC0C0C0C0u), (int)(w & 0xC0C0C0C0u)};
            if (t4 & 1) acc1 = __builtin_amdgcn_mfma_i32_16x16x64_i8(wo, xo[t4], acc1, 0, 0, 0);
            else acc0 = __builtin_amdgcn_mfma_i32_16x16x64_i8(wo, xo[t4], acc0, 0, 0, 0);
          }
        }
      }
    }
    flush();
  }
  __syncthreads();

  // ---- add the waves' parts, rescale, store: wave w finishes entry w (GLU: the pair w, n0 + w)
  constexpr int SHIFT = (A4 && QM == 0) ? 10 : 6;                      // weights carry 64 T, nibble codes 16 q
  const int m = li;
  if (m >= M) return;
  const float d = (QM > 0 || TK > 0) ? sh_dq[m] : scale[m];
  auto entry_sum = [&](int e, int (&iv)[4]) {
    v4i sum = (v4i){0, 0, 0, 0};
#pragma unroll
    for (int w = 0; w < GV_WAVES; ++w) sum += red[(e * GV_WAVES + w) * 64 + lane];
#pragma unroll
    for (int r = 0; r < 4; ++r) iv[r] = sum[r] >> SHIFT;
  };
  if (!GLU) {
    if (wave >= NE) return;
    const bool second = wave >= n0;
    const GvMat& mm = second ? m1 : m0;
    const int nt = second ? nt1 + wave - n0 : nt0 + wave;
    const int n = nt * 16 + 4 * lg;
    if (n >= mm.N) return;
    int iv[4];
    entry_sum(wave, iv);
    const float alpha = mm.alpha[0];
    float fv[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) fv[r] = ((float)iv[r] * d) * alpha;
    gv_store4(mm.Y, y_bf16, mm.acc, (size_t)m * mm.N + n, n, mm.N, iv, fv);
  } else {
    if (wave >= n0) return;
    const int nt = nt0 + wave;
    const int n = nt * 16 + 4 * lg, N = m0.N;
    if (n >= N) return;
    int ig[4], iu[4];
    entry_sum(wave, ig);
    entry_sum(n0 + wave, iu);
    const float ag = m0.alpha[0], au = m1.alpha[0];
    float g[4], uu[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      g[r] = ((float)ig[r] * d) * ag;
      uu[r] = ((float)iu[r] * d) * au;
    }
    const size_t o = (size_t)m * N + n;
    if (m0.Y || m0.acc) gv_store4(m0.Y, y_bf16, m0.acc, o, n, N, ig, g);
    if (m1.Y || m1.acc) gv_store4(m1.Y, y_bf16, m1.acc, o, n, N, iu, uu);
    if (H) {
      uint16_t h[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float rl = fmaxf(g[r], 0.0f);
        const float rr = rl * rl;
        h[r] = bl_f32_to_bf16_rne(uu[r] * rr);
      }
      if ((N & 3) == 0) {
        *reinterpret_cast<uint2*>(H + o) = make_uint2((u32)h[0] | ((u32)h[1] << 16), (u32)h[2] | ((u32)h[3] << 16));
      } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (n + r < N) H[o + r] = h[r];
      }
    }
  }
}

// ---------------------------------------------------------------- host side
// Workgroups and LDS for `units` output units (tiles, or gate/up tile pairs) of `epu` entries each.
static bool gv_plan(int64_t M, int64_t Kp, int64_t units, int epu, bool quant_inside, int& grid, size_t& smem) {
  if (M < 1 || M > 16 || units < 1) return false;
  const int upb_max = GV_NE / epu;                                     // units per workgroup at most
  int64_t g = bl_num_cus();
  if (g > units) g = units;
  if ((units + g - 1) / g > upb_max) g = (units + upb_max - 1) / upb_max;
  const int64_t ne = ((units + g - 1) / g) * epu;
  // codes, the partial tiles of the entries, and (quantizer inside) the float64 partial sums
  smem = (size_t)M * (size_t)(Kp + 16) + (size_t)ne * GV_WAVES * 1024 + (quant_inside ? (size_t)M * GV_THREADS * 8 : 0);
  grid = (int)g;
  return smem <= GV_LDS_MAX && bl_grid_ok(g);
}

bool bl_gemv_stream_ok(int64_t M, int64_t N, int64_t K, bool quant_inside) {
  int grid;
  size_t smem;
  const int64_t Kp = bl_round_up(K, BL_KPAD);
  if (quant_inside && (M > 8 || K % 8 != 0 || Kp > 8192)) return false;
  return gv_plan(M, Kp, (N + 15) / 16, 1, quant_inside, grid, smem);
}

bool bl_gemv_stream_pair_ok(int64_t M, int64_t N, int64_t K, bool glu) {
  int grid;
  size_t smem;
  const int64_t Kp = bl_round_up(K, BL_KPAD);
  if (M > 8 || K % 8 != 0 || Kp > 8192) return false;
  return glu ? gv_plan(M, Kp, (N + 15) / 16, 2, true, grid, smem) : gv_plan(M, Kp, 2 * ((N + 15) / 16), 1, true, grid, smem);
}

template <bool A4, int QM, bool GLU, int UNR, int TK = 0, int JT = 0>
static int gv_go2(const void* src, const float* scale, int M, int K, int Kp, float eps, const GvMat& m0,
                  const GvMat& m1, uint16_t* H, int ybf, int grid, size_t smem, hipStream_t s, int topk = 0) {
  BL_SET_MAX_LDS_ONCE((gemv_stream_kernel<A4, QM, GLU, UNR, TK, JT>), GV_LDS_MAX);
  const int64_t units = GLU ? m0.NT : (int64_t)m0.NT + m1.NT;
  gemv_stream_kernel<A4, QM, GLU, UNR, TK, JT><<<(unsigned)grid, GV_THREADS, smem, s>>>(
      src, scale, M, K, Kp, eps, m0, m1, H, ybf, (int)(units / grid), (int)(units % grid), topk);
  BL_HIP_CHECK_LAUNCH();
  return BL_OK;
}

// The loads a wave keeps in flight: all tiles of its share where that is at most 12 (the 7B shapes
// need 2, 6 and 12; 2 runs as 6), else rounds of 12.
template <bool A4, int QM, bool GLU>
static int gv_go(const void* src, const float* scale, int M, int K, int Kp, float eps, const GvMat& m0,
                 const GvMat& m1, uint16_t* H, int ybf, int grid, size_t smem, hipStream_t s) {
  const int64_t units = GLU ? m0.NT : (int64_t)m0.NT + m1.NT;
  const int64_t ne = ((units + grid - 1) / grid) * (GLU ? 2 : 1);
  const int64_t per_wave = (ne * (Kp >> 8) + GV_WAVES - 1) / GV_WAVES;
  if ((Kp >> 8) == 16 && per_wave <= GV_UNR) {                         // 4096 channels: the compile-time schedule
    if (per_wave <= 6) return gv_go2<A4, QM, GLU, 6, 0, 2>(src, scale, M, K, Kp, eps, m0, m1, H, ybf, grid, smem, s);
    return gv_go2<A4, QM, GLU, GV_UNR, 0, 2>(src, scale, M, K, Kp, eps, m0, m1, H, ybf, grid, smem, s);
  }
  if (per_wave <= 6) return gv_go2<A4, QM, GLU, 6>(src, scale, M, K, Kp, eps, m0, m1, H, ybf, grid, smem, s);
  return gv_go2<A4, QM, GLU, GV_UNR>(src, scale, M, K, Kp, eps, m0, m1, H, ybf, grid, smem, s);
}

// Codes from the stand-alone quantizer (INT4 nibbles or INT8), one matrix.
int bl_launch_gemv_stream(const void* q, const float* scale, bool a4, int64_t M, int64_t K, const void* Wp,
                          const float* alpha, int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out, hipStream_t s) {
  const int Kp = (int)bl_round_up(K, BL_KPAD);
  int grid;
  size_t smem;
  if (!gv_plan(M, Kp, (N + 15) / 16, 1, false, grid, smem)) return BL_EUNSUPPORTED;
  const GvMat m0 = {(const unsigned char*)Wp, alpha, Y, acc_out, (int)N, (int)((N + 15) / 16)};
  const GvMat m1 = {nullptr, nullptr, nullptr, nullptr, 0, 0};
  const int ybf = ydt == BL_BF16 ? 1 : 0;
  if (a4) return gv_go<true, 0, false>(q, scale, (int)M, (int)K, Kp, 0.0f, m0, m1, nullptr, ybf, grid, smem, s);
  return gv_go<false, 0, false>(q, scale, (int)M, (int)K, Kp, 0.0f, m0, m1, nullptr, ybf, grid, smem, s);
}

template <bool GLU>
static int gv_quant_dispatch(const void* X, int M, int K, int Kp, float eps, const GvMat& m0, const GvMat& m1,
                             uint16_t* H, int ybf, int grid, size_t smem, hipStream_t s) {
  if (M <= 1) return gv_go<true, 1, GLU>(X, nullptr, M, K, Kp, eps, m0, m1, H, ybf, grid, smem, s);
  if (M <= 2) return gv_go<true, 2, GLU>(X, nullptr, M, K, Kp, eps, m0, m1, H, ybf, grid, smem, s);
  if (M <= 4) return gv_go<true, 4, GLU>(X, nullptr, M, K, Kp, eps, m0, m1, H, ybf, grid, smem, s);
  return gv_go<true, 8, GLU>(X, nullptr, M, K, Kp, eps, m0, m1, H, ybf, grid, smem, s);
}

// bfloat16 tokens, eq. 7 inside, one matrix.
int bl_launch_gemv_stream_a4(const void* X, int64_t M, int64_t K, float eps, const void* Wp, const float* alpha,
                             int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out, hipStream_t s) {
  if (!bl_gemv_stream_ok(M, N, K, true)) return BL_EUNSUPPORTED;
  const int Kp = (int)bl_round_up(K, BL_KPAD);
  int grid;
  size_t smem;
  gv_plan(M, Kp, (N + 15) / 16, 1, true, grid, smem);
  const GvMat m0 = {(const unsigned char*)Wp, alpha, Y, acc_out, (int)N, (int)((N + 15) / 16)};
  const GvMat m1 = {nullptr, nullptr, nullptr, nullptr, 0, 0};
  return gv_quant_dispatch<false>(X, (int)M, (int)K, Kp, eps, m0, m1, nullptr, ydt == BL_BF16 ? 1 : 0, grid, smem, s);
}

// bfloat16 tokens, eq. 7 inside, gate and up matrices of one shape: G and U (either may be null)
// and / or H = bf16(U * max(G, 0)^2).
int bl_launch_gemv_stream_gate_up(const void* X, int64_t M, int64_t K, float eps, const void* Wg, const float* ag,
                                  const void* Wu, const float* au, int64_t N, void* G, void* U, bl_dtype ydt,
                                  void* H, hipStream_t s) {
  const bool glu = H != nullptr;
  if (!bl_gemv_stream_pair_ok(M, N, K, glu)) return BL_EUNSUPPORTED;
  const int Kp = (int)bl_round_up(K, BL_KPAD), NT = (int)((N + 15) / 16);
  int grid;
  size_t smem;
  if (glu) gv_plan(M, Kp, NT, 2, true, grid, smem);
  else gv_plan(M, Kp, 2 * NT, 1, true, grid, smem);
  const GvMat m0 = {(const unsigned char*)Wg, ag, G, nullptr, (int)N, NT};
  const GvMat m1 = {(const unsigned char*)Wu, au, U, nullptr, (int)N, NT};
  const int ybf = ydt == BL_BF16 ? 1 : 0;
  if (glu) return gv_quant_dispatch<true>(X, (int)M, (int)K, Kp, eps, m0, m1, (uint16_t*)H, ybf, grid, smem, s);
  return gv_quant_dispatch<false>(X, (int)M, (int)K, Kp, eps, m0, m1, nullptr, ybf, grid, smem, s);
}

// INT4 codes from the stand-alone quantizer (up to 16 tokens), gate and up matrices, H = bf16(U * max(G, 0)^2) only.
bool bl_gemv_stream_glu_codes_ok(int64_t M, int64_t N, int64_t K) {
  int grid;
  size_t smem;
  return gv_plan(M, bl_round_up(K, BL_KPAD), (N + 15) / 16, 2, false, grid, smem);
}

int bl_launch_gemv_stream_glu_codes(const void* q, const float* scale, int64_t M, int64_t K, const void* Wg,
                                    const float* ag, const void* Wu, const float* au, int64_t N, void* H, hipStream_t s) {
  const int Kp = (int)bl_round_up(K, BL_KPAD), NT = (int)((N + 15) / 16);
  int grid;
  size_t smem;
  if (!gv_plan(M, Kp, NT, 2, false, grid, smem)) return BL_EUNSUPPORTED;
  const GvMat m0 = {(const unsigned char*)Wg, ag, nullptr, nullptr, (int)N, NT};
  const GvMat m1 = {(const unsigned char*)Wu, au, nullptr, nullptr, (int)N, NT};
  return gv_go<true, 0, true>(q, scale, (int)M, (int)K, Kp, 0.0f, m0, m1, (uint16_t*)H, 1, grid, smem, s);
}

// One bfloat16 token, Top_k + INT8 (eq. 1, eq. 3) inside, one matrix.
bool bl_gemv_stream_topk_ok(int64_t M, int64_t N, int64_t K) {
  int grid;
  size_t smem;
  const int64_t Kp = bl_round_up(K, BL_KPAD);
  return M == 1 && K % 4 == 0 && Kp <= 16384 && gv_plan(1, Kp, (N + 15) / 16, 1, false, grid, smem);
}

int bl_launch_gemv_stream_topk(const void* X, int64_t K, int64_t topk, float eps, const void* Wp, const float* alpha,
                               int64_t N, void* Y, bl_dtype ydt, int32_t* acc_out, hipStream_t s) {
  if (!bl_gemv_stream_topk_ok(1, N, K)) return BL_EUNSUPPORTED;
  const int Kp = (int)bl_round_up(K, BL_KPAD);
  int grid;
  size_t smem;
  gv_plan(1, Kp, (N + 15) / 16, 1, false, grid, smem);
  const GvMat m0 = {(const unsigned char*)Wp, alpha, Y, acc_out, (int)N, (int)((N + 15) / 16)};
  const GvMat m1 = {nullptr, nullptr, nullptr, nullptr, 0, 0};
  const int ybf = ydt == BL_BF16 ? 1 : 0;
  const int64_t ne = (m0.NT + grid - 1) / grid;
  const int64_t per_wave = (ne * (Kp >> 8) + GV_WAVES - 1) / GV_WAVES;
  const bool small = (Kp >> 8) <= 4 * GV_WAVES;            // at most 4 chunks of 256 channels per wave
#define GV_TK(UNRV)                                                                                                \
  ((Kp >> 8) == 16 && per_wave <= UNRV                                                                             \
       ? gv_go2<false, 0, false, UNRV, 4, 2>(X, nullptr, 1, (int)K, Kp, eps, m0, m1, nullptr, ybf, grid, smem, s, (int)topk) \
   : small ? gv_go2<false, 0, false, UNRV, 4>(X, nullptr, 1, (int)K, Kp, eps, m0, m1, nullptr, ybf, grid, smem, s, (int)topk) \
           : gv_go2<false, 0, false, UNRV, 8>(X, nullptr, 1, (int)K, Kp, eps, m0, m1, nullptr, ybf, grid, smem, s, (int)topk))
  if (per_wave <= 6) return GV_TK(6);
  return GV_TK(GV_UNR);
#undef GV_TK
}
