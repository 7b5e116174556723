// Top_k + INT8 absmax (eq. 1, eq. 3) with the keys of a token in registers: helpers and the body for
// one token per workgroup of 4 waves.  Shared by the quantizer kernels and by the decode kernel that
// quantizes its one token itself.
#pragma once
#include "common.h"

// Selection key = bit pattern of |x| (15 bits for bfloat16; monotone for finite values, -0 equals
// +0).  tau = the topk-th largest key; keys above tau are kept, and of the keys equal to tau the
// first r in channel order, r = topk - #(key > tau).  A wave owns a contiguous range of chunks of
// 256 channels, a lane 4 consecutive channels of each chunk, so channel order is (wave, chunk,
// lane, j) order.  Everything is counted on the vector ALU (the scalar unit, which ballots go
// through, is shared by the four SIMDs of a compute unit); lane counts are summed inside the wave
// with DPP adds.
__device__ __forceinline__ int qa_wave_sum_dpp(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);    // quad_perm [1,0,3,2]
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);    // quad_perm [2,3,0,1]
  v += __builtin_amdgcn_update_dpp(0, v, 0x124, 0xF, 0xF, false);   // row_ror:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x128, 0xF, 0xF, false);   // row_ror:8
  return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) +
         __builtin_amdgcn_readlane(v, 32) + __builtin_amdgcn_readlane(v, 48);
}

#define QA_GUARD 0x80008000u

// Four consecutive channels of a token as bfloat16 bit patterns (two words).  GLU = 0: the row
// itself (`a`).  GLU = 1 / 2: the token is H = bf16(U * max(G, 0)^2) (eq. 5, float32 steps in that
// order) of a gate row `a` and an up row `b`, bfloat16 / float32: the product never goes to memory.
template <int GLU>
__device__ __forceinline__ uint2 qa_token4(const void* a, const void* b, int ch) {
  if (GLU == 0) return *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(a) + ch);
  float g[4], u[4];
  if (GLU == 1) {
    const uint2 gv = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(a) + ch);
    const uint2 uv = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint16_t*>(b) + ch);
    g[0] = __uint_as_float(gv.x << 16); g[1] = __uint_as_float(gv.x & 0xFFFF0000u);
    g[2] = __uint_as_float(gv.y << 16); g[3] = __uint_as_float(gv.y & 0xFFFF0000u);
    u[0] = __uint_as_float(uv.x << 16); u[1] = __uint_as_float(uv.x & 0xFFFF0000u);
    u[2] = __uint_as_float(uv.y << 16); u[3] = __uint_as_float(uv.y & 0xFFFF0000u);
  } else {
    const float4 gv = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(a) + ch);
    const float4 uv = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(b) + ch);
    g[0] = gv.x; g[1] = gv.y; g[2] = gv.z; g[3] = gv.w;
    u[0] = uv.x; u[1] = uv.y; u[2] = uv.z; u[3] = uv.w;
  }
  u32 h[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const float r = fmaxf(g[j], 0.0f);
    const float rr = r * r;
    h[j] = bl_f32_to_bf16_rne(u[j] * rr);
  }
  return make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
}

// Bit planes.  The search for tau looks at one bit of every key per pass, so the keys of a lane are
// turned into bit planes once: 16 keys (8 words of two 16-bit rows) -> 16 planes of 16 bits (word
// p / 2, half p % 2 holds bit p of the 16 keys, key r in bit r).  The usual recursive block swap, on
// packed halves: byte blocks with v_perm, 4-, 2- and 1-bit blocks with shift / xor / mask.
__device__ __forceinline__ void qa_bit_transpose16(u32 (&w)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const u32 a = w[i], b = w[i + 4];
    w[i] = __builtin_amdgcn_perm(b, a, 0x06020400u);        // a.b0 b.b0 a.b2 b.b2
    w[i + 4] = __builtin_amdgcn_perm(b, a, 0x07030501u);    // a.b1 b.b1 a.b3 b.b3
  }
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int i = (k & 1) + 4 * (k >> 1);                   // 0, 1, 4, 5
    const u32 t = ((w[i] >> 4) ^ w[i + 2]) & 0x0F0F0F0Fu;
    w[i + 2] ^= t;
    w[i] ^= t << 4;
  }
#pragma unroll
  for (int i = 0; i < 8; i += 2) {
    const u32 t = ((w[i] >> 2) ^ w[i + 1]) & 0x33333333u;
    w[i + 1] ^= t;
    w[i] ^= t << 2;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const u32 t = ((w[i] >> 1) ^ (w[i] >> 16)) & 0x5555u;
    w[i] ^= (t << 16) | (t << 1);
  }
}

// Codes of one wave's chunks once tau is known.  Of the keys equal to tau the first r in channel
// order are kept (eq_base = keys equal to tau in earlier waves, eq_here = in this wave): for a whole
// wave that is all of them, none of them, or (for one wave of the token) a prefix found with
// ballots.  raw / pg: the wave's chunks as loaded / with the guard bits set; out0: this lane's word
// of the wave's first chunk (chunk i at out0[64 i]); sum: the sum of the lane's codes is added to it.
// ties_matter = false: the keys equal to tau have code 0 whether they are kept or not (tau is at least 8
// binades below the row maximum: |x| s <= 127 / 256), so the wave keeps all of them and the prefix
// search is skipped -- the usual case for rows that are mostly zeros, where tau = 0.
template <int CPW>
__device__ __forceinline__ void qa_code_chunks(const u32 (&raw)[CPW][2], const u32 (&pg)[CPW][2], int nc, u32 tau,
                                               int r, int eq_base, int eq_here, float s, u32* out0, int& sum,
                                               bool ties_matter = true) {
  const int lane = threadIdx.x & 63;
  const bool eq_all = !ties_matter || eq_base + eq_here <= r;
  const bool eq_none = eq_base >= r;
  const u32 t1 = (tau + 1u) * 0x10001u, t0 = tau * 0x10001u;
  const u32 tk = eq_all ? t0 : t1;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
#pragma unroll
  for (int i = 0; i < CPW; ++i) {
    if (i < nc) {                                         // wave-uniform
      // kept keys as guard-bit flags: key >= tau where the wave keeps all its keys equal to tau,
      // key > tau where it keeps none of them
      u32 k0 = (pg[i][0] - tk) & QA_GUARD, k1 = (pg[i][1] - tk) & QA_GUARD;
      if (!eq_all && !eq_none) {                          // the wave that holds the r-th equal key
        const u32 e0 = ((pg[i][0] - t0) & QA_GUARD) ^ k0, e1 = ((pg[i][1] - t0) & QA_GUARD) ^ k1;
        const bool eqf[4] = {(e0 & 0x8000u) != 0, (e0 >> 31) != 0, (e1 & 0x8000u) != 0, (e1 >> 31) != 0};
        uint64_t beq[4], any_eq = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) { beq[j] = __ballot(eqf[j]); any_eq |= beq[j]; }
        if (any_eq) {
          int rank = eq_base, in_chunk = 0;
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            rank += __popcll(beq[j] & lt_mask);
            in_chunk += __popcll(beq[j]);
          }
          if (eqf[0]) { if (rank < r) k0 |= 0x8000u; ++rank; }
          if (eqf[1]) { if (rank < r) k0 |= 0x80000000u; ++rank; }
          if (eqf[2]) { if (rank < r) k1 |= 0x8000u; ++rank; }
          if (eqf[3]) { if (rank < r) k1 |= 0x80000000u; ++rank; }
          eq_base += in_chunk;
        }
      }
      // codes: |x * s| <= 127 for every finite row, so RoundClip is the rounding alone, taken
      // from the low byte of (x * s) + 1.5 * 2^23 (round to nearest even at integer spacing)
      const float xs[4] = {__uint_as_float(raw[i][0] << 16), __uint_as_float(raw[i][0] & 0xFFFF0000u),
                           __uint_as_float(raw[i][1] << 16), __uint_as_float(raw[i][1] & 0xFFFF0000u)};
      u32 rb[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) rb[j] = __float_as_uint(xs[j] * s + 12582912.0f);
      const u32 w01 = __builtin_amdgcn_perm(rb[1], rb[0], 0x0c0c0400u);   // bytes: rb0.b0, rb1.b0, 0, 0
      const u32 w23 = __builtin_amdgcn_perm(rb[3], rb[2], 0x04000c0cu);   // bytes: 0, 0, rb2.b0, rb3.b0
      // the four flags (bits 15 and 31 of k0, k1) as a byte mask: bytes 1 and 3 of each word hold
      // 0x80 or 0; shifted down that is 1 or 0 per byte, times 255 it is the mask
      const u32 keep4 = (__builtin_amdgcn_perm(k1, k0, 0x07050301u) >> 7) * 255u;
      const u32 word = (w01 | w23) & keep4;
      sum = __builtin_amdgcn_sdot4((int)word, 0x01010101, sum, false);
      out0[i * 64] = word;
    }
  }
}

// Body for one token and one workgroup of 4 waves: row x of K channels -> Kp / 4 code words at
// `out`, the dequantization scale at `scale_out` (both may point into LDS), the sum of the codes at
// `rowsum_out` if not null.  Every thread of the workgroup must call it (it has barriers).
template <int CPW, int GLU = 0>
__device__ __forceinline__ void qa_topk_row_regs(const void* __restrict__ x, const void* __restrict__ x2, int K,
                                                 int Kp, int topk, float eps, u32* out, float* scale_out,
                                                 int32_t* rowsum_out) {
  constexpr int NW = 4;
  __shared__ __align__(16) u32 sh_a[2][NW];
  __shared__ __align__(16) u32 sh_b[NW];
  __shared__ __align__(16) u32 sh_c[NW];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int n_chunks = Kp / 256;
  const int per_wave = (n_chunks + NW - 1) / NW;          // <= CPW by dispatch
  const int c_begin = min(wave * per_wave, n_chunks), c_end = min(c_begin + per_wave, n_chunks);
  const int nc = c_end - c_begin;                         // chunks of this wave; the rest hold key 0

  // one pass over the row: 4 consecutive channels (8 bytes) per lane and chunk, zero beyond K
  // (one address per lane, the chunks at constant distances from it)
  u32 raw[CPW][2], pg[CPW][2];
  u32 km2 = QA_GUARD;
  const int ch0 = c_begin * 256 + lane * 4;
  const int left = K - ch0;                               // channels from this lane's first one on
#pragma unroll
  for (int i = 0; i < CPW; ++i) {
    uint2 v = make_uint2(0u, 0u);
    if (i < nc && i * 256 < left) v = qa_token4<GLU>(x, x2, ch0 + i * 256);   // K % 4 == 0 by dispatch
    raw[i][0] = v.x; raw[i][1] = v.y;
    pg[i][0] = v.x | QA_GUARD; pg[i][1] = v.y | QA_GUARD;
  }
  {
    typedef unsigned short us2 __attribute__((ext_vector_type(2)));
    us2 km = __builtin_bit_cast(us2, km2);
#pragma unroll
    for (int i = 0; i < CPW; ++i)
#pragma unroll
      for (int h = 0; h < 2; ++h) km = __builtin_elementwise_max(km, __builtin_bit_cast(us2, pg[i][h]));   // v_pk_max_u16
    km2 = __builtin_bit_cast(u32, km);
  }
  u32 kmax = max(km2 & 0x7FFFu, (km2 >> 16) & 0x7FFFu);
  kmax = bl_wave_max_u32(kmax);
  if (lane == 0) sh_b[wave] = kmax;
  __syncthreads();
  {
    const uint4 t = *reinterpret_cast<const uint4*>(sh_b);
    kmax = (u32)__builtin_amdgcn_readfirstlane((int)max(max(t.x, t.y), max(t.z, t.w)));
  }
  const float gamma = __uint_as_float(kmax << 16);
  const float s = 127.0f / (gamma + eps);
  if (threadIdx.x == 0) scale_out[0] = gamma / 127.0f;

  // tau = topk-th largest key, bit by bit from the top, on bit planes.  `act` marks the keys whose
  // bits above the current one equal tau's; `above` counts the keys already known to be larger.
  // A bit of tau is 1 iff at least topk keys are >= the candidate, i.e. above + #(active keys with
  // the bit set) >= topk; then those keys stay active, otherwise they join `above`.  Cost per pass:
  // a handful of instructions per lane instead of 1.5 per key.
  constexpr int NBK = CPW / 4;                            // blocks of 16 keys per lane
  static_assert(CPW % 4 == 0 && NBK >= 1 && NBK <= 3, "16 keys per block, at most 48 keys per lane");
  // Mostly-zero rows (the FFN's intermediate state) need no search at all: a key at or below
  // C = kmax - 8 binades has code 0 kept or not, so if no more than topk keys lie above C, keeping
  // exactly those gives the codes of the exact selection.  One count and one barrier decide it.
  if (kmax > 1024u) {                                     // workgroup-uniform
    const u32 cc = (kmax - 1024u + 1u) * 0x10001u;        // key > C  <=>  guard bit of (key | guard) - (C + 1) stays set
    int n_hi = 0;
#pragma unroll
    for (int i = 0; i < CPW; ++i)
#pragma unroll
      for (int h = 0; h < 2; ++h) n_hi += __popc((pg[i][h] - cc) & QA_GUARD);
    n_hi = qa_wave_sum_dpp(n_hi);
    if (lane == 0) sh_c[wave] = (u32)n_hi;
    __syncthreads();
    const uint4 t = *reinterpret_cast<const uint4*>(sh_c);
    const int total_hi = __builtin_amdgcn_readfirstlane((int)(t.x + t.y + t.z + t.w));
    if (total_hi <= topk) {
      int sum = 0;
      qa_code_chunks<CPW>(raw, pg, nc, kmax - 1024u, 0, 0, 0, s, out + c_begin * 64 + lane, sum, false);
      if (rowsum_out) {
        sum = qa_wave_sum_dpp(sum);
        if (lane == 0) sh_a[0][wave] = (u32)sum;
        __syncthreads();
        if (threadIdx.x == 0) {
          const uint4 t2 = *reinterpret_cast<const uint4*>(sh_a[0]);
          rowsum_out[0] = (int32_t)(t2.x + t2.y + t2.z + t2.w);
        }
      }
      return;
    }
    // (sh_c is written again only after the barriers of the passes below)
  }
  u32 pl[NBK][8];
#pragma unroll
  for (int B = 0; B < NBK; ++B) {
#pragma unroll
    for (int i = 0; i < 8; ++i) pl[B][i] = raw[4 * B + (i >> 1)][i & 1] & 0x7FFF7FFFu;
    qa_bit_transpose16(pl[B]);
  }
  // keys of chunks this wave does not have (key 0) stay out: they would count as equal to tau = 0
  const unsigned long long real = nc >= 16 ? ~0ull : ((1ull << (4 * nc)) - 1ull);
  u32 act_lo = (u32)real, act_hi = (u32)(real >> 32) & 0xFFFFu;
  if (NBK == 1) act_lo &= 0xFFFFu;
  u32 tau = 0;
  int above = 0;
  int pass = 0;
  const int top_bit = 31 - __clz((int)(kmax | 1u));
#pragma unroll
  for (int bit = 14; bit >= 0; --bit) {
    if (bit <= top_bit) {                                 // wave-uniform
      u32 p_lo, p_hi = 0;
      if (NBK == 1) p_lo = (bit & 1) ? pl[0][bit >> 1] >> 16 : pl[0][bit >> 1] & 0xFFFFu;
      else p_lo = __builtin_amdgcn_perm(pl[1][bit >> 1], pl[0][bit >> 1], (bit & 1) ? 0x07060302u : 0x05040100u);
      if (NBK == 3) p_hi = (bit & 1) ? pl[2][bit >> 1] >> 16 : pl[2][bit >> 1] & 0xFFFFu;
      const u32 x_lo = act_lo & p_lo, x_hi = act_hi & p_hi;
      const int cnt = qa_wave_sum_dpp(__popc(x_lo) + __popc(x_hi));
      if (lane == 0) sh_a[pass & 1][wave] = (u32)cnt;
      __syncthreads();                                    // one barrier per pass: slots alternate
      const uint4 t = *reinterpret_cast<const uint4*>(sh_a[pass & 1]);
      const int total = __builtin_amdgcn_readfirstlane((int)(t.x + t.y + t.z + t.w));
      if (above + total >= topk) {
        tau |= 1u << bit;
        act_lo = x_lo;
        act_hi = x_hi;
      } else {
        above += total;
        act_lo ^= x_lo;
        act_hi ^= x_hi;
      }
      ++pass;
    }
  }

  // keys equal to tau per wave (the active ones); `above` is the number of keys larger than tau
  {
    const int eq = qa_wave_sum_dpp(__popc(act_lo) + __popc(act_hi));
    __syncthreads();                                      // sh_b was read above by every thread
    if (lane == 0) sh_c[wave] = (u32)eq;
    __syncthreads();
  }
  const uint4 eqw4 = *reinterpret_cast<const uint4*>(sh_c);
  const int r = topk - above;
  const u32 eqs[4] = {eqw4.x, eqw4.y, eqw4.z, eqw4.w};
  int eq_base = 0;                                        // keys equal to tau in earlier waves
#pragma unroll
  for (int w = 0; w < NW - 1; ++w)
    if (w < wave) eq_base += (int)eqs[w];
  eq_base = __builtin_amdgcn_readfirstlane(eq_base);
  const int eq_here = __builtin_amdgcn_readfirstlane((int)sh_c[wave]);
  int sum = 0;
  qa_code_chunks<CPW>(raw, pg, nc, tau, r, eq_base, eq_here, s, out + c_begin * 64 + lane, sum, tau + 1024u > kmax);
  if (rowsum_out) {
    sum = qa_wave_sum_dpp(sum);
    __syncthreads();
    if (lane == 0) sh_a[0][wave] = (u32)sum;
    __syncthreads();
    if (threadIdx.x == 0) {
      const uint4 t = *reinterpret_cast<const uint4*>(sh_a[0]);
      rowsum_out[0] = (int32_t)(t.x + t.y + t.z + t.w);
    }
  }
}

// ---------------------------------------------------------------- one token, 8 waves, 3 bits of tau per pass
// The same selection for a workgroup of 8 waves that has one token to quantize and little time (the
// decode kernel that streams a weight matrix past one token), and that needs the token's CODES only
// (no mask, no index list).  What costs there is not the counting but the chain of dependent steps --
// count, add up over the workgroup, decide, next bits -- so:
//   * Keys are cut to 11 bits.  A channel below gamma / 256 has code 0 whether Top_k keeps it or not
//     (|x| s < 127 / 256 rounds to 0), so the keys at or below C = key(gamma) - 8 binades are
//     collapsed into one lowest class: key' = max(key, C) - C, at most 1024.  If the topk-th largest
//     key' is positive the selection among the keys above C is the exact one, ties included; if it
//     is 0 every key above C is kept, and what happens inside the lowest class changes no code.
//   * A pass settles three bits of tau' at once: the still-undecided keys are split by their next
//     three bits into eight classes (bit planes: fourteen ANDs), the class sizes are packed two to a
//     word, added over the wave with DPP (row rotations, then the row broadcasts into the last row)
//     and left in LDS by the wave's last lane; after one barrier lane l takes wave l % 8's words,
//     three more DPP steps give every lane the workgroup's sums, and the decision is scalar
//     arithmetic.  Four passes (bits 10..8, 7..5, 4..2, 1..0).
//   * The last pass's per-wave class sizes are also the per-wave counts of keys equal to tau that the
//     tie rule (lower channel first; waves own contiguous channel ranges) needs: no further exchange.
//   raw     this wave's chunks of 256 channels as loaded by the caller (chunk i of the wave = chunk
//           c_begin + i of the token; 4 consecutive channels per lane; zero beyond K and beyond nc)
//   sh      80 words of LDS scratch (16-byte aligned): row maxima [8], early counts [8], class sizes [2][32]
// Chunks are dealt to the waves in contiguous ranges of per_wave = ceil(n_chunks / 8), so channel
// order is (wave, chunk, lane, j) order as in the 4-wave body.  Every thread of the workgroup must
// call it (it has barriers); the caller adds the barrier that publishes the codes.
__device__ __forceinline__ u32 qa_sum8_dpp(u32 x) {       // sum over each aligned group of 8 lanes, in all of them
  int v = (int)x;
  v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);      // quad_perm [1,0,3,2]
  v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);      // quad_perm [2,3,0,1]
  v += __builtin_amdgcn_update_dpp(0, v, 0x124, 0xF, 0xF, false);     // row_ror:4 (lanes hold every value twice per row)
  return (u32)v;
}
__device__ __forceinline__ u32 qa_max8_dpp(u32 x) {
  u32 v = x;
  v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, false));
  v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, false));
  v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x124, 0xF, 0xF, false));
  return v;
}

template <int CPW>
__device__ __forceinline__ void qa_topk_row_regs8(const u32 (&raw)[CPW][2], int nc, int c_begin, int topk, float eps,
                                                  u32* out, float* scale_out, u32* sh) {
  static_assert(CPW == 4 || CPW == 8, "16 or 32 keys per lane");
  constexpr int NBK = CPW / 4;
  typedef unsigned short us2 __attribute__((ext_vector_type(2)));
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  u32* sh_max = sh;              // [8]
  u32* sh_cnt = sh + 16;         // [2][8 waves][4] class sizes of a pass per wave (slots alternate)

  u32 pg[CPW][2];
  u32 km2 = QA_GUARD;
  {
    us2 km = __builtin_bit_cast(us2, km2);
#pragma unroll
    for (int i = 0; i < CPW; ++i)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        pg[i][h] = raw[i][h] | QA_GUARD;
        km = __builtin_elementwise_max(km, __builtin_bit_cast(us2, pg[i][h]));   // v_pk_max_u16
      }
    km2 = __builtin_bit_cast(u32, km);
  }
  u32 kmax = max(km2 & 0x7FFFu, (km2 >> 16) & 0x7FFFu);
  kmax = bl_wave_max_u32(kmax);
  if (lane == 0) sh_max[wave] = kmax;
  __syncthreads();
  kmax = (u32)__builtin_amdgcn_readfirstlane((int)qa_max8_dpp(sh_max[lane & 7]));
  const float gamma = __uint_as_float(kmax << 16);
  const float s = 127.0f / (gamma + eps);
  if (tid == 0) scale_out[0] = gamma / 127.0f;

  const u32 C = kmax > 1024u ? kmax - 1024u : 0u;
  // Wide rows are FFN states, mostly zeros: if no more than topk keys lie above C, keeping exactly those
  // gives the codes of the exact selection (a key at or below C has code 0 kept or not), and neither bit
  // planes nor passes are needed.  One count, one barrier (words 8..15 of `sh`).
  if constexpr (CPW == 8) {
    if (C > 0u) {                                         // workgroup-uniform
      const u32 cc = (C + 1u) * 0x10001u;
      int n_hi = 0;
#pragma unroll
      for (int i = 0; i < CPW; ++i)
#pragma unroll
        for (int h = 0; h < 2; ++h) n_hi += __popc((pg[i][h] - cc) & QA_GUARD);
      n_hi = qa_wave_sum_dpp(n_hi);
      if (lane == 0) sh[8 + wave] = (u32)n_hi;
      __syncthreads();
      const int total_hi = __builtin_amdgcn_readfirstlane((int)qa_sum8_dpp(sh[8 + (lane & 7)]));
      if (total_hi <= topk) {
        int sum = 0;
        qa_code_chunks<CPW>(raw, pg, nc, C, 0, 0, 0, s, out + c_begin * 64 + lane, sum, false);
        return;
      }
    }
  }
  // 11-bit keys and their bit planes: plane(bit) has key r of the lane in bit r
  const us2 C2 = __builtin_bit_cast(us2, C * 0x10001u);
  u32 pl[NBK][8];
#pragma unroll
  for (int B = 0; B < NBK; ++B) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const us2 k = __builtin_bit_cast(us2, raw[4 * B + (i >> 1)][i & 1] & 0x7FFF7FFFu);
      pl[B][i] = __builtin_bit_cast(u32, (us2)(__builtin_elementwise_max(k, C2) - C2));
    }
    qa_bit_transpose16(pl[B]);
  }
  auto plane = [&](int bit) -> u32 {
    if (bit < 0) return 0u;
    if (NBK == 1) return (bit & 1) ? pl[0][bit >> 1] >> 16 : pl[0][bit >> 1] & 0xFFFFu;
    return __builtin_amdgcn_perm(pl[NBK - 1][bit >> 1], pl[0][bit >> 1], (bit & 1) ? 0x07060302u : 0x05040100u);
  };
  // keys of chunks this wave does not have stay out: they would count as members of the lowest class
  u32 act = nc >= 8 ? ~0u : ((1u << (4 * nc)) - 1u);
  if (NBK == 1) act &= 0xFFFFu;
  u32 tau = 0;                                            // tau' (11 bits)
  int above = 0;
  int d = 0;
  uint4 q = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int b0 = 8 - 3 * p;                             // the pass settles bits b0 + 2, b0 + 1, b0 (b0 = -1: two bits)
    const u32 P2 = plane(b0 + 2), P1 = plane(b0 + 1), P0 = plane(b0);
    // classes by the three bits: m[c] = undecided keys whose bits spell c
    u32 m[8];
    {
      const u32 hi = act & P2, lo = act ^ hi;
      const u32 h1 = hi & P1, h0 = hi ^ h1, l1 = lo & P1, l0 = lo ^ l1;
      m[7] = h1 & P0; m[6] = h1 ^ m[7];
      m[5] = h0 & P0; m[4] = h0 ^ m[5];
      m[3] = l1 & P0; m[2] = l1 ^ m[3];
      m[1] = l0 & P0; m[0] = l0 ^ m[1];
    }
    // class sizes, two to a word (a token has at most 16384 keys: no carry between the halves)
    u32 w[4];
    w[0] = (u32)__popc(m[1]) | ((u32)__popc(m[2]) << 16);
    w[1] = (u32)__popc(m[3]) | ((u32)__popc(m[4]) << 16);
    w[2] = (u32)__popc(m[5]) | ((u32)__popc(m[6]) << 16);
    w[3] = (u32)__popc(m[7]) | ((u32)__popc(m[0]) << 16);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int v = (int)w[j];
      v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);    // quad_perm [1,0,3,2]
      v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);    // quad_perm [2,3,0,1]
      v += __builtin_amdgcn_update_dpp(0, v, 0x124, 0xF, 0xF, false);   // row_ror:4
      v += __builtin_amdgcn_update_dpp(0, v, 0x128, 0xF, 0xF, false);   // row_ror:8
      v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);   // row_bcast:15 into rows 1 and 3
      v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);   // row_bcast:31 into rows 2 and 3
      w[j] = (u32)v;                                      // (the wave's sum, in the lanes of the last row)
    }
    u32* slot = sh_cnt + (p & 1) * 32;                    // (one barrier per pass: slots alternate)
    if (lane == 63) *reinterpret_cast<uint4*>(slot + 4 * wave) = make_uint4(w[0], w[1], w[2], w[3]);
    __syncthreads();
    q = *reinterpret_cast<const uint4*>(slot + 4 * (lane & 7));         // lane l: the sizes in wave l % 8
    const u32 t0 = (u32)__builtin_amdgcn_readfirstlane((int)qa_sum8_dpp(q.x));
    const u32 t1 = (u32)__builtin_amdgcn_readfirstlane((int)qa_sum8_dpp(q.y));
    const u32 t2 = (u32)__builtin_amdgcn_readfirstlane((int)qa_sum8_dpp(q.z));
    const u32 t3 = (u32)__builtin_amdgcn_readfirstlane((int)qa_sum8_dpp(q.w));
    // cum[c] = undecided keys of class c or higher; the topk-th largest key is in the highest class
    // c with above + cum[c] >= topk (class 0 if none).  Scalar arithmetic from here.
    const int need = topk - above;
    int cum[9];
    cum[8] = 0;
    cum[7] = (int)(t3 & 0xFFFFu);
    cum[6] = cum[7] + (int)(t2 >> 16);
    cum[5] = cum[6] + (int)(t2 & 0xFFFFu);
    cum[4] = cum[5] + (int)(t1 >> 16);
    cum[3] = cum[4] + (int)(t1 & 0xFFFFu);
    cum[2] = cum[3] + (int)(t0 >> 16);
    cum[1] = cum[2] + (int)(t0 & 0xFFFFu);
    d = 0;
#pragma unroll
    for (int c = 1; c < 8; ++c) d += cum[c] >= need ? 1 : 0;
    int add = cum[1];
#pragma unroll
    for (int c = 1; c < 8; ++c)
      if (d == c) add = cum[c + 1];
    above += add;
    // the class's members: keys whose three bits spell d
    act &= (P2 ^ ((d & 4) ? 0u : ~0u)) & (P1 ^ ((d & 2) ? 0u : ~0u)) & (P0 ^ ((d & 1) ? 0u : ~0u));
    tau |= b0 >= 0 ? (u32)d << b0 : (u32)d >> 1;
  }

  // Keys equal to tau per wave = the sizes of class d of the last pass, which lane l still holds for
  // wave l % 8.  tau' = 0: the lowest class is dropped as a whole (its codes are 0 either way).
  const u32 qw = d == 0 ? q.w : d <= 2 ? q.x : d <= 4 ? q.y : d <= 6 ? q.z : q.w;
  const u32 e = ((d == 0 || ((d - 1) & 1)) ? qw >> 16 : qw) & 0xFFFFu;
  const int r = topk - above;
  int eq_base = 0, eq_here = 0;                           // keys equal to tau in earlier waves, in this one
#pragma unroll
  for (int ww = 0; ww < 8; ++ww) {
    const int ev = __builtin_amdgcn_readlane((int)e, ww);
    if (ww < wave) eq_base += ev;
    if (ww == wave) eq_here = ev;
  }
  const bool low = tau == 0;
  int sum = 0;
  qa_code_chunks<CPW>(raw, pg, nc, tau + C, r, low ? r : eq_base, eq_here, s, out + c_begin * 64 + lane, sum);
}
