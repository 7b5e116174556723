/*
 * bitlinear.h — C ABI of the MI355X (gfx950) quantized linear layers of BitNet a4.8
 * (arXiv 2411.04965).
 *
 * Notation follows the paper: X activations [M, K] row-major (one token per row),
 * W latent weights [N, K] row-major (out x in), Y = Q(X) . Q_w(W)^T [M, N] row-major.
 *
 * General rules for every entry point
 *   - All data pointers are DEVICE pointers unless a comment says "host".
 *   - The caller owns every buffer.  The library never allocates, frees or
 *     synchronises; every kernel is enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream) and the call returns at once.
 *   - Data pointers must be 16-byte aligned (per-token float32 scales, E8M0 block scales and
 *     alpha: 4 bytes; G and H of bitlinear_a4_up_gated: their element size); rows are dense
 *     (no strides).
 *   - Inputs must be finite.  NaN/Inf give unspecified codes, never a trap.
 *   - Return value: BL_OK (0) or a negative bl_status.  Arguments are validated
 *     before anything is launched; on an argument error nothing has been enqueued.  The one
 *     exception is BL_EHIP (the driver refused a launch or a kernel attribute): a call that
 *     runs several kernels may by then have enqueued the earlier ones.
 *   - eps is the epsilon of eq. 2, 3 and 7 (the paper gives no value; 1e-5 is used
 *     by the tests and the benchmark).  eps = 0 is accepted, but an all-zero token (or weight
 *     matrix) then scales by 1 / 0: its codes are unspecified and a linear layer's outputs
 *     for that token may be NaN.  With eps > 0 an all-zero token gives zero codes and outputs.
 *
 * Packed formats (all little-endian; Kp = bl_padded_k(K) = K rounded up to 256,
 * Np = N rounded up to 16; padding codes are zero):
 *
 *   Ternary code (2 bits, two's complement): 00 = 0, 01 = +1, 11 = -1, 10 unused.
 *
 *   BL_W_GEMM   tiles of 16 output channels x 256 input channels, 1024 bytes each,
 *               stored tile-row major: tile (nt, kt) at byte ((nt * Kp/256) + kt) * 1024.
 *               Inside a tile, the 16 bytes at offset ((g*16 + i) * 16) hold output
 *               channel n = 16*nt + i, input channels k0 = 256*kt + 64*g ... k0+63 as four
 *               32-bit words; word t covers k0 + 16*t ... + 15, and inside a word the
 *               2-bit field f (bits 2f, 2f+1) holds channel k0 + 16*t + 4*(f%4) + f/4.
 *   BL_W_KMAJOR input-channel major inside column blocks of 512 outputs (N rounded up to 512):
 *               the 128 bytes at byte (cb * K + k) * 128 hold outputs 512*cb ... 512*cb+511 of
 *               input channel k; inside, 32-bit word d holds outputs 512*cb + 16*d ... + 15,
 *               field f = n % 16.  (K rows only, no K padding.)  Used by the row-skipping
 *               decode path: one weight row segment is one 128-byte line.
 *
 *   BL_W_MX4    ternary weights as E2M1 nibbles (0000 = 0, 0010 = +1, 1010 = -1) in the order the
 *               block-float matrix instruction reads them: blocks of 32 output channels x 128
 *               input channels, 2048 bytes each, block (nb, kb) at byte (nb * Kp/128 + kb) * 2048
 *               (N rounded up to 32).  Inside a block, row r = n % 32 takes 64 bytes; its 16-byte
 *               piece p holds unit u = p ^ ((r / 4) % 4), i.e. channels 128*kb + 32*u ... + 31,
 *               channel i of the unit in nibble i (low nibble of a byte first).  Used by the
 *               prefill GEMM of the INT4 path; twice the bytes of BL_W_GEMM.
 *
 *   BL_W_MX2    the same blocks of 32 output channels x 128 input channels for the block-float GEMM,
 *               with the weights kept as 2-bit codes (1024 bytes per block, block (nb, kb) at byte
 *               (nb * Kp/128 + kb) * 1024) and expanded to E2M1 in registers.  Row r = n % 32 takes
 *               32 bytes; its 8-byte piece p holds unit u = p ^ ((r / 8) % 4), i.e. channels
 *               128*kb + 32*u ... + 31, as two 32-bit words of 16 channels each: nibble j (0..7) of a
 *               word holds channels j and 8 + j of its 16, as (sign of j, sign of 8+j, magnitude of j,
 *               magnitude of 8+j) from bit 3 down to bit 0, so that `w & 0xAAAAAAAA` and
 *               `(w << 1) & 0xAAAAAAAA` are the E2M1 nibbles of channels 0..7 and 8..15.
 *   BL_W_ROWS   output-channel major: row n takes Kp/4 bytes at n * Kp/4; 32-bit word w of the
 *               row holds channels 16w ... 16w+15, channel 16w + f in bits 2f, 2f+1 (so byte b of
 *               the word holds channels 4b ... 4b+3).  A row can be fetched, or skipped, on its
 *               own: the layout of the gate-first up projection (bitlinear_a4_up_gated).
 *
 *   INT4 activations  [M][Kp/2] bytes.  Channels are taken 8 at a time into one
 *               32-bit word; byte b (0..3) of the word is (q[k0+b] & 15) | (q[k0+4+b] << 4).
 *   INT4 activations, MX6 form: the same 16 levels, each stored as its 6-bit E3M2 code
 *               (bit 5 sign, bits 4..2 exponent with bias 3, bits 1..0 mantissa; all INT4
 *               levels are exact), in blocks of 32 tokens x 128 channels, 3072 bytes each,
 *               block (mb, kb) at byte (mb * Kp/128 + kb) * 3072 (M rounded up to 32; rows past
 *               M are not written).  The 32 channels of unit u (channels 128*kb + 32*u ... + 31)
 *               form a 24-byte little-endian bit stream, channel i in bits 6i ... 6i+5.  Inside a
 *               block, token row r = m % 32 keeps stream bytes 0..15 of unit u in the 16-byte
 *               piece p = u ^ ((r / 4) % 4) at byte r*64 + 16*p, and stream bytes 16..23 in the
 *               8-byte piece p' = u ^ ((r / 8) % 4) at byte 2048 + r*32 + 8*p'.
 *   INT8 activations  [M][Kp] bytes, plain int8, zeros where the Top_k mask is 0.
 *   FP4 activations   [M][Kp/2] bytes of E2M1 nibbles (bit 3 sign, bits 2..0 code of
 *               {0, .5, 1, 1.5, 2, 3, 4, 6}).  Channels are taken 16 at a time into two
 *               32-bit words; nibble j (bits 4j..4j+3) of word 0 holds channel
 *               k0 + 8*(j%2) + j/2, nibble j of word 1 holds channel k0 + 4 + 8*(j%2) + j/2.
 *               Block scales: one E8M0 byte (value 2^(byte-127)) per 32 channels,
 *               [M][Kp/32] bytes.
 *   FP4 activations, MX form: the same nibbles and scales in blocks of 32 tokens x 128
 *               channels.  Codes: 2048 bytes per block, block (mb, kb) at byte
 *               (mb * Kp/128 + kb) * 2048 (M rounded up to 32; rows past M are not written);
 *               token row r = m % 32 takes 64 bytes, its 16-byte piece p holds unit
 *               u = p ^ ((r / 4) % 4), i.e. channels 128*kb + 32*u ... + 31, channel i of the unit
 *               in nibble i (low nibble of a byte first) -- the geometry of BL_W_MX4.
 *               Scales: 128 bytes per block at (mb * Kp/128 + kb) * 128, the E8M0 byte of
 *               unit u of token row r at r*4 + u.
 */
#ifndef BITLINEAR_H_
#define BITLINEAR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { BL_F32 = 0, BL_BF16 = 1 } bl_dtype;

typedef enum {
  BL_ACT_INT4_ABSMEAN = 0,     /* eq. 7 */
  BL_ACT_TOPK_INT8_ABSMAX = 1, /* eq. 1 + eq. 3 */
  BL_ACT_FP4_E2M1_B32 = 2,     /* eq. 8-9 with one power-of-two scale per 32 channels */
  BL_ACT_INT4_ABSMEAN_MX6 = 3, /* eq. 7, levels stored as E3M2 codes for the block-float GEMM */
  BL_ACT_FP4_E2M1_B32_MX = 4,  /* eq. 8-9, codes and scales in the block order of the block-float GEMM */
  BL_ACT_INT4_ABSMEAN2 = 5,    /* eq. 7 with beta = 2 mean|x| (ablation: inputs to the down projection) */
  BL_ACT_INT4_ABSMAX = 6,      /* 4-bit absmax, the form of eq. 3 with 7 in place of 127 (ablation) */
  BL_ACT_FP4_E1M2_B32 = 7      /* eq. 8-9 with E = 1, M = 2 (ablation); quantizer and unpack_act only */
} bl_act_mode;

typedef enum { BL_W_GEMM = 0, BL_W_KMAJOR = 1, BL_W_MX4 = 2, BL_W_ROWS = 3, BL_W_MX2 = 4 } bl_w_layout;

typedef enum {
  BL_OK = 0,
  BL_EINVAL = -1,       /* null pointer, bad enum, non-positive size */
  BL_ESHAPE = -2,       /* size outside what the kernels support */
  BL_EALIGN = -3,       /* a pointer is not 16-byte aligned */
  BL_EWORKSPACE = -4,   /* workspace missing or too small */
  BL_EHIP = -5,         /* a HIP call failed (launch error) */
  BL_EUNSUPPORTED = -6, /* valid request that this build does not implement */
  BL_ESCRATCH = -7      /* bitlinear_a8_sparse_static: the request needs more than BL_STATIC_SCRATCH_BYTES */
} bl_status;

/* Largest sizes accepted: M, N, K >= 1, K <= BL_MAX_K, M*N and N*K below 2^40. */
#define BL_MAX_K 32768

/* K rounded up to the padding unit of the packed formats (256). */
int64_t bl_padded_k(int64_t K);

/* ---------------------------------------------------------------- weights (eq. 2)
 * pack_ternary: alpha = mean|W| over the whole matrix (float64 sum, one rounding to
 * float32); T = RoundClip(W / (alpha + eps), -1, 1); T is written 2-bit packed in
 * `layout`; alpha (not alpha + eps) goes to alpha_out[0] (device, float32).
 *   W          device, [N, K] of w_dtype (BL_F32 or BL_BF16)
 *   packed_out device, pack_ternary_bytes(N, K, layout) bytes, fully overwritten
 *   workspace  device, >= pack_ternary_workspace_bytes(N, K) bytes (partial sums)
 * Offline step (done once per weight matrix). */
size_t pack_ternary_bytes(int64_t N, int64_t K, bl_w_layout layout);
size_t pack_ternary_workspace_bytes(int64_t N, int64_t K);
int pack_ternary(const void* W, bl_dtype w_dtype, int64_t N, int64_t K, float eps,
                 bl_w_layout layout, void* packed_out, float* alpha_out,
                 void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------- activations
 * quantize_act: one token per row, statistics per token.
 *   BL_ACT_INT4_ABSMEAN (eq. 7):  beta = mean|x| (float64 sum, rounded once);
 *       q = RoundClip(x * (sqrt7 / (beta + eps)), -8, 7);  scale_out[m] = beta / sqrt7.
 *   BL_ACT_INT4_ABSMEAN_MX6: the same quantizer, codes in the MX6 form (for BL_W_MX4 / BL_W_MX2 weights).
 *   BL_ACT_INT4_ABSMEAN2 (Section 4.3): eq. 7 with beta = 2 mean|x|; BL_ACT_INT4_ABSMAX (Section 4.3):
 *       gamma = max|x|; q = RoundClip(x * (7 / (gamma + eps)), -8, 7); scale_out[m] = gamma / 7.
 *       Both write the INT4 nibble form; the linear layers take their output as BL_ACT_INT4_ABSMEAN's.
 *   BL_ACT_TOPK_INT8_ABSMAX (eq. 1, 3): mask = the `topk` largest |x| of the token
 *       (exactly topk entries; equal magnitudes: lower channel first; 1 <= topk <= K,
 *       topk = K is the dense INT8 quantizer); gamma = max|x|;
 *       q = mask ? RoundClip(x * (127 / (gamma + eps)), -128, 127) : 0;
 *       scale_out[m] = gamma / 127.
 *   BL_ACT_FP4_E2M1_B32 (eq. 8-9): per block of 32 channels the smallest power of two
 *       2^e with max|x| / 2^e <= 6 (e = 0 for an all-zero block, clamped to [-127, 127]);
 *       codes = x / 2^e rounded to the nearest E2M1 value, ties to the even code, zero
 *       always stored as +0; scale_out = E8M0 bytes (e + 127), [M][Kp/32]; eps unused.
 *   BL_ACT_FP4_E2M1_B32_MX: the same quantizer, codes and scales in the MX form (for BL_W_MX4 /
 *       BL_W_MX2 weights); scale_out then takes round_up(M, 32) * Kp/32 bytes.
 *   BL_ACT_FP4_E1M2_B32 (Section 4.3, the other 4-bit float format of the comparison): eq. 8-9
 *       with E = 1, M = 2, whose values are the uniform grid j / 4, j = 0..7: per block of 32
 *       channels the smallest 2^e with max|x| / 2^e <= 1.75, code j = x / 2^e * 4 rounded half
 *       to even, nibble = sign << 3 | j (zero as +0).  Same containers and sizes as
 *       BL_ACT_FP4_E2M1_B32.  No matrix instruction takes this format as an operand: the linear
 *       entry points and bitlinear_gemm return BL_EUNSUPPORTED for it; quantize_act and
 *       unpack_act (which returns the nibbles) serve it.
 *   X           device, [M, K] of x_dtype
 *   q_out       device, quantize_act_bytes(mode, M, K) bytes, fully overwritten
 *   scale_out   device, float32[M] (INT modes) or uint8[M * Kp/32] (FP4; MX form: M rounded up to 32)
 *   rowsum_out  nullable; int32[M] = sum of the token's codes (INT modes only)
 *   sel_idx_out nullable; TOPK mode only: int32[M, topk], the masked channel indices of
 *               each token in ascending order
 * Multiplications are single float32 operations (never fused), round() is
 * round-half-to-even. */
size_t quantize_act_bytes(bl_act_mode mode, int64_t M, int64_t K);
int quantize_act(const void* X, bl_dtype x_dtype, int64_t M, int64_t K, bl_act_mode mode,
                 int64_t topk, float eps, void* q_out, void* scale_out,
                 int32_t* rowsum_out, int32_t* sel_idx_out, void* stream);

/* ---------------------------------------------------------------- linear layers
 * bitlinear_a4 (eq. 6): Y = Q_INT4(X) . Q_w(W)^T, or the FP4 variant (act_fp4 = 1).
 *   acc[m, n] = sum_k q[m, k] * T[n, k]          exact int32 (INT4 path)
 *   Y[m, n]   = (float(acc) * scale[m]) * alpha  two float32 multiplies, then a
 *               round-to-nearest-even conversion if y_dtype is BL_BF16.
 *   FP4 path: Y = alpha * sum over blocks 2^e * sum_k v_k * T[n, k], accumulated in
 *   float32 by the scaled FP4 matrix instruction (not bit-exact; acc_out must be NULL).
 *   X          device, [M, K] of x_dtype
 *   W_packed   device, output of pack_ternary for [N, K]; layout BL_W_GEMM, or BL_W_MX4 / BL_W_MX2
 *              (the block-float forms): then the activations are quantized to the MX6 form and the
 *              product runs on the 6-bit x 4-bit block-float matrix instruction at twice the
 *              INT8 rate; every product and every partial sum is an integer below 2^24, so the
 *              float32 accumulator equals the int32 one bit for bit.  Size the workspace with
 *              mode BL_ACT_INT4_ABSMEAN_MX6 in that case.  With act_fp4 = 1 and a block-float form the
 *              activations go to the FP4 MX form and the product runs on the same instruction
 *              with the block scales as its scale operand (mode BL_ACT_FP4_E2M1_B32_MX).
 *   alpha      device, float32[1]
 *   Y          device, [M, N] of y_dtype
 *   acc_out    nullable; device int32[M, N], receives the integer accumulators
 *   workspace  device, >= bitlinear_workspace_bytes(mode, M, N, K) bytes; holds the
 *              packed activations and their scales between the two kernels
 * Kernel choice (BL_W_GEMM) is by M: up to BL_DECODE_MAX_M tokens the weights are streamed once
 * by a skinny (decode) kernel, with the quantizer inside the same launch for up to 8 bfloat16
 * tokens (INT4) or one (Top_k + INT8); above that the tiled MFMA GEMM runs.  The block-float forms
 * always take the tiled GEMM.
 *
 * bitlinear_a8_sparse (eq. 1): Y = (Q_INT8(X) (.) Top_k(|X|)) . Q_w(W)^T, same
 * accumulation and rescale.  With layout BL_W_KMAJOR (decode, M <= BL_SPARSE_MAX_M; more tokens:
 * BL_EUNSUPPORTED, their union of kept channels is nearly every channel) only the weight rows of
 * channels with a non-zero code in at least one token are read.
 */
#define BL_DECODE_MAX_M 64
#define BL_SPARSE_MAX_M 8
size_t bitlinear_workspace_bytes(bl_act_mode mode, int64_t M, int64_t N, int64_t K);
int bitlinear_a4(const void* X, bl_dtype x_dtype, int64_t M, int64_t K,
                 const void* W_packed, bl_w_layout layout, const float* alpha, int64_t N,
                 float eps, int act_fp4, void* Y, bl_dtype y_dtype, int32_t* acc_out,
                 void* workspace, size_t workspace_bytes, void* stream);
int bitlinear_a8_sparse(const void* X, bl_dtype x_dtype, int64_t M, int64_t K, int64_t topk,
                        const void* W_packed, bl_w_layout layout, const float* alpha,
                        int64_t N, float eps, void* Y, bl_dtype y_dtype, int32_t* acc_out,
                        void* workspace, size_t workspace_bytes, void* stream);

/* bitlinear_a8_sparse for callers that cannot allocate device memory or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and errors as bitlinear_a8_sparse, without `workspace`: the packed activations, their scales and
 * the integer partial sums of the decode kernels live in a buffer of BL_STATIC_SCRATCH_BYTES inside the
 * library's device image (one per GPU, held until the process ends).  The call allocates and frees
 * nothing and calls no allocating routine.
 *   Limits: M <= BL_DECODE_MAX_M and bitlinear_workspace_bytes(BL_ACT_TOPK_INT8_ABSMAX, M, N, K) <=
 *           BL_STATIC_SCRATCH_BYTES, otherwise BL_ESCRATCH (nothing enqueued).
 *   Every call on a GPU uses that GPU's one buffer, which keeps the last call's contents (nothing in
 *   it needs clearing: each call writes what it reads): calls that overlap in time on one GPU (two
 *   streams, two threads) race; calls on one stream are ordered and safe. */
#define BL_STATIC_SCRATCH_BYTES (8 << 20)
int bitlinear_a8_sparse_static(const void* X, bl_dtype x_dtype, int64_t M, int64_t K, int64_t topk,
                               const void* W_packed, bl_w_layout layout, const float* alpha,
                               int64_t N, float eps, void* Y, bl_dtype y_dtype, int32_t* acc_out,
                               void* stream);

/* The matmul + rescale stage alone, on activations already quantized by quantize_act
 * (what the two calls above run after their quantize kernel).  q and scale are the
 * outputs of quantize_act in `mode`; BL_ACT_INT4_ABSMEAN_MX6 and BL_ACT_FP4_E2M1_B32_MX go with
 * BL_W_MX4 / BL_W_MX2 and with nothing else.  `workspace` must hold bitlinear_workspace_bytes(mode, M, N, K) bytes when
 * M <= BL_DECODE_MAX_M (partial sums of the split-K decode kernels) or the layout is
 * BL_W_KMAJOR; otherwise it may be NULL. */
int bitlinear_gemm(const void* q, const void* scale, bl_act_mode mode, int64_t M, int64_t K,
                   const void* W_packed, bl_w_layout layout, const float* alpha, int64_t N,
                   void* Y, bl_dtype y_dtype, int32_t* acc_out,
                   void* workspace, size_t workspace_bytes, void* stream);

/* Gate and up projection of an FFN block on ONE quantized input, and their ReLU^2 GLU combine
 * (eq. 5 with eq. 6 and eq. 7): the token is quantized once (INT4 absmean),
 *     G = Q(X) . Q_w(W_gate)^T,  U = Q(X) . Q_w(W_up)^T   (accumulate and rescale as bitlinear_a4),
 *     H = bf16(U * max(G, 0)^2)  from the float32 G and U, float32 steps in that order, one rounding.
 * Any of G, U, H may be NULL (not all three): only the others are written.  G and U are the same
 * numbers bitlinear_a4 returns for each matrix, H the same as relu2_glu of their float32 forms.
 *   X          device, [M, K] of x_dtype
 *   W_gate, W_up  device, outputs of pack_ternary for [N, K] in `layout` (BL_W_GEMM, BL_W_MX4 or BL_W_MX2)
 *   G, U       device, [M, N] of gu_dtype, nullable;   H  device, [M, N] bfloat16, nullable
 *   workspace  device, >= bitlinear_gate_up_workspace_bytes(M, N, K, layout) bytes (packed activations,
 *              scales, decode partial sums, and float32 G and U where H is wanted without them)
 * Up to 8 bfloat16 tokens with BL_W_GEMM weights (K % 8 == 0, K <= 8192) run as one launch that
 * streams both matrices once and uses no workspace (it may then be NULL); up to 64 tokens with
 * BL_W_GEMM weights and only H asked for run the quantizer and then one launch over both matrices
 * (K up to 4096 beyond 32 tokens, 8192 beyond 16).  With block-float weights
 * (BL_W_MX4 / BL_W_MX2) and only H asked for, the quantizer is followed by one GEMM over both
 * matrices whose epilogue applies eq. 5 to its accumulators: G and U never reach memory.  Other
 * cases run the quantizer, the two products and the combine as separate kernels. */
size_t bitlinear_gate_up_workspace_bytes(int64_t M, int64_t N, int64_t K, bl_w_layout layout);
int bitlinear_a4_gate_up(const void* X, bl_dtype x_dtype, int64_t M, int64_t K, const void* W_gate,
                         const float* alpha_gate, const void* W_up, const float* alpha_up,
                         bl_w_layout layout, int64_t N, float eps, void* G, void* U, bl_dtype gu_dtype,
                         void* H, void* workspace, size_t workspace_bytes, void* stream);

/* The product stage of bitlinear_a4_gate_up alone, on activations already quantized by quantize_act in
 * mode BL_ACT_INT4_ABSMEAN_MX6: one GEMM over both weight matrices (BL_W_MX4 or BL_W_MX2, [N, K] each)
 * whose epilogue writes H = bf16(U * max(G, 0)^2) (eq. 5 on the rescaled float32 accumulators); G and U
 * are not written.  H device [M, N] bfloat16.  Other layouts: BL_EUNSUPPORTED. */
int bitlinear_gemm_glu(const void* q, const float* scale, int64_t M, int64_t K, const void* W_gate,
                       const float* alpha_gate, const void* W_up, const float* alpha_up,
                       bl_w_layout layout, int64_t N, void* H, void* stream);

/* Gate-first up projection of the FFN for a few tokens (Section 2.1's observation that the up
 * projection is only needed where the gate is open, eq. 5): with G = the gate projection's
 * outputs, H[m, n] = bf16(U[m, n] * max(G[m, n], 0)^2) where U = the INT4 linear (eq. 6, eq. 7) of
 * X with the up weights -- but row n of the weights is read, and U[., n] computed, only if
 * G[m, n] > 0 for some token m; elsewhere H = +0.  U is kept in float32 (never rounded to
 * bfloat16) before the product, float32 steps in the order of relu2_glu.
 *   X        device, [M, K] bfloat16, M <= 4, K % 8 == 0, K <= 8192 and M * bl_padded_k(K) <= 16384
 *   W_rows   device, output of pack_ternary in layout BL_W_ROWS for [N, K]
 *   alpha    device, float32[1]
 *   G        device, [M, N] of g_dtype
 *   H        device, [M, N] bfloat16, fully overwritten
 * Other shapes: BL_EUNSUPPORTED (run bitlinear_a4 and relu2_glu). */
int bitlinear_a4_up_gated(const void* X, int64_t M, int64_t K, const void* W_rows,
                          const float* alpha, int64_t N, float eps, const void* G,
                          bl_dtype g_dtype, void* H, void* stream);

/* Low-bit attention states (Section 4.2, "Low-bit Attention"; Table 3): each head vector of a token
 * (post-RoPE query, key or value) is quantized on its own with the absmax function to `bits` = 4 or
 * 3 bits and stored as an unsigned integer.  The paper gives one sentence and no formula; the form
 * taken is eq. 3's with Q_b = 2^(bits-1) - 1 levels on each side:
 *     gamma = max|x| over the head;  q = RoundClip(x * (Q_b / (gamma + eps)), -Q_b, Q_b);
 *     code = q + 2^(bits-1), in [1, 2^bits - 1];  scale_out = gamma / Q_b
 * (the value a code stands for is (code - 2^(bits-1)) * scale).  The paper's 3-bit cache keeps the
 * first token's heads at 4 bits: kv_cache_append below writes that mixed-width form.
 *   X          device, [T, H, D] of x_dtype, 16-byte aligned, D % 8 == 0, D <= BL_MAX_K
 *   q_out      device, quantize_heads_bytes(bits, T, H, D) = T * H * D * bits / 8 bytes, 16-byte
 *              aligned: per head D * bits / 8 bytes, heads in [T, H] order; code j of a head in
 *              bits bits*j .. bits*j + bits-1 of the head's little-endian bit stream (4 bits: two
 *              codes per byte, the even channel in the low nibble; 3 bits: eight codes in three bytes)
 *   scale_out  device, float32 [T, H]
 * Errors: BL_EINVAL (null pointer, bits, eps < 0, sizes < 1), BL_ESHAPE (D % 8 != 0 or too large),
 * BL_EALIGN. */
size_t quantize_heads_bytes(int bits, int64_t T, int64_t H, int64_t D);
int quantize_heads(const void* X, bl_dtype x_dtype, int64_t T, int64_t H, int64_t D, int bits, float eps,
                   void* q_out, float* scale_out, void* stream);

/* The value a code of quantize_heads stands for: out = (code - 2^(bits-1)) * scale, one float32
 * multiply (and one rounding to bfloat16 if out_dtype is BL_BF16).
 *   q, scale   the outputs of quantize_heads for [T, H, D] at `bits`
 *   out        device, [T, H, D] of out_dtype, 16-byte aligned */
int dequantize_heads(const void* q, const float* scale, int64_t T, int64_t H, int64_t D, int bits,
                     void* out, bl_dtype out_dtype, void* stream);

/* Key / value cache of one sequence at 3 bits with the first token's heads at 4 bits (Table 3: "4-bit Q,
 * 3-bit KV", the heads of the bos token kept at 4 bits; Section 4.2).  The paper defines no storage
 * format; this one is: the token at position 0 takes H * D / 2 bytes (4-bit codes), every later token
 * H * 3 D / 8 bytes (3-bit codes), tokens in order of position, heads in order inside a token, a head's
 * codes as quantize_heads writes them; the token at position p > 0 starts at byte
 * H * D / 2 + (p - 1) * H * 3 D / 8.  Scales: float32 [positions, H].  D % 32 == 0.
 *   kv_cache_bytes(T, H, D)   bytes of the codes of T positions
 *   kv_cache_append           quantizes X [T, H, D] (the tokens at positions pos0 .. pos0 + T - 1) into
 *                             `cache` and scales[pos0 ..]: position 0 at 4 bits, the others at 3
 *   kv_cache_read             out [T, H, D] = the values of positions pos0 .. pos0 + T - 1 (dequantize_heads'
 *                             arithmetic)
 * cache, X, out 16-byte aligned.  Errors: BL_EINVAL, BL_ESHAPE (D % 32 != 0, sizes), BL_EALIGN. */
size_t kv_cache_bytes(int64_t T, int64_t H, int64_t D);
int kv_cache_append(const void* X, bl_dtype x_dtype, int64_t T, int64_t H, int64_t D, int64_t pos0,
                    float eps, void* cache, float* scales, void* stream);
int kv_cache_read(const void* cache, const float* scales, int64_t pos0, int64_t T, int64_t H, int64_t D,
                  void* out, bl_dtype out_dtype, void* stream);

/* Backward pass of a quantized linear layer under the straight-through estimator (Section 2.2,
 * "Gradient approximation": the quantization functions and the top-K function are passed over).  With
 * the forward pass's dequantized operands Xq[m, k] = scale[m] * q[m, k] (zeros where Top_k masked) and
 * Wq[n, k] = alpha * T[n, k]:
 *     dX[m, k] = sum_n dY[m, n] * Wq[n, k]      (the gradient for X itself: independent of X and of the mask)
 *     dW[n, k] = sum_m dY[m, n] * Xq[m, k]      (the gradient for the full-precision latent weight)
 * Mixed precision: bfloat16 operands on the matrix units, float32 accumulation.  T and q are exact in
 * bfloat16; the one operand rounding is bf16(dY[m, n] * scale[m]) in dW, so each dW[n, k] is within
 * (2^-8 + M 2^-24) * sum_m |dY[m, n] Xq[m, k]| of the exact sum, and dX within N 2^-24 * alpha * sum_n
 * |dY[m, n] T[n, k]| (plus one bfloat16 rounding if dx_dtype is BL_BF16).
 *   dY         device, bfloat16 [M, N], 16-byte aligned (rows of a length that is no multiple of 64 are first
 *              copied to padded rows in the workspace)
 *   q, scale   the codes and scales the forward pass's quantize_act wrote for X [M, K]: mode
 *              BL_ACT_INT4_ABSMEAN (nibble form) or BL_ACT_TOPK_INT8_ABSMAX
 *   W_packed   the layer's weights in BL_W_KMAJOR (other layouts: BL_EUNSUPPORTED), alpha its scale
 *   dX         device [M, K] of dx_dtype, or NULL;  dW  device float32 [N, K], or NULL (overwritten,
 *              not accumulated into); at least one of the two
 *   workspace  bitlinear_backward_workspace_bytes(M, N, K) bytes, 16-byte aligned (the transposed
 *              bfloat16 operands: 2 * (K * Nc + N * Mc + K * Mc) bytes, Nc and Mc rounded up to 64, plus
 *              2 * M * Nc for the padded copy of dY when N % 64 != 0)
 * Errors: BL_EINVAL, BL_ESHAPE, BL_EALIGN, BL_EWORKSPACE, BL_EUNSUPPORTED (mode, layout). */
size_t bitlinear_backward_workspace_bytes(int64_t M, int64_t N, int64_t K);
int bitlinear_backward(const void* dY, int64_t M, int64_t N, int64_t K, const void* q, const float* scale,
                       bl_act_mode mode, const void* W_packed, bl_w_layout layout, const float* alpha,
                       void* dX, bl_dtype dx_dtype, float* dW, void* workspace, size_t workspace_bytes,
                       void* stream);

/* ReLU^2 GLU combine (eq. 5): H = bf16(U * max(G, 0)^2), float32 steps in that order.
 * G, U device [M, N] of in_dtype; H device [M, N] bfloat16. */
int relu2_glu(const void* G, const void* U, bl_dtype in_dtype, int64_t M, int64_t N,
              void* H, void* stream);

/* Swish GLU combine (Section 4.3, the activation squared ReLU is compared with):
 * H = bf16(U * (G * sigmoid(G))), sigmoid(g) = 1 / (1 + exp(-g)) in float32, one bfloat16 rounding;
 * within one bfloat16 ulp of the exactly evaluated function (results below 2^-100 in magnitude:
 * within 2^-100; exp(-g) overflows float32 for g < -88.7 and H is then 0).  Arguments and errors as
 * relu2_glu. */
int swish_glu(const void* G, const void* U, bl_dtype in_dtype, int64_t M, int64_t N,
              void* H, void* stream);

/* eq. 5 followed by eq. 1 / eq. 3 in one pass over G and U: the tokens that are quantized are the
 * rows of H = bf16(U * max(G, 0)^2) as relu2_glu would write them, but H never goes to memory.
 * Outputs as quantize_act with mode BL_ACT_TOPK_INT8_ABSMAX (same formats, bit for bit the same
 * codes as relu2_glu followed by quantize_act).  G, U device [M, K] of in_dtype, 16-byte aligned;
 * K % 4 == 0 and K <= 12288 (the rows are held in registers), otherwise BL_EUNSUPPORTED: then
 * call relu2_glu and quantize_act.  rowsum_out nullable. */
int quantize_act_glu(const void* G, const void* U, bl_dtype in_dtype, int64_t M, int64_t K,
                     int64_t topk, float eps, void* q_out, float* scale_out, int32_t* rowsum_out,
                     void* stream);

/* ---------------------------------------------------------------- format helpers
 * Expand packed data back to one int8 per element so that tests can compare codes
 * without knowing the byte order: T_out int8[N, K]; codes_out int8[M, K] (INT modes)
 * or uint8[M, K] E2M1 nibbles (FP4). */
int unpack_ternary(const void* packed, int64_t N, int64_t K, bl_w_layout layout,
                   int8_t* T_out, void* stream);
int unpack_act(const void* q, bl_act_mode mode, int64_t M, int64_t K, int8_t* codes_out,
               void* stream);

/* Enqueue an empty kernel (one wave that does nothing) on `stream`: what a launch costs on its own,
 * the floor under every figure measured per launch at decode sizes. */
int bl_noop(void* stream);

/* Human-readable name of a status code (host pointer to a static string). */
const char* bl_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* BITLINEAR_H_ */
