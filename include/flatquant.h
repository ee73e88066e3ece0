/*
 * flatquant.h -- C ABI of the MI355X (gfx950) FlatQuant online path.
 *
 * The library fuses, in one kernel launch per call and with no intermediate
 * trip through device memory, the per-token Kronecker affine transform and the
 * low-bit quantization that FlatQuant runs in front of every quantized linear
 * layer (Sec. 3.1 "Kronecker Product", Eq. (2); Sec. 3.3 "Efficient Kernel
 * Design"; App. "Detailed Design of Kernel Fusion").
 *
 * General rules for every entry point
 *   - All data pointers are DEVICE pointers unless a comment says "host".
 *   - The caller owns every buffer.  The library allocates nothing and never
 *     synchronises: work is enqueued on `stream` (a hipStream_t passed as
 *     void*; NULL is the default stream) and outputs are valid once the stream
 *     reaches that point.
 *   - State the library keeps: a thread-local last-HIP-error code
 *     (fq_last_hip_error), per-device launch facts cached on first use (number
 *     of compute units, workgroups per compute unit of each kernel), and the
 *     process-wide tuning overrides of fq_set_tuning (launch-shape choices for
 *     measurements and tests; they never change results).  Nothing else:
 *     calls are independent and may come from several threads at once.
 *   - Two entry points are measurement aids and not part of the method:
 *     flatquant_stream_probe (the activation kernel's memory traffic without
 *     its arithmetic) and fq_set_tuning.
 *   - Inputs are never modified.  Inputs and outputs must not overlap.
 *   - Errors are reported through the return value only (no abort, no output).
 *     On any error nothing is launched and no output byte is written.
 *   - fp16 means IEEE binary16 bit patterns.
 */
#ifndef FLATQUANT_H_
#define FLATQUANT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int fq_status;
enum {
    FQ_OK = 0,
    FQ_INVALID_ARG = 1,       /* null pointer, negative size, odd n1*n2, bad mode, stride < n */
    FQ_UNSUPPORTED_SHAPE = 2, /* no kernel variant for this (n1, n2) / (H, D); see fq_supported() */
    FQ_MISALIGNED = 3,        /* a pointer or stride violates the alignment stated below */
    FQ_LAUNCH_FAILED = 4      /* the HIP runtime refused the launch; see fq_last_hip_error() */
};

/*
 * Activation path:  Q( P1^T x_1 X~ x_2 P2 )  ==  Q( X (P1 (x) P2) )
 * (Eq. (2), left factor; Sec. 3.3).  For every token row x_t of width
 * n = n1*n2, viewed row-major as X~_t (n1 x n2, channel c = i*n2 + j):
 *     Y_t = P1^T X~_t P2
 *     s_t = fp16( clip_t * max_c |Y_t[c]| / 7 )            (Sec. 3.1 "Learnable Clipping Thresholds",
 *     q_t[c] = clamp( round_half_even( Y_t[c] / s_t ), -8, 7 )   Sec. 4.1 "Quantization": per-token symmetric)
 * A row whose step rounds to zero gets step +0 and all-zero codes.
 *
 *   x          fp16 [T, n], row t starts at x + t*x_stride halves; x_stride >= n.
 *              Alignment: 4 bytes (base and row pitch, i.e. x_stride even).
 *   P1         fp16 [n1, n1] row-major, NOT transposed (the kernel applies P1^T).
 *   P2         fp16 [n2, n2] row-major.
 *              Either may be NULL and then stands for the identity: the one-sided transforms of Sec. 3.2, e.g. the
 *              online part of P_o once its per-head factor is fused into the value projection (n1 = heads, n2 =
 *              head_dim, P2 = NULL).  Both NULL gives plain per-token INT4 quantization of x.
 *   clip       fp32; clip_mode 0: one value shared by all tokens (the paper's
 *              layer-wise threshold); clip_mode 1: T values, one per token.
 *              Values are the thresholds after the sigmoid, expected in (0, 1].
 *   out_codes  u8 [T, n/2] contiguous; byte k of a row = (q[2k] & 15) | (q[2k+1] & 15) << 4,
 *              two's-complement nibbles.  Alignment: 4 bytes.
 *   out_scales fp16 [T].
 * T == 0 returns FQ_OK without launching.  n1*n2 must be even, 1 <= n1 <= 128,
 * 2 <= n2 <= 256 and n2 even (fq_supported).  The result is defined while x, the
 * intermediate X~ P2 and Y stay finite in fp16 range (|.| < 65504).
 */
fq_status flatquant_transform_quant(const void* x, const void* P1, const void* P2,
                                    const float* clip, int clip_mode,
                                    int64_t T, int n1, int n2, int64_t x_stride,
                                    uint8_t* out_codes, void* out_scales, void* stream);

/*
 * The same transform with MXFP4 output, the data type the paper's "Limitations" name as the next one to combine with
 * the method (the paper defines nothing for it; the format is the published OCP Microscaling one).  Per token row and
 * per block of 32 consecutive channels c = 32 b .. 32 b + 31 of Y = P1^T X~ P2 (flattened row-major as above):
 *     e  = clamp( floor(log2( clip * max|y_block| )) - 2 + 127, 0, 254 )    shared scale 2^(e - 127), stored as e (E8M0);
 *                                                                            an all-zero block stores e = 0
 *     q  = E2M1( y / 2^(e - 127) )   nearest of +-{0, 0.5, 1, 1.5, 2, 3, 4, 6}, ties to the even code, saturating,
 *                                    code = sign << 3 | magnitude index (a negative value that rounds to zero is -0)
 *   out_codes  u8 [T, n/2], even channel in the low nibble, 16-byte aligned.
 *   out_scales u8 [T, n/32], 4-byte aligned.
 * Shapes: n1 <= 128, n2 even and <= 256, n a multiple of 32.  With n2 a multiple of 32 and n a multiple of 128 a block is
 * 32 consecutive channels inside one row of X~ and the specialised kernels run; any other such shape (64 x 172: a block
 * straddles two rows of X~) goes through the general kernel, which stages the token's Y in LDS as fp32 and needs
 * 4 n + 64 (n1 + 31) / 32 * ((n2 + 31) / 32 * 32 + 8) bytes of it beside P1's fragments: FQ_UNSUPPORTED_SHAPE beyond 160 KB
 * (n above about 24000).  x 16-byte aligned with x_stride a multiple of 8; P1 4-byte and P2 16-byte aligned, both required.  Other arguments, T == 0 and error behaviour as for flatquant_transform_quant.
 */
fq_status flatquant_transform_mxfp4(const void* x, const void* P1, const void* P2,
                                    const float* clip, int clip_mode,
                                    int64_t T, int n1, int n2, int64_t x_stride,
                                    uint8_t* out_codes, uint8_t* out_scales, void* stream);

/*
 * The same, with the exponents written in the tile order that flatquant_mxfp4_gemm reads: rows (tokens) in tiles of
 * 128, channels in groups of 256 (8 exponents); for tile r/128 and group j the 128 rows' 8 bytes are contiguous:
 *     byte of (row r, block k)  =  ( ((r / 128) * (n / 256) + k / 8) * 128 + r % 128 ) * 8 + k % 8.
 * out_scales must hold fq_mxfp4_tiled_scale_bytes(T, n) bytes (rows padded to a multiple of 128; the padding is not
 * written) and be 16-byte aligned; n must also be a multiple of 256.  Codes and everything else as above.
 */
fq_status flatquant_transform_mxfp4_tiled(const void* x, const void* P1, const void* P2,
                                          const float* clip, int clip_mode,
                                          int64_t T, int n1, int n2, int64_t x_stride,
                                          uint8_t* out_codes, uint8_t* out_scales, void* stream);

/* Bytes of a tile-ordered exponent tensor for `rows` rows of n channels (0 if n is not a multiple of 256). */
int64_t fq_mxfp4_tiled_scale_bytes(int64_t rows, int64_t n);

/*
 * KV-cache path (Sec. 3.2 "Self-Attention": P_h / P_v applied head by head,
 * not decomposed; Sec. 4.1: group-wise asymmetric INT4, group = head_dim).
 * For every (token, head) group g of D values:
 *     y  = kv_g P_h
 *     mx = clip * max(max y, 0),  mn = clip * min(min y, 0)
 *     s  = fp16( (mx - mn) / 15 ),  z = clamp( round_half_even( -mn / s ), 0, 15 )
 *     q[d] = clamp( round_half_even( y[d] / s ) + z, 0, 15 )
 *
 *   kv         fp16 [T, H, D] contiguous, 16-byte aligned.  D must be 128.
 *   P          fp16 [Hp, D, D] row-major; Hp == 1 (one matrix shared by all
 *              heads: the groups are then read as T*H consecutive rows, which is
 *              the faster of the two) or Hp == H (one per head).
 *   out_codes  u8 [T, H, D/2], unsigned nibbles, even channel in the low nibble; 16-byte aligned.
 *   out_scales fp16 [T, H];  out_zeros fp16 [T, H] holding the integer z.
 */
fq_status flatquant_kv_transform_quant(const void* kv, const void* P, int Hp, float clip,
                                       int64_t T, int H, int D,
                                       uint8_t* out_codes, void* out_scales, void* out_zeros,
                                       void* stream);

/*
 * The same with b-bit codes, b = bits in {2, 3, 4} (App. "KV Cache Quantization", the tables over key and value bit
 * widths: the group-wise asymmetric grid of Sec. 4.1 with 2^b levels, Omega(b) = {0 .. 2^b - 1} of Sec. 2.1):
 *     s = fp16( (mx - mn) / (2^b - 1) ),  z = clamp( round_half_even( -mn / s ), 0, 2^b - 1 ),
 *     q[d] = clamp( round_half_even( y[d] / s ) + z, 0, 2^b - 1 ).
 *   out_codes  u8 [T, H, D*b/8]: code d of a group at bits [b d, b d + b) of the group's D*b/8 bytes read as one
 *              little-endian integer (b = 4: the nibble layout above; b = 2: four codes per byte, lowest channel in
 *              the lowest bits; b = 3: eight codes per three bytes).  16-byte aligned.
 * Everything else as for flatquant_kv_transform_quant, which is this call with bits = 4.  Keys and values may use
 * different widths: one call per tensor.
 */
fq_status flatquant_kv_transform_quant_bits(const void* kv, const void* P, int Hp, float clip, int bits,
                                            int64_t T, int H, int D,
                                            uint8_t* out_codes, void* out_scales, void* out_zeros,
                                            void* stream);

/*
 * Per-head transform with fp16 output (Sec. 3.2 "Self-Attention": P_h acts head by head and is not decomposed;
 * queries stay in FP16).  out[t, h, :] = fp16( x[t, h, :] P_h ), fp32 accumulation, one rounding.  With the key cache
 * stored as Q(K P_h) the scores are kept by feeding the queries through this call with P = (P_h^-1)^T
 * (fq_inverse_transpose, head by head).
 *   x, out  fp16 [T, H, D] contiguous, 16-byte aligned, not overlapping.  D must be 128.
 *   P       fp16 [Hp, D, D] row-major, Hp == 1 or Hp == H.
 */
fq_status flatquant_head_transform(const void* x, const void* P, int Hp, int64_t T, int H, int D, void* out, void* stream);

/*
 * Weight side of the same layer (Eq. (2), right factor; Sec. 4.1 "Quantization": per-channel symmetric weights):
 *     Q( P1^-1 x_1 W~ x_2 (P2^-1)^T )   ==   Q( W (P1 (x) P2)^-T ),   one step per output channel.
 * Row o of W (width n = n1*n2, reshaped row-major to n1 x n2) becomes A1^T W~_o A2 with A1 = (P1^-1)^T and
 * A2 = (P2^-1)^T, then is quantized like a token row: this is flatquant_transform_quant applied to the weight matrix
 * with the inverse-transposed factors (fq_inverse_transpose builds them on the host), `m` output channels in the role
 * of tokens and the weight clipping ratio(s) in `clip`.  Run once, offline; layouts, alignment and errors as above.
 *   w          fp16 [m, n], row stride w_stride halves.      A1 fp16 [n1, n1], A2 fp16 [n2, n2] row-major.
 *   out_codes  u8 [m, n/2];  out_scales fp16 [m] (one step per output channel).
 * The product of flatquant_dequant(activation codes) and flatquant_dequant(weight codes)^T replaces X W^T (Eq. (1)).
 */
fq_status flatquant_weight_transform_quant(const void* w, const void* A1, const void* A2,
                                           const float* clip, int clip_mode,
                                           int64_t m, int n1, int n2, int64_t w_stride,
                                           uint8_t* out_codes, void* out_scales, void* stream);

/*
 * W4A4 matrix product of the two quantized factors (Sec. 3.2: low-bit matrix multiplications for all linear layers;
 * Eq. (1)-(2)):   out[t, o] = fp16( s_x[t] * s_w[o] * sum_k q_x[t, k] * q_w[o, k] ),
 * exact integer accumulation (int8 MFMA on the widened codes), two fp32 multiplications, one rounding to fp16.
 *   x_codes  u8 [T, n/2], x_scales fp16 [T]   : outputs of flatquant_transform_quant
 *   w_codes  u8 [m, n/2], w_scales fp16 [m]   : outputs of flatquant_weight_transform_quant
 *   out      fp16 [T, m], row t at out + t*out_stride halves, out_stride >= m.
 * n must be a multiple of 256 (and <= 65536, so that the int32 sums cannot overflow); code tensors 16-byte aligned.  T == 0 or m == 0 returns FQ_OK.
 * Values beyond the fp16 range come out as infinities.
 */
fq_status flatquant_w4a4_gemm(const uint8_t* x_codes, const void* x_scales, const uint8_t* w_codes, const void* w_scales,
                              int64_t T, int m, int n, void* out, int64_t out_stride, void* stream);

/*
 * Matrix product of two MXFP4 factors (the same low-bit multiplication for the MXFP4 data type), on the scaled FP4
 * matrix instruction of gfx950:   out[t, o] = fp16( sum_k x^[t, k] * w^[o, k] ),
 * x^ and w^ the de-quantized factors (E2M1 element times 2^(e - 127) of its block of 32 channels); products are exact,
 * the sum is accumulated in fp32 and rounded once to fp16.
 *   x_codes u8 [T, n/2], x_scales tile-ordered exponents  : outputs of flatquant_transform_mxfp4_tiled
 *   w_codes u8 [m, n/2], w_scales tile-ordered exponents  : the same call on the weight rows with the inverse-transposed factors
 *   out     fp16 [T, m], row t at out + t*out_stride halves, out_stride >= m.
 * n must be a multiple of 256; code and exponent tensors 16-byte aligned; the exponent tensors hold
 * fq_mxfp4_tiled_scale_bytes(T or m, n) bytes (the rows of the padding are read and ignored).  T == 0 or m == 0
 * returns FQ_OK.  Values beyond the fp16 range come out as infinities.  The order of the fp32 additions belongs to the
 * kernel the library picks for (T, m, n) on the device at hand (K split over the waves of a workgroup for few tokens,
 * K in sequence for many): the same call gives the same bits every time, two different T need not agree in the last
 * bit of a row they share.  (The INT4 product sums integers and has no such dependence.)
 */
fq_status flatquant_mxfp4_gemm(const uint8_t* x_codes, const uint8_t* x_scales, const uint8_t* w_codes, const uint8_t* w_scales,
                               int64_t T, int m, int n, void* out, int64_t out_stride, void* stream);

/*
 * De-quantization check helper (Sec. 2.1: W^ = s * Pi(W / s)).
 *   zeros == NULL : out[r, c] = s[r] * q[r, c]            (signed nibbles)
 *   zeros != NULL : out[r, c] = s[r] * (q[r, c] - z[r])   (unsigned nibbles)
 *   codes u8 [rows, n/2]; scales, zeros fp16 [rows]; out fp32 [rows, n]; n even.
 */
fq_status flatquant_dequant(const uint8_t* codes, const void* scales, const void* zeros,
                            int64_t rows, int n, float* out, void* stream);

/*
 * The same for the output of flatquant_transform_mxfp4: out[r, c] = E2M1 value of code (r, c) times 2^(e[r, c/32] - 127).
 *   codes u8 [rows, n/2] (4-byte aligned), scales u8 [rows, n/32], out fp32 [rows, n]; n a multiple of 32.
 */
fq_status flatquant_dequant_mxfp4(const uint8_t* codes, const uint8_t* scales, int64_t rows, int n, float* out, void* stream);

/*
 * The same for unsigned b-bit codes in the layout of flatquant_kv_transform_quant_bits (bits in {2, 3, 4}):
 *   out[r, c] = s[r] * (q[r, c] - z[r]);  codes u8 [rows, n*bits/8]; zeros required; n a multiple of 8.
 */
fq_status flatquant_dequant_bits(const uint8_t* codes, const void* scales, const void* zeros,
                                 int64_t rows, int n, int bits, float* out, void* stream);

/*
 * Measurement aid (not part of the method): moves the bytes of flatquant_transform_quant without its arithmetic.
 * Reads every row of x once (fp16 [T, n], x_stride halves apart) and writes n/2 bytes per row to out ([T, n/2],
 * an xor-fold of the row, contents meaningless) with 16-byte accesses, in one of three launch shapes (tuning override
 * FLATQUANT_PROBE_SHAPE: 0 persistent two-wave workgroups, one row at a time; 1 one wave per row, every load of the
 * row in flight at once; 2 the same with ordinary instead of non-temporal loads).  Requires n % 32 == 0, x and out
 * 16-byte aligned, x_stride % 8 == 0.  The fastest shape's time is the ceiling that launch cost and memory latency
 * leave for a copy-like launch of that size on this machine.
 */
fq_status flatquant_stream_probe(const void* x, int64_t T, int n, int64_t x_stride, uint8_t* out, void* stream);

/* ---- host-only helpers: no GPU is touched ---------------------------------- */

/* 1 if flatquant_transform_quant has a kernel variant for (n1, n2), else 0. */
int fq_supported(int n1, int n2);

/* The paper's factor rule (Sec. 3.1): argmin (n1 + n2) s.t. n1*n2 == n, n1 <= n2.
 * n < 1 leaves the outputs untouched and returns FQ_INVALID_ARG.  Host pointers. */
fq_status fq_choose_factors(int64_t n, int* n1, int* n2);

/* Host helper for the weight side: out = fp16( (P^-1)^T ) for a square fp16 matrix P [n, n] (host pointers, row-major,
 * 1 <= n <= 256), inverted in fp64 by Gauss-Jordan elimination with partial pivoting and rounded once.  If
 * `max_residual` is not NULL it receives max |P^T out - I| of the rounded result, in fp64.  Returns FQ_INVALID_ARG
 * for null pointers, n out of range or a singular matrix (a pivot below 1e-12 times the largest entry). */
fq_status fq_inverse_transpose(const void* P, int n, void* out, double* max_residual);

/* On-chip footprint test of App. "Detailed Design of Kernel Fusion": returns 1
 * when (n1*n1 + 2*n1*n2)*2 < m and (n2*n2 + 2*n1*n2)*2 < m for m bytes of
 * on-chip memory per workgroup (the paper's "default design" condition). */
int fq_default_design_fits(int n1, int n2, int64_t m_bytes);

/* LDS bytes the fused kernel of this library requests for (n1, n2); 0 if unsupported. */
int64_t fq_lds_bytes(int n1, int n2);

const char* fq_status_string(fq_status s);

/* hipError_t of the most recent failed launch on this thread (0 if none). */
int fq_last_hip_error(void);

/* Library version, bumped when the ABI changes. */
int fq_abi_version(void);

/*
 * Tuning overrides, for measurements and tests (the defaults are what the library measures best).  `name` is one of
 * FLATQUANT_MODE (activation kernel flavour: 0..4 the slab kernels, 5 / 6 the wave-per-token kernel of 64-wide rows, one
 * shot / persistent; 5 also forces the wave-per-token kernel of the left-factor-only case), FLATQUANT_WAVE_TPW (2 / 4 / 8 waves per workgroup of that kernel), FLATQUANT_PROBE_SHAPE (0..2: launch
 * shape of flatquant_stream_probe), FLATQUANT_WG_PER_CU, FLATQUANT_KV_WG_PER_CU (cap on resident
 * workgroups), FLATQUANT_FORCE_GENERIC (1: general kernel on shapes the specialised ones would take),
 * FLATQUANT_GEMM_TILED (1: tiled product for any T), FLATQUANT_GEMM_WIDE (0 / 1: 128- or 256-token tiles),
 * FLATQUANT_GEMM_ROWS (16 / 32 output channels per workgroup), FLATQUANT_GEMM_WAVES (4 / 8 / 16) and
 * FLATQUANT_GEMM_DEPTH (1..8 line slots per wave) of the few-token products, FLATQUANT_GEMM_RING_MAX_T (token count up to
 * which the few-token kernel is used), FLATQUANT_KV_FOLD_HEADS (0: a shared P_h is applied head by head like separate
 * ones).  enable != 0 sets the override to `value`, enable == 0 removes it.  Each override starts from the environment variable of the same name, read once per process.
 * Process-wide; affects launches issued after the call returns.  Unknown names return FQ_INVALID_ARG.
 */
fq_status fq_set_tuning(const char* name, int value, int enable);

#ifdef __cplusplus
}
#endif
#endif /* FLATQUANT_H_ */
