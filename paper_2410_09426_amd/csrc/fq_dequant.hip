// De-quantization check helper: out = s * q (signed nibbles) or s * (q - z)
// (unsigned nibbles), Sec. 2.1.  Plain bandwidth kernel: one thread per 4 code bytes.
#include "fq_internal.h"

namespace fq {

__global__ __launch_bounds__(256) void dequant_kernel(const uint8_t* __restrict__ codes, const _Float16* __restrict__ scales,
                                                       const _Float16* __restrict__ zeros, int64_t rows, int n, float* __restrict__ out) {
    const int nbytes = n >> 1;
    const int units = (nbytes + 3) >> 2;                 // 4-byte units per row (last one may be partial)
    const int64_t total = rows * units;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = g / units;
        const int b0 = (int)(g - r * units) * 4;
        const float s = (float)scales[r];
        const float z = zeros ? (float)zeros[r] : 0.0f;
        const uint8_t* src = codes + r * nbytes;
        float* dst = out + r * (int64_t)n;
        for (int b = b0; b < b0 + 4 && b < nbytes; ++b) {
            const uint32_t v = src[b];
            int lo = v & 15, hi = v >> 4;
            if (!zeros) { lo = (lo ^ 8) - 8; hi = (hi ^ 8) - 8; }   // two's complement nibble -> int
            dst[2 * b] = s * ((float)lo - z);
            dst[2 * b + 1] = s * ((float)hi - z);
        }
    }
}

// Unsigned b-bit codes (b = 2, 3, 4), code k of a row at bits [b k, b k + b) of the row's bytes read little-endian:
// one thread per 8 codes = b bytes.  out = s * (q - z).
__global__ __launch_bounds__(256) void dequant_bits_kernel(const uint8_t* __restrict__ codes, const _Float16* __restrict__ scales,
                                                            const _Float16* __restrict__ zeros, int64_t rows, int n, int bits,
                                                            float* __restrict__ out) {
    const int units = n >> 3;
    const int64_t total = rows * units;
    const uint32_t mask = (1u << bits) - 1u;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = g / units;
        const int u = (int)(g - r * units);
        const float s = (float)scales[r];
        const float z = (float)zeros[r];
        const uint8_t* src = codes + r * ((int64_t)n * bits / 8) + (int64_t)u * bits;
        uint32_t v = 0;
        for (int b = 0; b < bits; ++b) v |= (uint32_t)src[b] << (8 * b);
        float* dst = out + r * (int64_t)n + 8 * u;
        for (int k = 0; k < 8; ++k) dst[k] = s * ((float)((v >> (bits * k)) & mask) - z);
    }
}

// MXFP4: E2M1 nibbles (even channel low) times the block's power-of-two scale 2^(e - 127); one thread per 4 code bytes.
__global__ __launch_bounds__(256) void dequant_mxfp4_kernel(const uint8_t* __restrict__ codes, const uint8_t* __restrict__ exps,
                                                             int64_t rows, int n, float* __restrict__ out) {
    const int units = n >> 3;
    const int64_t total = rows * units;
    for (int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; g < total; g += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = g / units;
        const int u = (int)(g - r * units);
        const uint32_t e = exps[r * (n >> 5) + (u >> 2)];
        const float scale = __builtin_bit_cast(float, e ? e << 23 : 0x00400000u);   // e = 0: 2^-127 (subnormal)
        const uint32_t v = *reinterpret_cast<const uint32_t*>(codes + r * (n >> 1) + 4 * u);
        float* dst = out + r * (int64_t)n + 8 * u;
        for (int k = 0; k < 8; ++k) {
            const uint32_t c = (v >> (4 * k)) & 15u, ex = (c >> 1) & 3u, m = c & 1u;
            const float mag = ex ? (float)(1u << (ex - 1)) * (1.0f + 0.5f * (float)m) : 0.5f * (float)m;
            dst[k] = (c & 8u) ? -(mag * scale) : mag * scale;
        }
    }
}

hipError_t dequant_mxfp4_launch(const uint8_t* codes, const uint8_t* exps, int64_t rows, int n, float* out, hipStream_t stream) {
    const int64_t total = rows * (n >> 3);
    int64_t grid = (total + 255) / 256;
    const int64_t cap = (int64_t)cu_count() * 16;
    if (grid > cap) grid = cap;
    if (grid < 1) grid = 1;
    return launch(dequant_mxfp4_kernel, dim3((unsigned)grid), dim3(256), 0, stream, codes, exps, rows, n, out);
}

hipError_t dequant_bits_launch(const uint8_t* codes, const _Float16* scales, const _Float16* zeros,
                               int64_t rows, int n, int bits, float* out, hipStream_t stream) {
    const int64_t total = rows * (n >> 3);
    int64_t grid = (total + 255) / 256;
    const int64_t cap = (int64_t)cu_count() * 16;
    if (grid > cap) grid = cap;
    if (grid < 1) grid = 1;
    return launch(dequant_bits_kernel, dim3((unsigned)grid), dim3(256), 0, stream, codes, scales, zeros, rows, n, bits, out);
}

hipError_t dequant_launch(const uint8_t* codes, const _Float16* scales, const _Float16* zeros,
                          int64_t rows, int n, float* out, hipStream_t stream) {
    const int units = ((n >> 1) + 3) >> 2;
    const int64_t total = rows * units;
    int64_t grid = (total + 255) / 256;
    const int64_t cap = (int64_t)cu_count() * 16;
    if (grid > cap) grid = cap;
    if (grid < 1) grid = 1;
    return launch(dequant_kernel, dim3((unsigned)grid), dim3(256), 0, stream, codes, scales, zeros, rows, n, out);
}

}  // namespace fq
