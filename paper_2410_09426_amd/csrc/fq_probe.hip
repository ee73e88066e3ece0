// Measurement aid: the memory traffic of the fused activation kernel without its arithmetic.
// Every token row of 2n bytes is read once with 16-byte non-temporal loads and n/2 bytes are written per row
// (an xor-fold of the row).  Three launch shapes (see stream_probe_launch); the benchmark times all of them on the
// same buffers as the real kernel and takes the best: what a copy-like launch of that size reaches on the machine at
// hand, i.e. the ceiling that launch cost, HBM latency and ramp-up leave.
#include "fq_internal.h"

namespace fq {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(128) void stream_probe_kernel(const u32x4* __restrict__ x, int64_t T, int chunks, int64_t stride16,
                                                            u32x4* __restrict__ out) {
    const int out_chunks = chunks >> 2;   // n/2 bytes = a quarter of the row
    for (int64_t t = blockIdx.x; t < T; t += gridDim.x) {
        const u32x4* row = x + t * stride16;
        u32x4* dst = out + t * out_chunks;
        for (int q0 = 0; q0 < out_chunks; q0 += 128) {
            const int q = q0 + threadIdx.x;
            if (q < out_chunks) {
                const u32x4 a = __builtin_nontemporal_load(row + q), b = __builtin_nontemporal_load(row + q + out_chunks);
                const u32x4 c = __builtin_nontemporal_load(row + q + 2 * out_chunks), d = __builtin_nontemporal_load(row + q + 3 * out_chunks);
                __builtin_nontemporal_store(a ^ b ^ c ^ d, dst + q);
            }
        }
    }
}

// Second shape: one wave per row, the loads of a pass (8 or 16 per lane) all in flight before the first is used, no
// persistence: the hardware hands out workgroups of four rows.  PLAIN: ordinary loads instead of non-temporal ones.
template <bool PLAIN, int NL>
__global__ __launch_bounds__(256) void stream_probe_rows_kernel(const u32x4* __restrict__ x, int64_t T, int chunks, int64_t stride16,
                                                                 u32x4* __restrict__ out) {
    const int l = threadIdx.x & 63;
    int64_t t = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (t >= T) t = T - 1;                 // spare waves redo the last row: same bytes stored again
    const u32x4* row = x + t * stride16;
    u32x4* dst = out + t * (chunks >> 2);
    for (int q0 = 0; q0 < chunks; q0 += 64 * NL) {   // NL loads per lane and pass; a pass yields NL / 4 output units per lane
        u32x4 v[NL];
#pragma unroll
        for (int k = 0; k < NL; ++k) {
            const int q = q0 + 64 * k + l;
            const u32x4* p = row + (q < chunks ? q : chunks - 1);
            v[k] = PLAIN ? *p : __builtin_nontemporal_load(p);
        }
#pragma unroll
        for (int k = 0; k < NL / 4; ++k) {
            const int q = (q0 >> 2) + 64 * k + l;
            if (q < (chunks >> 2)) __builtin_nontemporal_store(v[4 * k] ^ v[4 * k + 1] ^ v[4 * k + 2] ^ v[4 * k + 3], dst + q);
        }
    }
}

// shape (tuning knob FLATQUANT_PROBE_SHAPE): 0 persistent two-wave workgroups, 1 a wave per row, 2 the same with plain loads
hipError_t stream_probe_launch(const void* x, int64_t T, int n, int64_t x_stride, uint8_t* out, hipStream_t stream) {
    const int shape = env_int("FLATQUANT_PROBE_SHAPE", 0);
    if (shape == 1 || shape == 2) {
        if (T > 0x7fffffff) return hipErrorInvalidConfiguration;
        const unsigned grid = (unsigned)((T + 3) / 4);
        const bool small = (n / 8) % 1024 != 0 && (n / 8) % 512 == 0;   // rows of a whole number of 8-load passes (n = 4096)
        auto fn = shape == 1 ? (small ? &stream_probe_rows_kernel<false, 8> : &stream_probe_rows_kernel<false, 16>)
                             : (small ? &stream_probe_rows_kernel<true, 8> : &stream_probe_rows_kernel<true, 16>);
        return launch(fn, dim3(grid), dim3(256), 0, stream, static_cast<const u32x4*>(x), T, n / 8, x_stride / 8, reinterpret_cast<u32x4*>(out));
    }
    int64_t grid = (int64_t)cu_count() * 8;
    if (grid > T) grid = T;
    return launch(stream_probe_kernel, dim3((unsigned)grid), dim3(128), 0, stream, static_cast<const u32x4*>(x), T, n / 8,
                       x_stride / 8, reinterpret_cast<u32x4*>(out));
}

}  // namespace fq
