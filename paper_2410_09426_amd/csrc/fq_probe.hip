// Measurement aid: the memory traffic of the fused activation kernel without its arithmetic.
// Every token row of 2n bytes is read once with 16-byte non-temporal loads and n/2 bytes are written per row
// (an xor-fold of the row), one 128-thread workgroup per row, workgroups persistent over rows.  bench.py times
// it on the same buffers as the real kernel: what it reaches is the ceiling that launch cost, HBM latency and
// ramp-up leave for a launch of that size on the machine at hand.
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

hipError_t stream_probe_launch(const void* x, int64_t T, int n, int64_t x_stride, uint8_t* out, hipStream_t stream) {
    int64_t grid = (int64_t)cu_count() * 8;
    if (grid > T) grid = T;
    hipLaunchKernelGGL(stream_probe_kernel, dim3((unsigned)grid), dim3(128), 0, stream, static_cast<const u32x4*>(x), T, n / 8,
                       x_stride / 8, reinterpret_cast<u32x4*>(out));
    return hipGetLastError();
}

}  // namespace fq
