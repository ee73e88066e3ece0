// Internal declarations shared by the translation units of libflatquant.
// Nothing here is part of the public ABI (see include/flatquant.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace fq {

constexpr int kTile = 32;          // MFMA tile edge (v_mfma_f32_32x32x16_f16)
constexpr int kMaxN1 = 128;        // up to 4 row tiles
constexpr int kMaxN2 = 256;        // up to 8 column slabs (one wavefront each)
constexpr int kLdsPad = 8;         // halves of padding per LDS row (keeps 16-byte reads off one bank group)

struct TqArgs {
    const _Float16* x;
    const _Float16* P1;
    const _Float16* P2;
    const float* clip;
    int clip_mode;
    int64_t T;
    int n1, n2;
    int64_t x_stride;
    uint8_t* out_codes;
    _Float16* out_scales;
    int mx_tiled = 0;
};

// Kernel-side argument block of the activation kernels.
struct TqDev {
    const _Float16* x;
    const _Float16* P1;
    const _Float16* P2;
    const float* clip;
    uint8_t* out_codes;
    _Float16* out_scales;
    int64_t x_stride;
    int64_t T;
    int n1, n2;
    int clip_mode;
    int vec8;       // rows can be moved in 16-byte chunks that never straddle a row of X~
    int out_vec16;  // code rows are whole 16-byte units at 16-byte aligned addresses
    int mx_tiled = 0;   // MXFP4 output only: exponents in the tile order the MXFP4 product reads (see flatquant.h)
    uint32_t n1_magic = 0;   // floor(2^32 / n1) + 1 (n1 >= 2): floor(f / n1) = umulhi(f, n1_magic) for f < 2^16
    uint32_t n2_magic = 0;   // the same for n2
};

// Specialised kernels for n2 a multiple of 32 and 16-byte aligned buffers (fq_tq_fast.hip).
bool tq_fast_applicable(const TqDev& d);
int64_t tq_fast_lds_bytes(int n1, int n2);
hipError_t tq_fast_launch(const TqDev& d, hipStream_t stream);
// One wavefront per token, rows through a wave-private LDS tile (fq_tq_wave.hip; n2 = 64, n1 = 32 or 64; INT4 or MXFP4).
bool tq_wave_applicable(const TqDev& d);
hipError_t tq_wave_launch(const TqDev& d, hipStream_t stream, int tpw, bool loop, bool mx);
// ... and its left-factor-only sibling for 128-wide rows (P2 == nullptr, n1 = 32 or 64; loop-free).
bool po_wave_applicable(const TqDev& d);
hipError_t po_wave_launch(const TqDev& d, hipStream_t stream);
// MXFP4 output variant of the specialised kernels (d.out_scales points at the u8 [T, n/32] shared exponents).
bool tq_mx_applicable(const TqDev& d);
hipError_t tq_mx_launch(const TqDev& d, hipStream_t stream);
// ... and of the general kernel, for the shapes those do not take (fq_transform_quant.hip).
bool tq_mx_generic_applicable(const TqDev& d);
hipError_t tq_mx_generic_launch(const TqDev& d, hipStream_t stream);
// Fills the kernel-side block from the checked arguments (alignment facts included).
TqDev tq_dev_args(const TqArgs& a);

// LDS bytes of the fused activation kernel for (n1, n2); 0 if unsupported.
int64_t tq_lds_bytes(int n1, int n2);
bool tq_supported(int n1, int n2);
// Enqueue the fused kernel; returns hipSuccess or the launch error.
hipError_t tq_launch(const TqArgs& a, hipStream_t stream);

struct KvArgs {
    const _Float16* kv;
    const _Float16* P;
    int Hp;
    float clip;
    int64_t T;
    int H, D;
    uint8_t* out_codes;
    _Float16* out_scales;
    _Float16* out_zeros;
    bool fp16_out = false;   // transform only: out_codes points at an fp16 [T, H, D] tensor, no steps / zero points
    int bits = 4;            // code width of the quantizing mode: 2, 3 or 4
};
hipError_t kv_launch(const KvArgs& a, hipStream_t stream);

hipError_t dequant_mxfp4_launch(const uint8_t* codes, const uint8_t* exps, int64_t rows, int n, float* out, hipStream_t stream);
hipError_t dequant_bits_launch(const uint8_t* codes, const _Float16* scales, const _Float16* zeros,
                               int64_t rows, int n, int bits, float* out, hipStream_t stream);
hipError_t dequant_launch(const uint8_t* codes, const _Float16* scales, const _Float16* zeros,
                          int64_t rows, int n, float* out, hipStream_t stream);

struct GemmArgs {
    const uint8_t* x_codes;
    const _Float16* x_scales;
    const uint8_t* w_codes;
    const _Float16* w_scales;
    _Float16* out;
    int64_t T;
    int64_t out_stride;
    int m, n;
};
// W4A4 matrix product of the two quantized factors (fq_gemm.hip).
hipError_t w4a4_launch(const GemmArgs& a, hipStream_t stream);

struct MxGemmArgs {
    const uint8_t* x_codes;
    const uint8_t* x_exps;
    const uint8_t* w_codes;
    const uint8_t* w_exps;
    _Float16* out;
    int64_t T;
    int64_t out_stride;
    int m, n;
};
hipError_t mxfp4_gemm_launch(const MxGemmArgs& a, hipStream_t stream);

// Few-token products (fq_gemm.hip, fq_gemm_mx.hip): per wave a ring of LDS slots filled by global-to-LDS loads.
constexpr int kRingMaxDepth = 8;
constexpr int kRingLdsMax = 160 * 1024;
#if defined(__HIP_DEVICE_COMPILE__) || defined(__HIPCC__)
// Every kernel launch of the library goes through here.  The runtime keeps the last error of any earlier call on the
// thread (the caller's own, unrelated ones included) until somebody reads it: it is read and dropped first, so that
// what is returned belongs to this launch.
template <typename... KArgs, typename... Args>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, int lds, hipStream_t stream, Args&&... args) {
    (void)hipGetLastError();
    hipLaunchKernelGGL(kernel, grid, block, lds, stream, static_cast<KArgs>(args)...);
    return hipGetLastError();
}
// until at most N of this wave's vector-memory loads are outstanding (they complete in order)
template <int N>
__device__ __forceinline__ void wait_vm_pending() {
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// until the ring step with `pend` later steps of NI load instructions each in flight has landed
template <int NI>
__device__ __forceinline__ void wait_ring_step(int pend) {
    switch (pend) {
        case 0: wait_vm_pending<0>(); break;
        case 1: if constexpr (NI <= 63) wait_vm_pending<NI>(); else wait_vm_pending<0>(); break;
        case 2: if constexpr (2 * NI <= 63) wait_vm_pending<2 * NI>(); else wait_vm_pending<0>(); break;
        case 3: if constexpr (3 * NI <= 63) wait_vm_pending<3 * NI>(); else wait_vm_pending<0>(); break;
        case 4: if constexpr (4 * NI <= 63) wait_vm_pending<4 * NI>(); else wait_vm_pending<0>(); break;
        case 5: if constexpr (5 * NI <= 63) wait_vm_pending<5 * NI>(); else wait_vm_pending<0>(); break;
        case 6: if constexpr (6 * NI <= 63) wait_vm_pending<6 * NI>(); else wait_vm_pending<0>(); break;
        case 7: if constexpr (7 * NI <= 63) wait_vm_pending<7 * NI>(); else wait_vm_pending<0>(); break;
        default: wait_vm_pending<0>(); break;
    }
}
#endif

// Copy-like probe with the activation kernel's traffic (fq_probe.hip).
hipError_t stream_probe_launch(const void* x, int64_t T, int n, int64_t x_stride, uint8_t* out, hipStream_t stream);

// Launch facts of one kernel, cached per device: the first call on a device raises the kernel's dynamic-LDS limit to
// `lds` bytes and asks the runtime how many workgroups of `threads` threads fit on a CU.  Concurrent first calls
// compute the same value; devices past the table are served without caching.
constexpr int kMaxDevices = 64;
struct OccCache {
    std::atomic<int> per_device[kMaxDevices];
};
hipError_t kernel_occupancy(const void* fn, int threads, int lds, OccCache& cache, int& wg_per_cu);

// Number of compute units of the current device (cached per device).
int cu_count();
// Integer tuning override from the environment (bench / sweep aid); `dflt` if unset.
int env_int(const char* name, int dflt);

}  // namespace fq
