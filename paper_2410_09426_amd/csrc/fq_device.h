// Device-side helpers shared by the kernels of libflatquant (gfx950 only; not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}

// max over the 64 lanes of a wave; every lane returns the result
__device__ __forceinline__ float wave_max(float x) {
    x = __builtin_fmaxf(x, dpp_move<0xB1>(x));    // quad_perm [1,0,3,2]
    x = __builtin_fmaxf(x, dpp_move<0x4E>(x));    // quad_perm [2,3,0,1]
    x = __builtin_fmaxf(x, dpp_move<0x141>(x));   // row_half_mirror
    x = __builtin_fmaxf(x, dpp_move<0x140>(x));   // row_mirror: every lane of a 16-lane row holds the row max
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 48));
    return __builtin_fmaxf(__builtin_fmaxf(r0, r1), __builtin_fmaxf(r2, r3));
}

// z - (float)half(hi or lo 16 bits of `packed`), in one mixed-precision fma (the fp16 operand is read in place)
template <int HI>
__device__ __forceinline__ float sub_half(float z, unsigned int packed) {
    float r;
    if constexpr (HI) asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(z));
    else asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(z));
    return r;
}

// fp32 x8 -> fp16 hi (round toward zero, cannot overflow to inf) and fp16 lo = fp16(z - hi).
// (Writing the residual with v_fma_mixlo_f16 / v_fma_mixhi_f16 saves one instruction per pair, but the two
// half-register writes need a wait state between them on gfx950 (without it, a single wave per SIMD gets wrong
// residuals), and with the wait states the kernel measured slower than this form.)
__device__ __forceinline__ void split_hi_lo(const f32x16& acc, int base, half8& hi, half8& lo) {
    u32x4 h, l;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float z0 = acc[base + 2 * k], z1 = acc[base + 2 * k + 1];
        const unsigned int ph = __builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_pkrtz(z0, z1));
        h[k] = ph;
        l[k] = __builtin_bit_cast(unsigned int, __builtin_amdgcn_cvt_pkrtz(sub_half<0>(z0, ph), sub_half<1>(z1, ph)));
    }
    hi = __builtin_bit_cast(half8, h);
    lo = __builtin_bit_cast(half8, l);
}

// (a << sh) + b in one instruction (the compiler otherwise re-associates the nibble chain into more operations)
__device__ __forceinline__ uint32_t lshl_add(uint32_t a, int sh, uint32_t b) {
    uint32_t r;
    asm("v_lshl_add_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "n"(sh), "v"(b));
    return r;
}

// Eight fp16 values of one column of a row-major fp16 matrix in LDS, rows r0..r0+3 and r0+gap..r0+gap+3, for every
// lane: two transposing LDS reads (ds_read_b64_tr_b16).  Within each block of 16 lanes, lane s supplies the address
// of a 64-bit chunk and lane i receives element i%4 of the chunks supplied by lanes i/4, 4 + i/4, 8 + i/4, 12 + i/4
// (measured on gfx950).  So lane s points at row r0 + s/4, columns col0 + 4(s%4).., and lane i ends up with rows
// r0..r0+3 of column col0 + i.  `lane16` = lane % 16; `col0` is the first column of the lane's 16-lane block.
// SWAP12: lane s points at column chunk swap12(s % 4) instead (chunks of 4 columns, 1 and 2 exchanged), so lane i ends
// up with column col0 + 4 swap12(i / 4) + i % 4.
template <bool SWAP12 = false>
__device__ __forceinline__ half8 lds_column8(const _Float16* m, int pitch, int r0, int gap, int col0, int lane16) {
    const int ch = lane16 & 3, chs = SWAP12 ? (((ch & 1) << 1) | (ch >> 1)) : ch;
    const _Float16* a0 = m + (r0 + (lane16 >> 2)) * pitch + col0 + 4 * chs;
    typedef short4v __attribute__((address_space(3))) * lds_ptr;
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(a0));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(a0 + gap * pitch));
    typedef short short8v __attribute__((ext_vector_type(8)));
    const short8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(half8, v);
}

}  // namespace fq
