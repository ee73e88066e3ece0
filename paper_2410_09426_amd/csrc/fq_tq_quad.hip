// Fused transform + INT4 kernel for 64 x 64 tokens (n1 = n2 = 64): four wavefronts per token, a workgroup of four
// waves takes its tokens one after the other.
//
// Same method as the other activation kernels (Eq. (2) left factor, fused as in Sec. 3.3: Z = X~ P2, Y^T = Z^T P1 with Z
// split into fp16 hi + lo, per-token absmax, clip, round, pack).  What this kernel is built around is the end of a
// short launch (T = 2048: eight tokens per CU): the rows of a CU arrive over 2 - 3 us in the order they were requested,
// and what is left to do when the last of them arrives is what the launch waits for.  So
//   * the four waves of a workgroup request their tokens together, token by token (two 16-byte loads per lane and
//     token): the tokens of a workgroup arrive one after the other, not all at once at the end;
//   * each token is split over the four waves (slab q of P2's columns x row tile It of X~), one per SIMD, so that the
//     work on the token that arrives last is a quarter of a token per SIMD:
//       wave (q, It):  Z[It, q] = X~[It rows, :] P2[:, slab q]            4 MFMAs
//                      split into hi + lo, handed to wave (q, 1 - It) through LDS
//                      Y^T[slab q, tile It] = sum over both row tiles Z[., q]^T P1[., tile It]   8 MFMAs
//     with no MFMA done twice;
//   * three workgroup barriers per token (tile written / hi + lo parts exchanged / absmax exchanged), among four waves.
// Rounding, packing and stores as in the wave-per-token kernel (v_cvt_pknorm_i16_f32 puts clamp(rne(y / s), -8, 7) in
// the top nibble of a 16-bit field; one v_permlane32_swap gives each lane 8 contiguous bytes of its row).
#include "fq_internal.h"
#include "fq_device.h"

namespace fq {

// NTOK: tokens per workgroup.  The launch gives every workgroup NTOK consecutive tokens (the last one may re-do token
// T - 1 in its spare rounds: the same bytes are stored again).
template <int NTOK>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void tq_quad_kernel(
    const _Float16* __restrict__ P2, const _Float16* __restrict__ P1, const _Float16* __restrict__ x, int64_t x_stride, int64_t T,
    const float* __restrict__ clip, uint8_t* __restrict__ out_codes, _Float16* __restrict__ out_scales, int clip_mode) {
    // (plain arguments in the order they are needed, so that the first ones can be delivered in registers at wave start)
    constexpr int N = 64, KB = 4;                    // n1 = n2 = 64; K blocks of 16 per contraction
    constexpr int TILE_BYTES = N * N * 2;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    _Float16* P2flat = reinterpret_cast<_Float16*>(smem);             // prologue: P2, P1 row-major
    _Float16* P1flat = P2flat + N * N;
    u32x4* zbuf = reinterpret_cast<u32x4*>(smem);                     // afterwards: hi / lo parts, [wave][4][lane]
    unsigned char* tiles = smem + 2 * TILE_BYTES;
    float* red = reinterpret_cast<float*>(tiles + NTOK * TILE_BYTES); // [2][4] absmax partials

    const int tid = threadIdx.x;
    const int l = tid & 63, c = l & 31, h = l >> 5;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = w & 1, It = w >> 1;
    const int64_t t0 = (int64_t)blockIdx.x * NTOK;

    // ---- requests: the transforms first (L2), then the tokens (HBM), token by token
    u32x4 pv[4];
#pragma unroll
    for (int k = 0; k < 4; ++k)
        pv[k] = reinterpret_cast<const u32x4*>(k < 2 ? P2 : P1)[tid + 256 * (k & 1)];
    // Thread tid brings 16-byte units tid and tid + 256 of a token: row r = tid / 8 (+ 32), and of that row the chunk
    // (tid % 8) ^ ((r >> 1) & 7), which goes to LDS slot tid % 8 of the row: with that swizzle the 16-byte operand reads
    // of 32 consecutive rows (same chunk) spread over all banks although the pitch is a multiple of the bank width.
    const int ld_ofs = (tid >> 3) * (N * 2) + 16 * ((tid & 7) ^ ((tid >> 4) & 7));
    u32x4 pre[NTOK][2];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < NTOK; ++j) {
        const int64_t tok = t0 + j < T ? t0 + j : T - 1;
        const unsigned char* row = reinterpret_cast<const unsigned char*>(x + tok * x_stride) + ld_ofs;
        pre[j][0] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row));
        pre[j][1] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row + 32 * N * 2));
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- transforms -> LDS -> this wave's fragments (while the token rows are in flight)
#pragma unroll
    for (int k = 0; k < 4; ++k) reinterpret_cast<u32x4*>(smem)[tid + 256 * k] = pv[k];
    __syncthreads();
    // B operand of the first contraction: lane (c, h) holds P2[16 kb + 8 h + s][32 q + c], s = 0..7
    half8 p2f[KB], p1own[2], p1oth[2];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) p2f[kb] = lds_column8(P2flat, N, 16 * kb + 8 * h, 4, 32 * q + (c & 16), l & 15);
    // B operand of the second contraction for output tile It, gathered with the K permutation of the accumulator layout
    // that feeds it: K block kk, slot s, half-wave h  <->  i = 32 (kk / 2) + 8 (2 (kk % 2) + s / 4) + 4 h + s % 4.
    // K blocks 2 It + kq meet this wave's own rows of Z, K blocks 2 (1 - It) + kq the partner's.
#pragma unroll
    for (int kq = 0; kq < 2; ++kq) {
        p1own[kq] = lds_column8(P1flat, N, 32 * It + 16 * kq + 4 * h, 8, 32 * It + (c & 16), l & 15);
        p1oth[kq] = lds_column8(P1flat, N, 32 * (1 - It) + 16 * kq + 4 * h, 8, 32 * It + (c & 16), l & 15);
    }
    __builtin_amdgcn_sched_barrier(0);   // the fragment reads are issued before anything waits for the token rows

    const int rd_ofs = (32 * It + c) * (N * 2);
    const int rd_swz = (c >> 1) & 7;
    u32x4* zmine = zbuf + (w * 4) * 64 + l;
    const u32x4* ztheirs = zbuf + ((w ^ 2) * 4) * 64 + l;   // wave (q, 1 - It)
    uint8_t* out_lane = out_codes + (32 * It + c) * (N / 2) + 16 * q + 8 * h;

#pragma unroll
    for (int j = 0; j < NTOK; ++j) {
        const int64_t tok = t0 + j < T ? t0 + j : T - 1;
        const float clipv = clip[clip_mode ? tok : 0];   // wave-uniform address: a scalar load
        unsigned char* tile = tiles + j * TILE_BYTES;
        *reinterpret_cast<u32x4*>(tile + 16 * tid) = pre[j][0];
        *reinterpret_cast<u32x4*>(tile + 16 * (tid + 256)) = pre[j][1];
        __syncthreads();   // (1) the tile is complete; every wave is also done with the fragments' staging area / the last token's parts
        // ---- Z[It, q] = X~[It rows, :] P2[:, slab q]; lane (c, h), K block kb: chunk 2 kb + h of row 32 It + c
        f32x16 acc1, acc2;
#pragma unroll
        for (int r = 0; r < 16; ++r) { acc1[r] = 0.0f; acc2[r] = 0.0f; }
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const half8 a = *reinterpret_cast<const half8*>(tile + rd_ofs + 16 * ((2 * kb + h) ^ rd_swz));
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, p2f[kb], acc1, 0, 0, 0);
        }
        // ---- hi + lo parts of the two K blocks of this row tile: to the partner, and into this wave's own products
        half8 zh[2], zl[2];
#pragma unroll
        for (int kq = 0; kq < 2; ++kq) {
            split_hi_lo(acc1, 8 * kq, zh[kq], zl[kq]);
            zmine[(2 * kq) * 64] = __builtin_bit_cast(u32x4, zh[kq]);
            zmine[(2 * kq + 1) * 64] = __builtin_bit_cast(u32x4, zl[kq]);
            acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(zh[kq], p1own[kq], acc2, 0, 0, 0);
            acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(zl[kq], p1own[kq], acc2, 0, 0, 0);
        }
        __syncthreads();   // (2) parts exchanged
#pragma unroll
        for (int kq = 0; kq < 2; ++kq) {
            const half8 ph = __builtin_bit_cast(half8, ztheirs[(2 * kq) * 64]);
            const half8 pl = __builtin_bit_cast(half8, ztheirs[(2 * kq + 1) * 64]);
            acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(ph, p1oth[kq], acc2, 0, 0, 0);
            acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(pl, p1oth[kq], acc2, 0, 0, 0);
        }
        // ---- per-token absmax: in-lane, over the wave, over the four waves
        float m = 0.0f;
#pragma unroll
        for (int r = 0; r < 16; r += 2) m = __builtin_fmaxf(__builtin_fmaxf(m, __builtin_fabsf(acc2[r])), __builtin_fabsf(acc2[r + 1]));
        m = wave_max(m);
        if (l == 0) red[(j & 1) * 4 + w] = m;
        __syncthreads();   // (3) absmax exchanged
        const float* rj = red + (j & 1) * 4;
        m = __builtin_fmaxf(__builtin_fmaxf(rj[0], rj[1]), __builtin_fmaxf(rj[2], rj[3]));
        // ---- step = alpha * max / 7, rounded to fp16; the rounded step divides
        const _Float16 sh = (_Float16)(clipv * m * 0.142857149f);
        const float s = (float)sh;
        const float inv = (s > 0.0f && s <= 65504.0f) ? __builtin_amdgcn_rcpf(s) : 0.0f;   // 1 ulp: < 1e-6 code units
        const float kmul = inv * (4096.0f / 32767.0f);
        constexpr float kadd = 2047.5f / 32767.0f;
        // ---- round, clamp, pack.  Lane (c, h) holds, of row 32 It + c of X~, the channels 32 q + 8 g + 4 h + k in
        // acc2[4 g + k].  Eight of them (g = 2 m, 2 m + 1) become one dword of nibbles.
        uint32_t W[2];
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
            uint32_t D[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float r0 = __builtin_fmaf(acc2[8 * mm + k], kmul, kadd);
                const float r1 = __builtin_fmaf(acc2[8 * mm + 4 + k], kmul, kadd);
                D[k] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pknorm_i16(r0, r1));
            }
            // bytes 1 and 3 of D[k] carry nibbles k and k + 4 on top: even nibbles -> E, odd ones -> F
            const uint32_t E = __builtin_amdgcn_perm(D[2], D[0], 0x07030501u);
            const uint32_t F = __builtin_amdgcn_perm(D[3], D[1], 0x07030501u);
            W[mm] = (F & 0xF0F0F0F0u) | ((E >> 4) & 0x0F0F0F0Fu);
        }
        // lane pair exchange: afterwards half-wave 0 holds the groups g = 0, 1 of both lanes of the pair and half-wave 1
        // the groups g = 2, 3 (P = half-wave 0's codes, Q = half-wave 1's): 8 consecutive bytes of the row per lane
        const auto sw = __builtin_amdgcn_permlane32_swap(W[0], W[1], false, false);
        const uint32_t Pc = sw[0], Qc = sw[1];
        uint2 o;
        o.x = __builtin_amdgcn_perm(Qc, Pc, 0x05040100u);
        o.y = __builtin_amdgcn_perm(Qc, Pc, 0x07060302u);
        *reinterpret_cast<uint2*>(out_lane + tok * (int64_t)(N * N / 2)) = o;
        if (w == 0) out_scales[tok] = sh;   // every lane writes the same two bytes
    }
}

// ------------------------------------------------------------------------------------
bool tq_quad_applicable(const TqDev& d) {
    if (d.n2 != 64 || d.n1 != 64 || !d.P1 || !d.P2 || !d.vec8 || !d.out_vec16) return false;
    if ((reinterpret_cast<uintptr_t>(d.P1) | reinterpret_cast<uintptr_t>(d.P2)) & 15) return false;
    return d.T >= 1 && d.T <= 0x7fffffff;
}

template <int NTOK>
static hipError_t quad_launch(const TqDev& d, hipStream_t stream) {
    auto fn = &tq_quad_kernel<NTOK>;
    constexpr int lds = (2 + NTOK) * 64 * 64 * 2 + 64;
    static OccCache occ_cache;   // the first call on a device also raises the kernel's LDS limit
    int occ = 0;
    hipError_t e = kernel_occupancy(reinterpret_cast<const void*>(fn), 256, lds, occ_cache, occ);
    if (e != hipSuccess) return e;
    const int64_t grid = (d.T + NTOK - 1) / NTOK;
    (void)hipGetLastError();
    hipLaunchKernelGGL(fn, dim3((unsigned)grid), dim3(256), lds, stream, d.P2, d.P1, d.x, d.x_stride, d.T, d.clip, d.out_codes, d.out_scales, d.clip_mode);
    return hipGetLastError();
}

hipError_t tq_quad_launch(const TqDev& d, hipStream_t stream, int ntok) {
    switch (ntok) {
        case 1: return quad_launch<1>(d, stream);
        case 2: return quad_launch<2>(d, stream);
        case 8: return quad_launch<8>(d, stream);
        default: return quad_launch<4>(d, stream);
    }
}

}  // namespace fq
